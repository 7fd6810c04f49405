// Block-scaled NVFP4 GEMM of libqii:  C = A_hat * B_hat^T  (paper Sec. 5; both operands
// K-contiguous, one E4M3 scale per 16 elements of K, one f32 scale per tensor).
//
// gfx950's scaled FP4 MFMA takes one power-of-two (E8M0) scale per 32 elements, which
// cannot carry NVFP4's E4M3 scale per 16.  The product e2m1 * e4m3 has at most 6
// significant bits and lies in [2^-10, 2688], so it is EXACT in f16: the kernel keeps
// the raw 4.5-bit data in LDS, dequantizes fragments in registers
// (v_cvt_scalef32_pk_f16_fp4 then one packed f16 multiply by the group scale) and feeds
// v_mfma_f32_32x32x16_f16; every product and the f32 accumulation are those of the
// dequantized operands.  The two tensor scales are applied once in the epilogue.
//
// Three kernels share this scheme (launch_gemm picks one): gemm_kernel_v4, the main one
// (K a multiple of 256, scale bytes re-tiled into a workspace, LDS-direct loads, explicit
// software pipeline); gemm_kernel_v2 (K a multiple of 128, no workspace); gemm_kernel (any
// K that is a multiple of 16, NVFP4's own rule; ragged everything).
//
// Tiling: 256 x 256 block tile, K tile 128 or 256, 4 waves (2 x 2) each owning 128 x 128 =
// 4 x 4 MFMA tiles (256 accumulator registers).  One 32x32x16 MFMA consumes exactly
// one scale group per lane: lanes 0..31 supply k 0..31 of a 64-element K slice and
// lanes 32..63 supply k 32..63, four MFMAs walk the four dwords of a lane's 16 bytes
// (the order of k inside the contraction is free as long as A and B agree).
#include "gemm_common.h"
#include "gemm_sharing_map.h"
#include "qii_device.h"
#include "qii_internal.h"

namespace qii {
namespace {

constexpr int BM = 256, BN = 256, BK = 128;
constexpr int kPitch = 80;   // bytes per LDS row of codes: 64 data + 16 pad (bank spread)
constexpr int kSPitch = 8;   // scale bytes per row per K tile
constexpr int kStageBytes = BM * kPitch + BN * kPitch + BM * kSPitch + BN * kSPitch;

struct StagePtr {
    uint8_t *a, *b, *as, *bs;
};
__device__ __forceinline__ StagePtr stage_ptr(uint8_t *smem, int s)
{
    uint8_t *base = smem + s * kStageBytes;
    return StagePtr{base, base + BM * kPitch, base + (BM + BN) * kPitch,
                    base + (BM + BN) * kPitch + BM * kSPitch};
}

// raw global -> register staging of one K tile (per thread: 4+4 code vectors, 1+1 scale vectors)
struct Staged {
    uint4 a[4], b[4];
    uint2 as, bs;
};

// scale bytes of one row for the K tile at k0 (8 groups); groups beyond K read as 0
__device__ __forceinline__ uint2 load_scales(const uint8_t *scales, int64_t row, int64_t nrows,
                                             int64_t K, int64_t k0)
{
    uint2 r = make_uint2(0u, 0u);
    if (row >= nrows) return r;
    const uint8_t *p = scales + row * (K / 16) + k0 / 16;
    uint32_t w[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (k0 + 16 * i < K) w[i >> 2] |= (uint32_t)p[i] << (8 * (i & 3));
    return make_uint2(w[0], w[1]);
}

// A 16-byte piece of a code row holds two scale groups.  K is any multiple of 16 here: when it is
// an odd multiple the last piece of a row is half valid and rows are only 8-byte aligned, so the
// tile is moved in 8-byte halves; everything beyond M, N or K is zero (code 0, scale 0).
__device__ __forceinline__ void load_tile(Staged &st, const uint8_t *a_codes, const uint8_t *a_scales,
                                          const uint8_t *b_codes, const uint8_t *b_scales, int64_t M,
                                          int64_t N, int64_t K, int64_t m0, int64_t n0, int64_t k0)
{
    const int t = threadIdx.x;
    const int seg = t & 3, r = t >> 2;
    const int64_t kbyte = k0 / 2 + 16 * seg;
    const bool lo_ok = k0 + 32 * seg < K, hi_ok = k0 + 32 * seg + 16 < K;
    const uint2 z = make_uint2(0u, 0u);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int64_t ra = m0 + p * 64 + r, rb = n0 + p * 64 + r;
        const uint8_t *pa = a_codes + ra * (K / 2) + kbyte, *pb = b_codes + rb * (K / 2) + kbyte;
        const uint2 al = (lo_ok && ra < M) ? *reinterpret_cast<const uint2 *>(pa) : z;
        const uint2 ah = (hi_ok && ra < M) ? *reinterpret_cast<const uint2 *>(pa + 8) : z;
        const uint2 bl = (lo_ok && rb < N) ? *reinterpret_cast<const uint2 *>(pb) : z;
        const uint2 bh = (hi_ok && rb < N) ? *reinterpret_cast<const uint2 *>(pb + 8) : z;
        st.a[p] = make_uint4(al.x, al.y, ah.x, ah.y);
        st.b[p] = make_uint4(bl.x, bl.y, bh.x, bh.y);
    }
    st.as = load_scales(a_scales, m0 + t, M, K, k0);
    st.bs = load_scales(b_scales, n0 + t, N, K, k0);
}

__device__ __forceinline__ void store_tile(const Staged &st, const StagePtr &sp)
{
    const int t = threadIdx.x;
    const int seg = t & 3, r = t >> 2;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        *reinterpret_cast<uint4 *>(sp.a + (p * 64 + r) * kPitch + 16 * seg) = st.a[p];
        *reinterpret_cast<uint4 *>(sp.b + (p * 64 + r) * kPitch + 16 * seg) = st.b[p];
    }
    *reinterpret_cast<uint2 *>(sp.as + t * kSPitch) = st.as;
    *reinterpret_cast<uint2 *>(sp.bs + t * kSPitch) = st.bs;
}

// 8 FP4 codes (one dword) times one E4M3 scale -> 8 exact f16 values.
// scale16x2 holds the scale byte shifted to f16 position in both halves: as f16 that is
// e4m3 * 2^-8 (subnormals included); the FP4 conversion multiplies by 2^8.
__device__ __forceinline__ half8_t dequant8(uint32_t codes, uint32_t scale16x2)
{
    const half2_t s2 = __builtin_bit_cast(half2_t, scale16x2);
    const half2_t h0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 256.0f, 0) * s2;
    const half2_t h1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 256.0f, 1) * s2;
    const half2_t h2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 256.0f, 2) * s2;
    const half2_t h3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 256.0f, 3) * s2;
    half8_t r;
    r[0] = h0[0]; r[1] = h0[1]; r[2] = h1[0]; r[3] = h1[1];
    r[4] = h2[0]; r[5] = h2[1]; r[6] = h3[0]; r[7] = h3[1];
    return r;
}

__device__ __forceinline__ uint32_t scale_pair(uint32_t two_bytes, int which)
{
    const uint32_t b = (two_bytes >> (8 * which)) & 0xFFu;
    return (b << 7) | (b << 23);
}

template <bool kBf16Out>
__global__ __launch_bounds__(256, 1) void gemm_kernel(const uint8_t *__restrict__ a_codes,
                                                      const uint8_t *__restrict__ a_scales,
                                                      const float *__restrict__ a_ts,
                                                      const uint8_t *__restrict__ b_codes,
                                                      const uint8_t *__restrict__ b_scales,
                                                      const float *__restrict__ b_ts, int64_t M,
                                                      int64_t N, int64_t K, void *__restrict__ Cout,
                                                      int64_t ldc, int tiles_n, uint32_t *amax_out)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int tile = blockIdx.x;
    const int64_t m0 = (int64_t)(tile / tiles_n) * BM, n0 = (int64_t)(tile % tiles_n) * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, kb = lane >> 5;

    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int64_t ktiles = (K + BK - 1) / BK;
    Staged st;
    load_tile(st, a_codes, a_scales, b_codes, b_scales, M, N, K, m0, n0, 0);
    store_tile(st, stage_ptr(smem, 0));
    __syncthreads();

    for (int64_t kt = 0; kt < ktiles; ++kt) {
        const StagePtr sp = stage_ptr(smem, (int)(kt & 1));
        if (kt + 1 < ktiles)
            load_tile(st, a_codes, a_scales, b_codes, b_scales, M, N, K, m0, n0, (kt + 1) * BK);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            uint4 ra[4], rb[4];
            uint32_t sa[4], sb[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int rowa = wm * 128 + t * 32 + li, rowb = wn * 128 + t * 32 + li;
                ra[t] = *reinterpret_cast<const uint4 *>(sp.a + rowa * kPitch + 32 * j + 16 * kb);
                rb[t] = *reinterpret_cast<const uint4 *>(sp.b + rowb * kPitch + 32 * j + 16 * kb);
                sa[t] = *reinterpret_cast<const uint16_t *>(sp.as + rowa * kSPitch + 4 * j + 2 * kb);
                sb[t] = *reinterpret_cast<const uint16_t *>(sp.bs + rowb * kSPitch + 4 * j + 2 * kb);
            }
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                half8_t fa[4], fb[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const uint32_t wa = d == 0 ? ra[t].x : d == 1 ? ra[t].y : d == 2 ? ra[t].z : ra[t].w;
                    const uint32_t wb = d == 0 ? rb[t].x : d == 1 ? rb[t].y : d == 2 ? rb[t].z : rb[t].w;
                    fa[t] = dequant8(wa, scale_pair(sa[t], d >> 1));
                    fb[t] = dequant8(wb, scale_pair(sb[t], d >> 1));
                }
#pragma unroll
                for (int ti = 0; ti < 4; ++ti)
#pragma unroll
                    for (int tj = 0; tj < 4; ++tj)
                        acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[ti], fb[tj], acc[ti][tj], 0, 0, 0);
            }
        }
        if (kt + 1 < ktiles) {
            store_tile(st, stage_ptr(smem, (int)((kt + 1) & 1)));
            __syncthreads();
        }
    }

    // epilogue: C = acc * (x32_A * x32_B).  acc[r] of a 32x32 tile is row
    // 8*(r/4) + 4*(lane/32) + r%4, column lane%32.
    const float ts = (*a_ts) * (*b_ts);
    float cmax = 0.0f;   // max |C| as stored, over this lane's entries inside the matrix
#pragma unroll
    for (int ti = 0; ti < 4; ++ti)
#pragma unroll
        for (int tj = 0; tj < 4; ++tj) {
            const int64_t col = n0 + wn * 128 + tj * 32 + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wm * 128 + ti * 32 + 8 * (r >> 2) + 4 * kb + (r & 3);
                if (row < M && col < N) {
                    const float v = acc[ti][tj][r] * ts;
                    if (kBf16Out) {
                        const uint32_t bits = f32_to_bf16_bits(v);
                        reinterpret_cast<uint16_t *>(Cout)[row * ldc + col] = (uint16_t)bits;
                        cmax = fmaxf(cmax, fabsf(u2f(bits << 16)));
                    } else {
                        reinterpret_cast<float *>(Cout)[row * ldc + col] = v;
                        cmax = fmaxf(cmax, fabsf(v));
                    }
                }
            }
        }
    emit_tile_max(cmax, amax_out);
}


// ------------------------------------------------------------------------------------------
// Main kernel (K a multiple of 128).  Differences from gemm_kernel above:
//  * global -> LDS with global_load_lds (no staging registers, no VALU, no ds_write): each
//    lane fetches one 16-byte piece of a code row (or one dword of scale bytes) and the wave's
//    64 pieces land contiguously in LDS.  The piece a lane fetches is chosen so that the LDS
//    image is XOR-swizzled: row r keeps its 16-byte segment s in slot 4r + (s ^ ((r>>1)&3)),
//    which makes the 128-bit fragment reads of 8 consecutive rows hit 8 different bank groups.
//  * three LDS stages: tile kt+2 streams in while tile kt is multiplied, and the raw
//    fragments of the next 64-wide K slice (also across the tile boundary) are read from LDS
//    one slice ahead, so no LDS latency sits between barriers and matrix instructions.
//  * epilogue through LDS: accumulators are scaled, converted and written to a per-wave
//    LDS tile, then stored as 16-byte pieces of full rows.
constexpr int kStages = 3;
constexpr int kOffA = 0, kOffB = 16384, kOffAs = 32768, kOffBs = 34816, kStage2Bytes = 36864;
constexpr int kSmem2 = kStages * kStage2Bytes;   // 108 KiB, also reused by the epilogue

struct RawFrag {
    uint4 a[4], b[4];
    uint32_t sa[4], sb[4];
};

__device__ __forceinline__ void issue_tile_loads(uint8_t *stage, const uint8_t *a_codes, const uint8_t *a_scales,
                                                 const uint8_t *b_codes, const uint8_t *b_scales, int64_t M,
                                                 int64_t N, int64_t K, int64_t m0, int64_t n0, int64_t k0,
                                                 int wave)
{
    const int t = threadIdx.x;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int row = p * 64 + (t >> 2);
        const int seg = (t & 3) ^ ((row >> 1) & 3);
        int64_t ra = m0 + row, rb = n0 + row;
        ra = ra < M ? ra : M - 1;   // rows beyond the matrix read a valid row; their results are dropped
        rb = rb < N ? rb : N - 1;
        __builtin_amdgcn_global_load_lds(a_codes + ra * (K / 2) + k0 / 2 + 16 * seg,
                                         (__attribute__((address_space(3))) void *)(stage + kOffA + (p * 256 + wave * 64) * 16), 16, 0, 0);
        __builtin_amdgcn_global_load_lds(b_codes + rb * (K / 2) + k0 / 2 + 16 * seg,
                                         (__attribute__((address_space(3))) void *)(stage + kOffB + (p * 256 + wave * 64) * 16), 16, 0, 0);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int row = (h * 256 + t) >> 1, half = t & 1;
        int64_t ra = m0 + row, rb = n0 + row;
        ra = ra < M ? ra : M - 1;
        rb = rb < N ? rb : N - 1;
        __builtin_amdgcn_global_load_lds(a_scales + ra * (K / 16) + k0 / 16 + 4 * half,
                                         (__attribute__((address_space(3))) void *)(stage + kOffAs + (h * 256 + wave * 64) * 4), 4, 0, 0);
        __builtin_amdgcn_global_load_lds(b_scales + rb * (K / 16) + k0 / 16 + 4 * half,
                                         (__attribute__((address_space(3))) void *)(stage + kOffBs + (h * 256 + wave * 64) * 4), 4, 0, 0);
    }
}

// raw fragments of K slice j (64 elements) of one stage for this lane
__device__ __forceinline__ void read_raw(RawFrag &f, const uint8_t *stage, int j, int wm, int wn, int li, int kb)
{
    const int seg = 2 * j + kb;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int rowa = wm * 128 + t * 32 + li, rowb = wn * 128 + t * 32 + li;
        f.a[t] = *reinterpret_cast<const uint4 *>(stage + kOffA + (rowa * 4 + (seg ^ ((rowa >> 1) & 3))) * 16);
        f.b[t] = *reinterpret_cast<const uint4 *>(stage + kOffB + (rowb * 4 + (seg ^ ((rowb >> 1) & 3))) * 16);
        f.sa[t] = *reinterpret_cast<const uint16_t *>(stage + kOffAs + rowa * 8 + 4 * j + 2 * kb);
        f.sb[t] = *reinterpret_cast<const uint16_t *>(stage + kOffBs + rowb * 8 + 4 * j + 2 * kb);
    }
}

// 64 elements of K for the wave's 4 x 4 MFMA tiles: 4 steps of 16 MFMAs, each step
// dequantizing one dword (8 codes) per fragment
__device__ __forceinline__ void mma_slice(floatx16 (&acc)[4][4], const RawFrag &f)
{
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        half8_t fa[4], fb[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const uint32_t wa = d == 0 ? f.a[t].x : d == 1 ? f.a[t].y : d == 2 ? f.a[t].z : f.a[t].w;
            const uint32_t wb = d == 0 ? f.b[t].x : d == 1 ? f.b[t].y : d == 2 ? f.b[t].z : f.b[t].w;
            fa[t] = dequant8(wa, scale_pair(f.sa[t], d >> 1));
            fb[t] = dequant8(wb, scale_pair(f.sb[t], d >> 1));
        }
#pragma unroll
        for (int ti = 0; ti < 4; ++ti)
#pragma unroll
            for (int tj = 0; tj < 4; ++tj)
                acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[ti], fb[tj], acc[ti][tj], 0, 0, 0);
    }
}

template <bool kBf16Out>
__global__ __launch_bounds__(256, 1) void gemm_kernel_v2(const uint8_t *__restrict__ a_codes,
                                                         const uint8_t *__restrict__ a_scales,
                                                         const float *__restrict__ a_ts,
                                                         const uint8_t *__restrict__ b_codes,
                                                         const uint8_t *__restrict__ b_scales,
                                                         const float *__restrict__ b_ts, int64_t M,
                                                         int64_t N, int64_t K, void *__restrict__ Cout,
                                                         int64_t ldc, int tiles_m, int tiles_n, uint32_t *amax_out)
{
    extern __shared__ __align__(16) uint8_t smem[];
    // XCD-aware order: consecutive block ids land on different XCDs (8 of them, each with its
    // own L2), so give every XCD a contiguous run of tiles, walked row-major over (m, n).
    int tile = blockIdx.x;
    const int ntiles = tiles_m * tiles_n;
    if ((ntiles & 7) == 0) tile = (tile & 7) * (ntiles >> 3) + (tile >> 3);
    const int64_t m0 = (int64_t)(tile / tiles_n) * BM, n0 = (int64_t)(tile % tiles_n) * BN;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, kb = lane >> 5;

    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int ktiles = (int)(K / BK);
    issue_tile_loads(smem, a_codes, a_scales, b_codes, b_scales, M, N, K, m0, n0, 0, wave);
    if (ktiles > 1)
        issue_tile_loads(smem + kStage2Bytes, a_codes, a_scales, b_codes, b_scales, M, N, K, m0, n0, BK, wave);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // the raw fragments ping-pong between two register sets: f0 holds K slice 0 of a tile,
    // f1 slice 1; each is refilled from LDS while the other is being multiplied
    RawFrag f0, f1;
    read_raw(f0, smem, 0, wm, wn, li, kb);
    int st_cur = 0;   // stage of tile kt
    for (int kt = 0; kt < ktiles; ++kt) {
        const int st_next = st_cur == kStages - 1 ? 0 : st_cur + 1;
        const int st_load = st_next == kStages - 1 ? 0 : st_next + 1;
        if (kt + 2 < ktiles)
            issue_tile_loads(smem + st_load * kStage2Bytes, a_codes, a_scales, b_codes, b_scales, M, N, K, m0,
                             n0, (int64_t)(kt + 2) * BK, wave);
        read_raw(f1, smem + st_cur * kStage2Bytes, 1, wm, wn, li, kb);
        mma_slice(acc, f0);
        // (after the last tile this reads a stale stage; the values are never used)
        read_raw(f0, smem + st_next * kStage2Bytes, 0, wm, wn, li, kb);
        mma_slice(acc, f1);
        // tile kt+2 (issued a whole tile ago) must have landed before anyone reads it, and
        // everyone must be done with stage st_cur before tile kt+3 overwrites it
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        st_cur = st_next;
    }

    store_tile_through_lds<kBf16Out>(acc, smem, (*a_ts) * (*b_ts), Cout, ldc, M, N, m0, n0, wave, wm, wn, lane, li, kb, amax_out);
}


// ------------------------------------------------------------------------------------------
// Main kernel (K a multiple of 256, scale bytes re-tiled into the workspace).
// The operand fetch is what bounds this GEMM once the matrix pipe is fed: with 128-wide K
// tiles every row contributes half a 128-byte line of codes and 8 bytes of a scale line per
// tile, i.e. five times more L2 line requests than useful bytes.  Here a K tile is 256 wide
// (one full line of codes per row) and the scale bytes come from a copy laid out as
// [row tile of 256][K tile of 256][row][16 bytes], so each block reads 4 KiB of contiguous
// scales per operand and tile.  Two LDS stages of 72 KiB; LDS image of the codes: row r keeps
// its 16-byte segment s in slot 8r + (s ^ (r & 7)) (conflict-free 128-bit fragment reads).
constexpr int BK4 = 256;
constexpr int kOff4A = 0, kOff4B = 32768, kOff4As = 65536, kOff4Bs = 69632, kStage4Bytes = 73728;
constexpr int kSmem4 = 2 * kStage4Bytes;   // 144 KiB

// scales[rows][K/16] -> tiled[(rt * (K/256) + ks) * 256 + r][16], one 16-byte piece per thread;
// both operands in one launch (threads [0, na) take A, [na, na + nb) take B).  Rows of the last
// row tile beyond M (or N) are not written and keep whatever the workspace held: they only ever
// scale operand rows beyond the matrix, whose products land in accumulator rows / columns that
// the epilogue never stores (matrix-instruction rows are independent of one another).
__global__ void retile_scales_kernel(const uint8_t *__restrict__ a_scales, uint8_t *__restrict__ a_tiled,
                                     int64_t M, const uint8_t *__restrict__ b_scales,
                                     uint8_t *__restrict__ b_tiled, int64_t N, int64_t K)
{
    const int64_t ksn = K / 256;
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // (row, ks)
    const uint8_t *scales = a_scales;
    uint8_t *tiled = a_tiled;
    if (idx >= M * ksn) {
        idx -= M * ksn;
        if (idx >= N * ksn) return;
        scales = b_scales;
        tiled = b_tiled;
    }
    const int64_t row = idx / ksn, ks = idx % ksn;
    const uint4 v = *reinterpret_cast<const uint4 *>(scales + row * (K / 16) + ks * 16);
    *reinterpret_cast<uint4 *>(tiled + (((row >> 8) * ksn + ks) * 256 + (row & 255)) * 16) = v;
}

__device__ __forceinline__ void issue_tile_loads4(uint8_t *stage, const uint8_t *a_codes, const uint8_t *a_tiled,
                                                  const uint8_t *b_codes, const uint8_t *b_tiled, int64_t M,
                                                  int64_t N, int64_t K, int64_t m0, int64_t n0, int64_t kt,
                                                  int wave)
{
    const int t = threadIdx.x;
    const int64_t kbyte = kt * (BK4 / 2);
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int row = p * 32 + (t >> 3);
        const int seg = (t & 7) ^ (row & 7);
        int64_t ra = m0 + row, rb = n0 + row;
        ra = ra < M ? ra : M - 1;   // rows beyond the matrix read a valid row; their results are dropped
        rb = rb < N ? rb : N - 1;
        __builtin_amdgcn_global_load_lds(a_codes + ra * (K / 2) + kbyte + 16 * seg,
                                         (__attribute__((address_space(3))) void *)(stage + kOff4A + (p * 256 + wave * 64) * 16), 16, 0, 0);
        __builtin_amdgcn_global_load_lds(b_codes + rb * (K / 2) + kbyte + 16 * seg,
                                         (__attribute__((address_space(3))) void *)(stage + kOff4B + (p * 256 + wave * 64) * 16), 16, 0, 0);
    }
    const int64_t ksn = K / BK4;
    __builtin_amdgcn_global_load_lds(a_tiled + (((m0 >> 8) * ksn + kt) * 256 + t) * 16,
                                     (__attribute__((address_space(3))) void *)(stage + kOff4As + (wave * 64) * 16), 16, 0, 0);
    __builtin_amdgcn_global_load_lds(b_tiled + (((n0 >> 8) * ksn + kt) * 256 + t) * 16,
                                     (__attribute__((address_space(3))) void *)(stage + kOff4Bs + (wave * 64) * 16), 16, 0, 0);
}

// ---- fragment pipeline of the main kernel -------------------------------------------------
// The compiler makes every LDS read that follows a global_load_lds wait for that load
// (it cannot tell the two LDS regions apart), which would serialise the fetch of the next
// K tile with the multiplication of the current one.  The fragment reads are therefore
// written as inline assembly, with their own wait: a read block only names its
// destination registers, and the matching wait "produces" them for the code that follows.
struct RawFrag4 {
    u32x4 a[4], b[4];       // 32 codes (16 bytes) of K for 4 row blocks of A and of B
    uint32_t sa[4], sb[4];  // their two scale bytes
};

struct FragAddr {
    uint32_t a, b, sa, sb;  // LDS byte addresses of this lane's row 0 pieces in stage 0
    uint32_t xo[4];         // swizzled 16-byte slot of K slice j, times 16
};

template <int J>
__device__ __forceinline__ void frag_read_issue(RawFrag4 &f, const FragAddr &fa, uint32_t stage_off)
{
    const uint32_t va = fa.a + fa.xo[J] + stage_off, vb = fa.b + fa.xo[J] + stage_off;
    const uint32_t vsa = fa.sa + stage_off, vsb = fa.sb + stage_off;
    // rows 32 t: codes 32 * 128 bytes apart, re-tiled scales 32 * 16 bytes apart
#define QII_RD(T)                                                                                       \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.a[T]) : "v"(va), "n"(T * 4096));              \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.b[T]) : "v"(vb), "n"(T * 4096));              \
    asm volatile("ds_read_u16 %0, %1 offset:%2" : "=v"(f.sa[T]) : "v"(vsa), "n"(T * 512 + 4 * J));      \
    asm volatile("ds_read_u16 %0, %1 offset:%2" : "=v"(f.sb[T]) : "v"(vsb), "n"(T * 512 + 4 * J))
    QII_RD(0); QII_RD(1); QII_RD(2); QII_RD(3);
#undef QII_RD
}

// all outstanding LDS reads have landed; ties the registers of f to the wait
__device__ __forceinline__ void frag_read_wait(RawFrag4 &f)
{
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.a[2]), "+v"(f.a[3]), "+v"(f.b[0]), "+v"(f.b[1]),
                   "+v"(f.b[2]), "+v"(f.b[3]), "+v"(f.sa[0]), "+v"(f.sa[1]), "+v"(f.sa[2]), "+v"(f.sa[3]),
                   "+v"(f.sb[0]), "+v"(f.sb[1]), "+v"(f.sb[2]), "+v"(f.sb[3]));
}

// The two scale bytes of a lane's 32 elements of K, as two f16 numbers in one register: byte b in
// f16 position (b << 7) is e4m3 * 2^-8, subnormals included.  v_perm_b32 spreads the bytes to the
// two halves, one shift moves them to f16 position.
__device__ __forceinline__ uint32_t scale_halves(uint32_t two_bytes)
{
    return __builtin_amdgcn_perm(0u, two_bytes, 0x0C010C00u) << 7;
}

// half of one fragment (4 of its 8 values): two conversions and two packed multiplies by the f16
// scale in the low (kHi = 0) or high half of `scales`, taken for both lanes of the packed multiply
// through the instruction's operand selectors
template <int H, int kHi>
__device__ __forceinline__ void dequant_half(half8_t &dst, uint32_t codes, uint32_t scales)
{
    const half2_t c0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 256.0f, 2 * H);
    const half2_t c1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, 256.0f, 2 * H + 1);
    half2_t h0, h1;
    if (kHi) {
        asm("v_pk_mul_f16 %0, %1, %2 op_sel:[0,1] op_sel_hi:[1,1]" : "=v"(h0) : "v"(c0), "v"(scales));
        asm("v_pk_mul_f16 %0, %1, %2 op_sel:[0,1] op_sel_hi:[1,1]" : "=v"(h1) : "v"(c1), "v"(scales));
    } else {
        asm("v_pk_mul_f16 %0, %1, %2 op_sel_hi:[1,0]" : "=v"(h0) : "v"(c0), "v"(scales));
        asm("v_pk_mul_f16 %0, %1, %2 op_sel_hi:[1,0]" : "=v"(h1) : "v"(c1), "v"(scales));
    }
    dst[4 * H] = h0[0]; dst[4 * H + 1] = h0[1]; dst[4 * H + 2] = h1[0]; dst[4 * H + 3] = h1[1];
}

struct Frags {
    half8_t a[4], b[4];
};

// chunk I (0..15) of the dequantization of dword D of raw fragments f into nx: fragment I/2
// (0..3 = A, 4..7 = B), half I%2.  The first chunk that touches a fragment of a freshly read
// slice (dword 0, half 0) first turns its two scale bytes into the two-f16 form, in place.
template <int I, int D>
__device__ __forceinline__ void dequant_chunk(Frags &nx, RawFrag4 &f)
{
    constexpr int t = (I >> 1) & 3, h = I & 1;
    if (I < 8) {
        if (D == 0 && h == 0) f.sa[t] = scale_halves(f.sa[t]);
        dequant_half<h, (D >> 1)>(nx.a[t], f.a[t][D], f.sa[t]);
    } else {
        if (D == 0 && h == 0) f.sb[t] = scale_halves(f.sb[t]);
        dequant_half<h, (D >> 1)>(nx.b[t], f.b[t][D], f.sb[t]);
    }
}

// One step = 16 matrix instructions on the fragments in cu, with the fragments of the next
// step (dword D of f) dequantized into nx in between, one chunk per matrix instruction; the
// scheduling barriers keep that order, so the conversions run in the shadow of the matrix pipe.
template <int D>
__device__ __forceinline__ void mma_step(floatx16 (&acc)[4][4], const Frags &cu, Frags &nx, RawFrag4 &f)
{
#define QII_MMA(I)                                                                                          \
    acc[(I) >> 2][(I) & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(cu.a[(I) >> 2], cu.b[(I) & 3],          \
                                                                    acc[(I) >> 2][(I) & 3], 0, 0, 0);       \
    dequant_chunk<I, D>(nx, f);                                                                             \
    __builtin_amdgcn_sched_barrier(0)
    QII_MMA(0); QII_MMA(1); QII_MMA(2); QII_MMA(3); QII_MMA(4); QII_MMA(5); QII_MMA(6); QII_MMA(7);
    QII_MMA(8); QII_MMA(9); QII_MMA(10); QII_MMA(11); QII_MMA(12); QII_MMA(13); QII_MMA(14); QII_MMA(15);
#undef QII_MMA
}

// Launch position -> origin of the output tile.  XCD-aware order: consecutive block ids land on
// different XCDs (8 of them, each with its own L2), so every XCD gets a contiguous run of tiles;
// within the run, tiles are walked in groups of 4 tile rows, column by column, so that the ~32
// tiles an XCD works on at once share 4 A panels and 8 B panels (about 3.5 MiB at K = 2048)
// instead of 1 + 32.
__device__ __forceinline__ void tile_origin(int pos, int tiles_m, int tiles_n, int64_t &m0, int64_t &n0)
{
    int tile = pos;
    const int ntiles = tiles_m * tiles_n;
    if ((ntiles & 7) == 0) tile = (tile & 7) * (ntiles >> 3) + (tile >> 3);
    constexpr int kGroupM = 4;
    const int width = kGroupM * tiles_n, first_m = (tile / width) * kGroupM;
    const int gm = tiles_m - first_m < kGroupM ? tiles_m - first_m : kGroupM;
    m0 = (int64_t)(first_m + (tile % width) % gm) * BM;
    n0 = (int64_t)((tile % width) / gm) * BN;
}

// kStream = false: one block per output tile (launch position blockIdx.x).
// kStream = true: the K tiles of the `sk_rem` tiles from position `sk_base` on form one sequence of
// units (tile-major) that the gridDim.x blocks cut into equal contiguous ranges; a block runs its
// range tile segment by tile segment (at most two when a range is shorter than a tile's K) and
// leaves each segment's unscaled f32 partial tile in slot (block + tile number) of `partial`,
// which streamk_fixup_kernel adds up in a fixed order.  (A separate instantiation: the plain
// kernel keeps its registers.)
template <bool kBf16Out, bool kStream>
__global__ __launch_bounds__(256, 1) void gemm_kernel_v4(const uint8_t *__restrict__ a_codes,
                                                         const uint8_t *__restrict__ a_tiled,
                                                         const float *__restrict__ a_ts,
                                                         const uint8_t *__restrict__ b_codes,
                                                         const uint8_t *__restrict__ b_tiled,
                                                         const float *__restrict__ b_ts, int64_t M,
                                                         int64_t N, int64_t K, void *__restrict__ Cout,
                                                         int64_t ldc, int tiles_m, int tiles_n, uint32_t *amax_out,
                                                         int sk_base, int sk_rem, float *__restrict__ partial)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, kb = lane >> 5;

    const int ktotal = (int)(K / BK4);
    // this block's range of units [u, u_end) and its number among the blocks (kStream)
    int64_t u = 0, u_end = 0;
    int blk = 0;
    if (kStream) {
        const int G = (int)gridDim.x;
        blk = sharing_block_number((int)blockIdx.x, G);
        sharing_block_units((int64_t)sk_rem * ktotal, G, blk, u, u_end);
    }
    for (;;) {
    // this segment: K tiles [kt0, kt0 + ktiles) of the tile at launch position pos
    int pos = (int)blockIdx.x, kt0 = 0, ktiles = ktotal, lt = 0;
    if (kStream) {
        sharing_segment(u, u_end, ktotal, lt, kt0, ktiles);
        pos = sharing_position(lt, sk_rem, sk_base);
    }
    int64_t m0, n0;
    tile_origin(pos, tiles_m, tiles_n, m0, n0);

    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    FragAddr fa;
    {
        const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
        fa.a = lds0 + kOff4A + (wm * 128 + li) * 128;
        fa.b = lds0 + kOff4B + (wn * 128 + li) * 128;
        fa.sa = lds0 + kOff4As + (wm * 128 + li) * 16 + 2 * kb;
        fa.sb = lds0 + kOff4Bs + (wn * 128 + li) * 16 + 2 * kb;
#pragma unroll
        for (int j = 0; j < 4; ++j) fa.xo[j] = (uint32_t)(((2 * j + kb) ^ (li & 7)) * 16);
    }

    issue_tile_loads4(smem, a_codes, a_tiled, b_codes, b_tiled, M, N, K, m0, n0, kt0, wave);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (ktiles > 1)
        issue_tile_loads4(smem + kStage4Bytes, a_codes, a_tiled, b_codes, b_tiled, M, N, K, m0, n0, kt0 + 1, wave);

    // Pipeline over K, in steps of 16 columns of K per lane half (4 steps = one 64-wide slice,
    // 4 slices = one tile).  While step n multiplies, the fragments of step n+1 are dequantized;
    // the raw fragments of slice g live in fe (g even) or fo (g odd) and are re-filled with
    // slice g+2 at the start of step (g, 3), once the last conversion of slice g is done, a
    // full slice ahead of their first use.  The hand-over between the two LDS stages sits at
    // step (2, 3) of a tile: this wave's last read of the current stage (slice 3) has landed,
    // so after the barrier tile kt+1, issued a whole tile earlier, is complete in the other
    // stage and the current stage can take tile kt+2.
    RawFrag4 fe, fo;
    Frags x, y;
    frag_read_issue<0>(fe, fa, 0);
    frag_read_issue<1>(fo, fa, 0);
    frag_read_wait(fe);   // (waits for both)
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        fe.sa[t] = scale_halves(fe.sa[t]);
        fe.sb[t] = scale_halves(fe.sb[t]);
        dequant_half<0, 0>(x.a[t], fe.a[t][0], fe.sa[t]);
        dequant_half<1, 0>(x.a[t], fe.a[t][0], fe.sa[t]);
        dequant_half<0, 0>(x.b[t], fe.b[t][0], fe.sb[t]);
        dequant_half<1, 0>(x.b[t], fe.b[t][0], fe.sb[t]);
    }
    for (int kt = 0; kt < ktiles; ++kt) {
        const uint32_t cur_off = (kt & 1) * kStage4Bytes, nxt_off = ((kt + 1) & 1) * kStage4Bytes;
        // slice 0 (raw: fe)
        mma_step<1>(acc, x, y, fe);
        mma_step<2>(acc, y, x, fe);
        mma_step<3>(acc, x, y, fe);
        frag_read_wait(fo);
        frag_read_issue<2>(fe, fa, cur_off);
        mma_step<0>(acc, y, x, fo);
        // slice 1 (raw: fo)
        mma_step<1>(acc, x, y, fo);
        mma_step<2>(acc, y, x, fo);
        mma_step<3>(acc, x, y, fo);
        frag_read_wait(fe);
        frag_read_issue<3>(fo, fa, cur_off);
        mma_step<0>(acc, y, x, fe);
        // slice 2 (raw: fe)
        mma_step<1>(acc, x, y, fe);
        mma_step<2>(acc, y, x, fe);
        mma_step<3>(acc, x, y, fe);
        frag_read_wait(fo);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (kt + 2 < ktiles)
            issue_tile_loads4(smem + cur_off, a_codes, a_tiled, b_codes, b_tiled, M, N, K, m0, n0, kt0 + kt + 2, wave);
        // (after the last tile the two reads below fetch a stale stage; the values are never used)
        frag_read_issue<0>(fe, fa, nxt_off);
        mma_step<0>(acc, y, x, fo);
        // slice 3 (raw: fo)
        mma_step<1>(acc, x, y, fo);
        mma_step<2>(acc, y, x, fo);
        mma_step<3>(acc, x, y, fo);
        frag_read_wait(fe);
        frag_read_issue<1>(fo, fa, nxt_off);
        mma_step<0>(acc, y, x, fe);
    }
    // the last read block is still in flight: its registers and the stages are reused below
    frag_read_wait(fo);
    __syncthreads();
    if (!kStream) {
        store_tile_through_lds<kBf16Out>(acc, smem, (*a_ts) * (*b_ts), Cout, ldc, M, N, m0, n0, wave, wm, wn, lane, li, kb, amax_out);
        break;
    }
    store_tile_through_lds<false, false>(acc, smem, 1.0f, partial + (int64_t)sharing_slot(blk, lt) * (BM * BN), BN, BM, BN, 0, 0, wave, wm, wn, lane,
                                  li, kb, nullptr);
    u += ktiles;
    if (u >= u_end) break;
    __syncthreads();   // every wave is done with its staging tile before the next segment's loads land in LDS
    }
}

// C = (x32_A * x32_B) * sum of a shared tile's partial tiles, in the order of their K ranges.  One
// block per 16 rows of a tile, 4 consecutive columns per thread and pass; the blocks that took part
// in tile lt are those whose unit ranges meet [lt * ktotal, (lt + 1) * ktotal), their slots
// (block + lt) are consecutive.  One atomic per block when max |C| is wanted.
template <bool kBf16Out>
__global__ __launch_bounds__(256) void streamk_fixup_kernel(const float *__restrict__ partial, int sk_base, int sk_rem, int G,
                                                            int ktotal, int tiles_m, int tiles_n, int64_t M, int64_t N,
                                                            const float *__restrict__ a_ts, const float *__restrict__ b_ts,
                                                            void *__restrict__ Cout, int64_t ldc, uint32_t *amax_out)
{
    __shared__ float wave_m[4];
    const int lt = (int)(blockIdx.x >> 4), strip = (int)(blockIdx.x & 15);
    const int64_t U = (int64_t)sk_rem * ktotal;
    const int64_t ufirst = (int64_t)lt * ktotal, ulast = ufirst + ktotal - 1;
    const int b_first = sharing_block_of_unit(ufirst, U, G), b_last = sharing_block_of_unit(ulast, U, G);
    int64_t m0, n0;
    tile_origin(sharing_position(lt, sk_rem, sk_base), tiles_m, tiles_n, m0, n0);
    const float ts = (*a_ts) * (*b_ts);
    float cmax = 0.0f;
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int row = strip * 16 + pass * 4 + (int)(threadIdx.x >> 6), col = (int)(threadIdx.x & 63) * 4;
        const float *src = partial + (int64_t)sharing_slot(b_first, lt) * (BM * BN) + row * BN + col;
        float4 acc = *reinterpret_cast<const float4 *>(src);
        for (int b = b_first + 1; b <= b_last; ++b) {
            src += BM * BN;
            const float4 p = *reinterpret_cast<const float4 *>(src);
            acc.x += p.x; acc.y += p.y; acc.z += p.z; acc.w += p.w;
        }
        const int64_t grow = m0 + row, gcol = n0 + col;
        if (grow >= M) continue;
        const float v[4] = {acc.x * ts, acc.y * ts, acc.z * ts, acc.w * ts};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (gcol + e < N) {
                if (kBf16Out) {
                    const uint32_t b = f32_to_bf16_bits(v[e]);
                    reinterpret_cast<uint16_t *>(Cout)[grow * ldc + gcol + e] = (uint16_t)b;
                    cmax = fmaxf(cmax, fabsf(u2f(b << 16)));
                } else {
                    reinterpret_cast<float *>(Cout)[grow * ldc + gcol + e] = v[e];
                    cmax = fmaxf(cmax, fabsf(v[e]));
                }
            }
    }
    if (amax_out) {   // uniform
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) cmax = fmaxf(cmax, __shfl_xor(cmax, off));
        if ((threadIdx.x & 63) == 0) wave_m[threadIdx.x >> 6] = cmax;
        __syncthreads();
        if (threadIdx.x == 0) atomicMax(amax_out, f2u(fmaxf(fmaxf(wave_m[0], wave_m[1]), fmaxf(wave_m[2], wave_m[3]))));
    }
}

}  // namespace

// The grid of the main kernel runs in rounds of 256 tiles (one block per compute unit).  A last round
// with few tiles leaves most units idle for a whole tile's time (2048 x 2048 x 32768, the weight
// gradient of a small layer, is 64 tiles; 2048 x 11264 is 352: the second round runs at 37 %).  Then
// the full rounds run as they are and the remaining tiles are shared: their K tiles form one sequence
// of units that `grid` blocks (at most 256, at least 4 units each) cut into equal ranges, partial
// tiles go to the workspace and a second kernel adds them up.
//
// The plan follows a cost model fitted to kernel traces (microseconds): a K tile takes 5.8 when all
// 256 units work and 4.6 when at most 176 do (the part is power-limited: fewer active units run at
// a higher clock, so filling idle units gains less than their number suggests); a tile costs 5 more
// for its first loads and its stores; a sharing block 26 more (all blocks store their 256 KiB
// partial tiles at the same moment), 38 when its range spans two tiles; the second kernel 0.05 per
// partial tile (they are stored with plain stores, not streaming ones, and mostly still in cache).  Sharing is used where the model promises at least 7 %.  Measured on one
// box, plain -> shared: 2048 x 2048 x 32768 600 -> 226, 3072 x 3072 x 16384 307 -> 267, 11264 x 2048 x
// 16384 654 -> 573; 6144 x 2048 x 32768 would go 655 -> 618 for 112 MiB of partial tiles and 2048 x
// 5632 x 16384 298 -> 320: both stay plain.
struct StreamPlan {
    int full;   // launch positions run one block per tile
    int rem;    // positions after them whose tiles are shared (0: none)
    int grid;   // blocks that share them
};

static StreamPlan stream_plan(int64_t M, int64_t N, int64_t K)
{
    const int64_t tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN), ktiles = K / BK4;
    StreamPlan plan{(int)tiles, 0, 0};
    if (K % BK4 != 0 || tiles == 0 || tiles > (1 << 24) || ktiles < 8) return plan;
    const int64_t rounds = tiles / 256, rem = tiles % 256;
    if (rem == 0) return plan;
    const int64_t units = rem * ktiles;
    int64_t grid = units / 4 < 256 ? units / 4 : 256;
    if (grid >= 8) grid &= ~(int64_t)7;
    if (grid <= rem) return plan;
    const double full_us = (double)rounds * (5.8 * (double)ktiles + 5.0);
    const double kt_us = 4.6 + (rem > 176 ? 1.2 * (double)(rem - 176) / 80.0 : 0.0);
    const double plain_us = full_us + kt_us * (double)ktiles + 5.0;
    const int64_t per = (units + grid - 1) / grid;
    const bool one_segment = ktiles % per == 0 && units % grid == 0;
    const double shared_us = full_us + 5.8 * (double)per + (one_segment ? 26.0 : 38.0) + 0.05 * (double)(grid + rem);
    if (shared_us >= 0.93 * plain_us) return plan;
    plan.full = (int)(rounds * 256);
    plan.rem = (int)rem;
    plan.grid = (int)grid;
    return plan;
}

static size_t scales_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    const int64_t mp = (M + 255) / 256 * 256, np = (N + 255) / 256 * 256;
    return (size_t)((mp + np) * (K / 16));
}

size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (K % BK4 != 0) return 0;
    const StreamPlan plan = stream_plan(M, N, K);
    const size_t sc = scales_workspace_bytes(M, N, K);
    return plan.rem ? (sc + 255) / 256 * 256 + (size_t)(plan.grid + plan.rem) * BM * BN * 4 : sc;
}

// test aids (host only): the sharing plan of a shape and the mapping the kernels use
void gemm_sharing_plan(int64_t M, int64_t N, int64_t K, int32_t plan[3])
{
    const StreamPlan p = stream_plan(M, N, K);
    plan[0] = p.full; plan[1] = p.rem; plan[2] = p.grid;
}

int gemm_sharing_segments(int rem, int ktotal, int grid, int block_id, int32_t *out)
{
    const int blk = sharing_block_number(block_id, grid);
    int64_t u, u_end;
    sharing_block_units((int64_t)rem * ktotal, grid, blk, u, u_end);
    int n = 0;
    while (u < u_end && n < 4) {
        int lt, kt0, ktiles;
        sharing_segment(u, u_end, ktotal, lt, kt0, ktiles);
        out[5 * n] = blk; out[5 * n + 1] = lt; out[5 * n + 2] = kt0; out[5 * n + 3] = ktiles; out[5 * n + 4] = sharing_slot(blk, lt);
        u += ktiles;
        ++n;
    }
    return u < u_end ? -1 : n;
}

void gemm_sharing_tile_slots(int rem, int ktotal, int grid, int lt, int32_t out[2])
{
    const int64_t U = (int64_t)rem * ktotal;
    out[0] = sharing_slot(sharing_block_of_unit((int64_t)lt * ktotal, U, grid), lt);
    out[1] = sharing_slot(sharing_block_of_unit((int64_t)lt * ktotal + ktotal - 1, U, grid), lt);
}

template <bool kBf16Out>
static hipError_t launch_main_kernel(const qii_nvfp4 &A, const uint8_t *a_tiled, const qii_nvfp4 &B, const uint8_t *b_tiled, void *C,
                                     int64_t ldc, int tiles_m, int tiles_n, uint32_t *amax_out, const StreamPlan &plan,
                                     float *partial, hipStream_t s)
{
    const int64_t M = A.rows, N = B.rows, K = A.cols;
    hipError_t e = allow_dynamic_lds(gemm_kernel_v4<kBf16Out, false>, kSmem4);
    if (e != hipSuccess) return e;
    e = allow_dynamic_lds(gemm_kernel_v4<kBf16Out, true>, kSmem4);
    if (e != hipSuccess) return e;
    if (plan.full > 0)
        hipLaunchKernelGGL((gemm_kernel_v4<kBf16Out, false>), dim3((unsigned)plan.full), dim3(256), kSmem4, s, A.codes, a_tiled,
                           A.tensor_scale, B.codes, b_tiled, B.tensor_scale, M, N, K, C, ldc, tiles_m, tiles_n, amax_out, 0, 0,
                           partial);
    if (plan.rem > 0) {
        hipLaunchKernelGGL((gemm_kernel_v4<kBf16Out, true>), dim3((unsigned)plan.grid), dim3(256), kSmem4, s, A.codes, a_tiled,
                           A.tensor_scale, B.codes, b_tiled, B.tensor_scale, M, N, K, C, ldc, tiles_m, tiles_n, amax_out, plan.full,
                           plan.rem, partial);
        hipLaunchKernelGGL(streamk_fixup_kernel<kBf16Out>, dim3((unsigned)plan.rem * 16), dim3(256), 0, s, partial, plan.full,
                           plan.rem, plan.grid, (int)(K / BK4), tiles_m, tiles_n, M, N, A.tensor_scale, B.tensor_scale, C, ldc,
                           amax_out);
    }
    return hipGetLastError();
}

hipError_t launch_gemm(const qii_nvfp4 &A, const qii_nvfp4 &B, void *C, int c_is_bf16, int64_t ldc,
                       float *amax_c, void *ws, size_t ws_bytes, hipStream_t s, int pretiled)
{
    const int64_t M = A.rows, N = B.rows, K = A.cols;
    if (pretiled && K % BK4 != 0) return hipErrorInvalidValue;
    uint32_t *amax_out = reinterpret_cast<uint32_t *>(amax_c);
    if (amax_out) {   // the running maximum starts at 0 (a kernel, not a memset node: graph capture)
        const hipError_t e = launch_fill_u32(amax_out, 0u, 1, 1, s);
        if (e != hipSuccess) return e;
    }
    if (M == 0 || N == 0) return hipSuccess;
    const int64_t tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(256);
    const size_t need = K % BK4 == 0 ? scales_workspace_bytes(M, N, K) : 0;
    // (the re-tiling kernel reads the row-major scale bytes 16 at a time)
    const bool a_ok = (pretiled & 4) || (reinterpret_cast<uintptr_t>(A.scales) & 15) == 0;
    const bool b_ok = (pretiled & 8) || (reinterpret_cast<uintptr_t>(B.scales) & 15) == 0;
    if (K % BK4 == 0 && ws && ws_bytes >= need && (reinterpret_cast<uintptr_t>(ws) & 15) == 0 && a_ok && b_ok) {
        uint8_t *a_ws = reinterpret_cast<uint8_t *>(ws);
        uint8_t *b_ws = a_ws + (M + 255) / 256 * 256 * (K / 16);
        const uint8_t *a_tiled = (pretiled & 1) ? A.scales : a_ws;   // (bits 2, 3: a_ws / b_ws are already filled)
        const uint8_t *b_tiled = (pretiled & 2) ? B.scales : b_ws;
        // the tiles of an incomplete last round are shared between blocks when the caller's workspace
        // has room for their partial tiles (behind the scales, 256-byte aligned)
        StreamPlan plan = stream_plan(M, N, K);
        const size_t poff = (need + 255) / 256 * 256;
        if (plan.rem && ws_bytes < poff + (size_t)(plan.grid + plan.rem) * BM * BN * 4) plan = StreamPlan{(int)(tiles_m * tiles_n), 0, 0};
        float *partial = plan.rem ? reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(ws) + poff) : nullptr;
        // (an operand whose scales arrive tiled takes no part: zero rows)
        const int64_t ma = (pretiled & 5) ? 0 : M, nb_rows = (pretiled & 10) ? 0 : N;
        const int64_t na = ma * (K / 256), nb = nb_rows * (K / 256);
        if (na + nb > 0)
            hipLaunchKernelGGL(retile_scales_kernel, dim3((unsigned)((na + nb + 255) / 256)), dim3(256), 0, s, A.scales,
                               a_ws, ma, B.scales, b_ws, nb_rows, K);
        return c_is_bf16 ? launch_main_kernel<true>(A, a_tiled, B, b_tiled, C, ldc, (int)tiles_m, (int)tiles_n, amax_out, plan, partial, s)
                         : launch_main_kernel<false>(A, a_tiled, B, b_tiled, C, ldc, (int)tiles_m, (int)tiles_n, amax_out, plan, partial, s);
    }
    if (pretiled) return hipErrorInvalidValue;   // only the main kernel reads tiled scales
    if ((K % 128) == 0) {
        hipError_t e;
        if (c_is_bf16) {
            e = allow_dynamic_lds(gemm_kernel_v2<true>, kSmem2);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(gemm_kernel_v2<true>, grid, block, kSmem2, s, A.codes, A.scales, A.tensor_scale,
                               B.codes, B.scales, B.tensor_scale, M, N, K, C, ldc, (int)tiles_m, (int)tiles_n, amax_out);
        } else {
            e = allow_dynamic_lds(gemm_kernel_v2<false>, kSmem2);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(gemm_kernel_v2<false>, grid, block, kSmem2, s, A.codes, A.scales, A.tensor_scale,
                               B.codes, B.scales, B.tensor_scale, M, N, K, C, ldc, (int)tiles_m, (int)tiles_n, amax_out);
        }
        return hipGetLastError();
    }
    // any K that is a multiple of 16: the ragged kernel (8-byte pieces, predicated tails)
    constexpr int smem = 2 * kStageBytes;
    hipError_t e;
    if (c_is_bf16) {
        e = allow_dynamic_lds(gemm_kernel<true>, smem);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(gemm_kernel<true>, grid, block, smem, s, A.codes, A.scales, A.tensor_scale, B.codes,
                           B.scales, B.tensor_scale, M, N, K, C, ldc, (int)tiles_n, amax_out);
    } else {
        e = allow_dynamic_lds(gemm_kernel<false>, smem);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(gemm_kernel<false>, grid, block, smem, s, A.codes, A.scales, A.tensor_scale, B.codes,
                           B.scales, B.tensor_scale, M, N, K, C, ldc, (int)tiles_n, amax_out);
    }
    return hipGetLastError();
}

}  // namespace qii
