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
// Tiling: 256 x 256 block tile, K tile 128, 4 waves (2 x 2) each owning 128 x 128 =
// 4 x 4 MFMA tiles (256 accumulator registers).  One 32x32x16 MFMA consumes exactly
// one scale group per lane: lanes 0..31 supply k 0..31 of a 64-element K slice and
// lanes 32..63 supply k 32..63, four MFMAs walk the four dwords of a lane's 16 bytes
// (the order of k inside the contraction is free as long as A and B agree).
#include "qii_device.h"
#include "qii_internal.h"

namespace qii {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

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

template <bool kAlignedK>
__device__ __forceinline__ uint2 load_scales(const uint8_t *scales, int64_t row, int64_t nrows,
                                             int64_t K, int64_t k0)
{
    uint2 r = make_uint2(0u, 0u);
    if (row >= nrows) return r;
    const uint8_t *p = scales + row * (K / 16) + k0 / 16;
    if (kAlignedK) return *reinterpret_cast<const uint2 *>(p);
    uint32_t w[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (k0 + 16 * i < K) w[i >> 2] |= (uint32_t)p[i] << (8 * (i & 3));
    return make_uint2(w[0], w[1]);
}

template <bool kAlignedK>
__device__ __forceinline__ void load_tile(Staged &st, const uint8_t *a_codes, const uint8_t *a_scales,
                                          const uint8_t *b_codes, const uint8_t *b_scales, int64_t M,
                                          int64_t N, int64_t K, int64_t m0, int64_t n0, int64_t k0)
{
    const int t = threadIdx.x;
    const int seg = t & 3, r = t >> 2;
    const int64_t kbyte = k0 / 2 + 16 * seg;
    const bool k_ok = kAlignedK || (k0 + 32 * seg < K);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int64_t ra = m0 + p * 64 + r, rb = n0 + p * 64 + r;
        st.a[p] = (k_ok && ra < M) ? *reinterpret_cast<const uint4 *>(a_codes + ra * (K / 2) + kbyte)
                                   : make_uint4(0u, 0u, 0u, 0u);
        st.b[p] = (k_ok && rb < N) ? *reinterpret_cast<const uint4 *>(b_codes + rb * (K / 2) + kbyte)
                                   : make_uint4(0u, 0u, 0u, 0u);
    }
    st.as = load_scales<kAlignedK>(a_scales, m0 + t, M, K, k0);
    st.bs = load_scales<kAlignedK>(b_scales, n0 + t, N, K, k0);
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

template <bool kAlignedK, bool kBf16Out>
__global__ __launch_bounds__(256, 1) void gemm_kernel(const uint8_t *__restrict__ a_codes,
                                                      const uint8_t *__restrict__ a_scales,
                                                      const float *__restrict__ a_ts,
                                                      const uint8_t *__restrict__ b_codes,
                                                      const uint8_t *__restrict__ b_scales,
                                                      const float *__restrict__ b_ts, int64_t M,
                                                      int64_t N, int64_t K, void *__restrict__ Cout,
                                                      int64_t ldc, int tiles_n)
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
    load_tile<kAlignedK>(st, a_codes, a_scales, b_codes, b_scales, M, N, K, m0, n0, 0);
    store_tile(st, stage_ptr(smem, 0));
    __syncthreads();

    for (int64_t kt = 0; kt < ktiles; ++kt) {
        const StagePtr sp = stage_ptr(smem, (int)(kt & 1));
        if (kt + 1 < ktiles)
            load_tile<kAlignedK>(st, a_codes, a_scales, b_codes, b_scales, M, N, K, m0, n0, (kt + 1) * BK);
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
        // ask the scheduler to slot the dequantization (VALU) of the next fragments under the
        // matrix instructions: one MFMA, then five VALU ops, over the whole K tile
#pragma unroll
        for (int i = 0; i < 128; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
        }
        if (kt + 1 < ktiles) {
            store_tile(st, stage_ptr(smem, (int)((kt + 1) & 1)));
            __syncthreads();
        }
    }

    // epilogue: C = acc * (x32_A * x32_B).  acc[r] of a 32x32 tile is row
    // 8*(r/4) + 4*(lane/32) + r%4, column lane%32.
    const float ts = (*a_ts) * (*b_ts);
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
                    if (kBf16Out) reinterpret_cast<uint16_t *>(Cout)[row * ldc + col] = (uint16_t)f32_to_bf16_bits(v);
                    else reinterpret_cast<float *>(Cout)[row * ldc + col] = v;
                }
            }
        }
}

}  // namespace

hipError_t launch_gemm(const qii_nvfp4 &A, const qii_nvfp4 &B, void *C, int c_is_bf16, int64_t ldc,
                       hipStream_t s)
{
    const int64_t M = A.rows, N = B.rows, K = A.cols;
    if (M == 0 || N == 0) return hipSuccess;
    const int64_t tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(256);
    const size_t smem = 2 * kStageBytes;
    const bool aligned = (K % 128) == 0;
#define QII_GEMM(AL, BF)                                                                          \
    do {                                                                                          \
        auto kern = gemm_kernel<AL, BF>;                                                          \
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); \
        if (e != hipSuccess) return e;                                                            \
        hipLaunchKernelGGL(kern, grid, block, smem, s, A.codes, A.scales, A.tensor_scale, B.codes, \
                           B.scales, B.tensor_scale, M, N, K, C, ldc, (int)tiles_n);              \
    } while (0)
    if (aligned) { if (c_is_bf16) QII_GEMM(true, true); else QII_GEMM(true, false); }
    else { if (c_is_bf16) QII_GEMM(false, true); else QII_GEMM(false, false); }
#undef QII_GEMM
    return hipGetLastError();
}

}  // namespace qii
