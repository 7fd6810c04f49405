// Exploratory NON-EXACT variants of the block-scaled GEMM, for measurement only: what gfx950's
// native block-scaled matrix instruction (v_mfma_scale_f32_32x32x64_f8f6f4, one power-of-two
// scale per 32 elements of K) delivers if NVFP4's numerics are given up.  Nothing in the layer
// passes reaches this file; the benchmark reports each variant's rate next to its error against
// the exact definition (paper Sec. 5 defines the GEMM on the dequantized operands).
//
//   QII_INEXACT_FP8      every operand element e2m1 * e4m3 (6 significant bits) is rounded to FP8
//                        E4M3 (4 significant bits) relative to a power-of-two scale per 32
//                        elements of K chosen from the block's largest magnitude; K = 64 per
//                        instruction at twice the f16 rate.
//   QII_INEXACT_FP4_POW2 the FP4 codes go to the instruction as they are, every 16-element group
//                        padded with 16 zeros to fill a 32-element scale block, and the group's
//                        E4M3 scale is rounded to the nearest power of two (its 3 mantissa bits
//                        are lost); 32 real elements of K per instruction at four times the f16
//                        rate (so twice the f16 rate per real element).
//
// A pre-pass writes both operands as images in the order of the kernel's LDS stages, per (row tile
// of 256, slice): 16 KiB of element bytes, row r keeping its 16-byte segment s in slot
// 4r + (s ^ ((r >> 2) & 3)), and the block scales as E8M0 bytes [row][blocks of the slice].  A slice
// is 64 elements of K: one instruction step for FP8, two for FP4 (whose image holds the padding
// zeros, so that a lane's operand is one 16-byte read).  The kernel is deliberately plain: the
// exact kernel's 256 x 256 tile and tile order, but 8 waves of 128 x 64 (two per SIMD, which cover
// each other's LDS latency: a step reads its operands, waits and multiplies), three LDS stages
// filled by linear LDS-direct loads two slices ahead, and stores straight from the accumulators.
#include "gemm_common.h"
#include "qii_device.h"
#include "qii_internal.h"

namespace qii {
namespace {

typedef int int8v __attribute__((ext_vector_type(8)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kImgBytes = 16384;     // element bytes of one operand per (row tile, slice)
constexpr int kImgScales = 2048;     // room for its scale bytes (FP8 uses 512, FP4 1024)
constexpr int kOffIA = 0, kOffIB = kImgBytes, kOffISA = 2 * kImgBytes, kOffISB = 2 * kImgBytes + kImgScales;
constexpr int kStageI = 2 * kImgBytes + 2 * kImgScales;   // 36 KiB
constexpr int kSmemI = 3 * kStageI;                        // 108 KiB

template <int kFmt> struct Fmt;
template <> struct Fmt<0> {   // FP8 E4M3
    static constexpr int kSliceK = 64, kSteps = 1, kScalesPerRow = 2;
};
template <> struct Fmt<4> {   // FP4, zero-padded groups
    static constexpr int kSliceK = 64, kSteps = 2, kScalesPerRow = 4;
};

__device__ __forceinline__ int swz(int r, int s) { return 4 * r + (s ^ ((r >> 2) & 3)); }

// E4M3 scale byte -> E8M0 byte of the nearest power of two (ties upward); 0 for a zero scale
__device__ __forceinline__ uint32_t e4m3_to_pow2_e8m0(uint32_t b)
{
    const uint32_t e = (b >> 3) & 15u, m = b & 7u;
    if (e == 0) {
        if (m == 0) return 0u;
        // subnormal: m * 2^-9, m = 1..7 -> 2^-9 (1), 2^-8 (2), 2^-7 (3: 1.5 up, .. 5), 2^-6 (6, 7)
        const int p = m == 1 ? -9 : m == 2 ? -8 : m <= 5 ? -7 : -6;
        return (uint32_t)(127 + p);
    }
    return 127u + e - 7u + (m >= 4 ? 1u : 0u);   // 1.5 and above round up (geometric midpoint 1.414)
}

// One thread = one row x one slice of one operand.  FP8: two blocks of 32; FP4: eight groups of 16.
template <int kFmt>
__global__ __launch_bounds__(256) void prepare_inexact_kernel(const uint8_t *__restrict__ a_codes,
                                                              const uint8_t *__restrict__ a_scales,
                                                              uint8_t *__restrict__ a_img, int64_t M,
                                                              const uint8_t *__restrict__ b_codes,
                                                              const uint8_t *__restrict__ b_scales,
                                                              uint8_t *__restrict__ b_img, int64_t N, int64_t K,
                                                              int64_t blocks_a)
{
    using F = Fmt<kFmt>;
    const int64_t nsl = K / F::kSliceK, sgroups = (nsl + 7) / 8;
    const bool is_b = (int64_t)blockIdx.x >= blocks_a;
    const int64_t blk = is_b ? (int64_t)blockIdx.x - blocks_a : (int64_t)blockIdx.x;
    const int64_t rows = is_b ? N : M;
    const uint8_t *codes = is_b ? b_codes : a_codes, *scales = is_b ? b_scales : a_scales;
    uint8_t *img = is_b ? b_img : a_img;
    const int64_t row = (blk / sgroups) * 32 + (threadIdx.x >> 3), sl = (blk % sgroups) * 8 + (threadIdx.x & 7);
    if (sl >= nsl) return;
    const int r8 = (int)(row & 255);
    uint8_t *dst = img + ((row >> 8) * nsl + sl) * (kImgBytes + kImgScales);
    uint8_t *dsc = dst + kImgBytes + r8 * F::kScalesPerRow;
    const bool live = row < rows;   // rows of the last tile beyond the matrix become zeros
    if (kFmt == 4) {
        uint4 c[2] = {};
        uint32_t sc = 0u;
        if (live) {
            const uint4 *src = reinterpret_cast<const uint4 *>(codes + row * (K / 2) + sl * 32);
            c[0] = src[0];
            c[1] = src[1];
            sc = *reinterpret_cast<const uint32_t *>(scales + row * (K / 16) + sl * 4);
        }
        // segment g of the row: the 16 codes of group g, then 16 zero codes (the padding of its scale block)
        *reinterpret_cast<uint4 *>(dst + swz(r8, 0) * 16) = make_uint4(c[0].x, c[0].y, 0u, 0u);
        *reinterpret_cast<uint4 *>(dst + swz(r8, 1) * 16) = make_uint4(c[0].z, c[0].w, 0u, 0u);
        *reinterpret_cast<uint4 *>(dst + swz(r8, 2) * 16) = make_uint4(c[1].x, c[1].y, 0u, 0u);
        *reinterpret_cast<uint4 *>(dst + swz(r8, 3) * 16) = make_uint4(c[1].z, c[1].w, 0u, 0u);
        *reinterpret_cast<uint32_t *>(dsc) = e4m3_to_pow2_e8m0(sc & 255u) | (e4m3_to_pow2_e8m0((sc >> 8) & 255u) << 8) |
                                             (e4m3_to_pow2_e8m0((sc >> 16) & 255u) << 16) | (e4m3_to_pow2_e8m0(sc >> 24) << 24);
    } else {
        uint4 c[2] = {};
        uint32_t sc = 0u;
        if (live) {
            const uint4 *src = reinterpret_cast<const uint4 *>(codes + row * (K / 2) + sl * 32);
            c[0] = src[0];
            c[1] = src[1];
            sc = *reinterpret_cast<const uint32_t *>(scales + row * (K / 16) + sl * 4);
        }
        const uint32_t w[8] = {c[0].x, c[0].y, c[0].z, c[0].w, c[1].x, c[1].y, c[1].z, c[1].w};
        uint32_t e8[2];
#pragma unroll
        for (int blk32 = 0; blk32 < 2; ++blk32) {
            // exact products of the block's 32 elements, their largest magnitude, the block scale
            float v[32];
            float mx = 0.0f;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const float x8 = e4m3_decode((sc >> (8 * (2 * blk32 + (d >> 1)))) & 255u);
#define QII_DQ(P)                                                                                     \
    do {                                                                                              \
        const float2_t t = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * blk32 + d], 1.0f, P);       \
        v[8 * d + 2 * P] = t[0] * x8;                                                                 \
        v[8 * d + 2 * P + 1] = t[1] * x8;                                                             \
        mx = fmaxf(mx, fmaxf(fabsf(v[8 * d + 2 * P]), fabsf(v[8 * d + 2 * P + 1])));                  \
    } while (0)
                QII_DQ(0); QII_DQ(1); QII_DQ(2); QII_DQ(3);
#undef QII_DQ
            }
            // largest element lands in [128, 256): inside E4M3's range (448)
            const int ex = mx > 0.0f ? (int)((f2u(mx) >> 23) & 255u) - 127 - 7 : 0;
            e8[blk32] = (uint32_t)(127 + ex);
            const float inv = u2f((uint32_t)(127 - ex) << 23);
            uint32_t out[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                uint32_t pk = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(v[4 * q] * inv, v[4 * q + 1] * inv, 0, false);
                pk = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(v[4 * q + 2] * inv, v[4 * q + 3] * inv, (int)pk, true);
                out[q] = pk;
            }
            // the block's 32 bytes: segments 2 blk32 and 2 blk32 + 1 of the row
            *reinterpret_cast<uint4 *>(dst + swz(r8, 2 * blk32) * 16) = make_uint4(out[0], out[1], out[2], out[3]);
            *reinterpret_cast<uint4 *>(dst + swz(r8, 2 * blk32 + 1) * 16) = make_uint4(out[4], out[5], out[6], out[7]);
        }
        *reinterpret_cast<uint16_t *>(dsc) = (uint16_t)(e8[0] | (e8[1] << 8));
    }
}

// 512 threads: 16 KiB of an operand are two block-wide loads of 16 bytes per lane; the scale bytes
// one load of 4 bytes per lane (FP8 has 512 bytes per operand: waves re-load them pairwise, which
// keeps the number of loads per thread uniform)
template <int kFmt>
__device__ __forceinline__ void issue_slice_loads_i(uint8_t *stage, const uint8_t *a_slice, const uint8_t *b_slice, int wave)
{
    using F = Fmt<kFmt>;
    const int t = threadIdx.x, lane = t & 63;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        __builtin_amdgcn_global_load_lds(a_slice + p * 8192 + t * 16,
                                         (__attribute__((address_space(3))) void *)(stage + kOffIA + p * 8192 + wave * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds(b_slice + p * 8192 + t * 16,
                                         (__attribute__((address_space(3))) void *)(stage + kOffIB + p * 8192 + wave * 1024), 16, 0, 0);
    }
    const int off = (F::kScalesPerRow == 2 ? (wave & 1) : (wave & 3)) * 256;
    __builtin_amdgcn_global_load_lds(a_slice + kImgBytes + off + lane * 4,
                                     (__attribute__((address_space(3))) void *)(stage + kOffISA + off), 4, 0, 0);
    __builtin_amdgcn_global_load_lds(b_slice + kImgBytes + off + lane * 4,
                                     (__attribute__((address_space(3))) void *)(stage + kOffISB + off), 4, 0, 0);
}
constexpr int kLoadsI = 6;   // LDS-direct loads per thread and slice

// Operands of one step of one wave (128 x 64 of the tile): 4 row blocks of A, 2 of B, as the LDS
// reads deliver them (FP8: two 16-byte pieces each; FP4: one, codes and padding) and their scale
// bytes.  The matrix instruction takes consecutive registers per operand; they are put together
// after the wait.
template <int kFmt> struct FragsI;
template <> struct FragsI<0> {
    u32x4 alo[4], ahi[4], blo[2], bhi[2];
    uint32_t sa[4], sb[2];
};
template <> struct FragsI<4> {
    u32x4 a4[4], b4[2];
    uint32_t sa[4], sb[2];
};

struct FragAddrI {
    uint32_t a, b, sa, sb;   // LDS byte addresses of row block 0 in stage 0 (without the step's part)
    uint32_t li, kb;
};

// LDS reads of step `step` of the slice in the stage at stage_off, and the wait for them
__device__ __forceinline__ void frag_read_i(FragsI<0> &f, const FragAddrI &fa, uint32_t stage_off, int)
{
    // FP8: this lane's 16 bytes of block 0 (segment kb) and of block 1 (segment 2 + kb); scale of block kb
    const uint32_t x0 = ((fa.kb) ^ ((fa.li >> 2) & 3)) * 16, x1 = ((2 + fa.kb) ^ ((fa.li >> 2) & 3)) * 16;
    const uint32_t va0 = fa.a + stage_off + x0, va1 = fa.a + stage_off + x1;
    const uint32_t vb0 = fa.b + stage_off + x0, vb1 = fa.b + stage_off + x1;
    const uint32_t vsa = fa.sa + stage_off + fa.kb, vsb = fa.sb + stage_off + fa.kb;
#define QII_RDA(T)                                                                                            \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.alo[T]) : "v"(va0), "n"(T * 2048));                 \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.ahi[T]) : "v"(va1), "n"(T * 2048));                 \
    asm volatile("ds_read_u8 %0, %1 offset:%2" : "=v"(f.sa[T]) : "v"(vsa), "n"(T * 64))
#define QII_RDB(T)                                                                                            \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.blo[T]) : "v"(vb0), "n"(T * 2048));                 \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.bhi[T]) : "v"(vb1), "n"(T * 2048));                 \
    asm volatile("ds_read_u8 %0, %1 offset:%2" : "=v"(f.sb[T]) : "v"(vsb), "n"(T * 64))
    QII_RDA(0); QII_RDA(1); QII_RDA(2); QII_RDA(3); QII_RDB(0); QII_RDB(1);
#undef QII_RDA
#undef QII_RDB
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f.alo[0]), "+v"(f.alo[1]), "+v"(f.alo[2]), "+v"(f.alo[3]), "+v"(f.ahi[0]), "+v"(f.ahi[1]),
                   "+v"(f.ahi[2]), "+v"(f.ahi[3]), "+v"(f.blo[0]), "+v"(f.blo[1]), "+v"(f.bhi[0]), "+v"(f.bhi[1]),
                   "+v"(f.sa[0]), "+v"(f.sa[1]), "+v"(f.sa[2]), "+v"(f.sa[3]), "+v"(f.sb[0]), "+v"(f.sb[1]));
}

__device__ __forceinline__ void frag_read_i(FragsI<4> &f, const FragAddrI &fa, uint32_t stage_off, int step)
{
    // FP4: group 2 step + kb of the slice, with its padding: segment 2 step + kb of the row
    const uint32_t x = (((uint32_t)(2 * step) + fa.kb) ^ ((fa.li >> 2) & 3)) * 16;
    const uint32_t va = fa.a + stage_off + x, vb = fa.b + stage_off + x;
    const uint32_t vsa = fa.sa + stage_off + 2 * step + fa.kb, vsb = fa.sb + stage_off + 2 * step + fa.kb;
#define QII_RDA(T)                                                                                            \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.a4[T]) : "v"(va), "n"(T * 2048));                   \
    asm volatile("ds_read_u8 %0, %1 offset:%2" : "=v"(f.sa[T]) : "v"(vsa), "n"(T * 128))
#define QII_RDB(T)                                                                                            \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.b4[T]) : "v"(vb), "n"(T * 2048));                   \
    asm volatile("ds_read_u8 %0, %1 offset:%2" : "=v"(f.sb[T]) : "v"(vsb), "n"(T * 128))
    QII_RDA(0); QII_RDA(1); QII_RDA(2); QII_RDA(3); QII_RDB(0); QII_RDB(1);
#undef QII_RDA
#undef QII_RDB
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f.a4[0]), "+v"(f.a4[1]), "+v"(f.a4[2]), "+v"(f.a4[3]), "+v"(f.b4[0]), "+v"(f.b4[1]), "+v"(f.sa[0]),
                   "+v"(f.sa[1]), "+v"(f.sa[2]), "+v"(f.sa[3]), "+v"(f.sb[0]), "+v"(f.sb[1]));
}

__device__ __forceinline__ int8v operand_i(const u32x4 &lo, const u32x4 &hi)
{
    return __builtin_bit_cast(int8v, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
// (an FP4 operand is 4 registers wide: the instruction does not read the upper half)
__device__ __forceinline__ int8v operand_i(const u32x4 &w)
{
    return __builtin_bit_cast(int8v, __builtin_shufflevector(w, w, 0, 1, 2, 3, -1, -1, -1, -1));
}

__device__ __forceinline__ void operands_i(int8v (&a)[4], int8v (&b)[2], const FragsI<0> &f)
{
#pragma unroll
    for (int t = 0; t < 4; ++t) a[t] = operand_i(f.alo[t], f.ahi[t]);
#pragma unroll
    for (int t = 0; t < 2; ++t) b[t] = operand_i(f.blo[t], f.bhi[t]);
}
__device__ __forceinline__ void operands_i(int8v (&a)[4], int8v (&b)[2], const FragsI<4> &f)
{
#pragma unroll
    for (int t = 0; t < 4; ++t) a[t] = operand_i(f.a4[t]);
#pragma unroll
    for (int t = 0; t < 2; ++t) b[t] = operand_i(f.b4[t]);
}

// 8 waves of a block, 2 (rows) x 4 (columns), each 128 x 64 of the 256 x 256 tile: two waves share a
// SIMD and cover each other's LDS latency, so a step simply reads its operands, waits and multiplies.
template <int kFmt, bool kBf16Out>
__global__ __launch_bounds__(512, 1) void gemm_inexact_kernel(const uint8_t *__restrict__ a_img, const float *__restrict__ a_ts,
                                                              const uint8_t *__restrict__ b_img, const float *__restrict__ b_ts,
                                                              int64_t M, int64_t N, int64_t K, void *__restrict__ Cout,
                                                              int64_t ldc, int tiles_m, int tiles_n)
{
    using F = Fmt<kFmt>;
    extern __shared__ __align__(16) uint8_t smem[];
    int tile = blockIdx.x;
    const int ntiles = tiles_m * tiles_n;
    if ((ntiles & 7) == 0) tile = (tile & 7) * (ntiles >> 3) + (tile >> 3);   // a contiguous run of tiles per die
    constexpr int kGroupM = 4;
    const int width = kGroupM * tiles_n, first_m = (tile / width) * kGroupM;
    const int gm = tiles_m - first_m < kGroupM ? tiles_m - first_m : kGroupM;
    const int tm = first_m + (tile % width) % gm, tn = (tile % width) / gm;
    const int64_t m0 = (int64_t)tm * 256, n0 = (int64_t)tn * 256;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int li = lane & 31, kb = lane >> 5;
    const int n = (int)(K / F::kSliceK);   // slices
    constexpr int64_t kSliceBytes = kImgBytes + kImgScales;
    const uint8_t *a_tile = a_img + (int64_t)tm * n * kSliceBytes, *b_tile = b_img + (int64_t)tn * n * kSliceBytes;

    floatx16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    FragAddrI fa;
    {
        const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
        fa.a = lds0 + kOffIA + (wm * 128 + li) * 64;
        fa.b = lds0 + kOffIB + (wn * 64 + li) * 64;
        fa.sa = lds0 + kOffISA + (wm * 128 + li) * F::kScalesPerRow;
        fa.sb = lds0 + kOffISB + (wn * 64 + li) * F::kScalesPerRow;
        fa.li = (uint32_t)li;
        fa.kb = (uint32_t)kb;
    }

    // slices 0, 1, 2 into stages 0, 1, 2; slice g + 3 follows into the stage of slice g once everybody
    // has finished reading it (the barrier at the end of slice g)
    for (int g = 0; g < 3 && g < n; ++g)
        issue_slice_loads_i<kFmt>(smem + g * kStageI, a_tile + g * kSliceBytes, b_tile + g * kSliceBytes, wave);
    uint32_t cur_off = 0;
    for (int g = 0; g < n; ++g) {
        // slice g must have landed for everybody: of this wave's loads at most those of slices g + 1, g + 2 may be in flight
        if (g + 2 < n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * kLoadsI) : "memory");
        else if (g + 1 < n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoadsI) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
#pragma unroll
        for (int st = 0; st < F::kSteps; ++st) {
            FragsI<kFmt> f;
            frag_read_i(f, fa, cur_off, st);
            int8v a[4], b[2];
            operands_i(a, b, f);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[j], acc[i][j], kFmt, kFmt, 0,
                                                                                (int)f.sa[i], 0, (int)f.sb[j]);
        }
        __builtin_amdgcn_s_barrier();   // everybody is done reading this stage
        asm volatile("" ::: "memory");
        if (g + 3 < n)
            issue_slice_loads_i<kFmt>(smem + cur_off, a_tile + (int64_t)(g + 3) * kSliceBytes, b_tile + (int64_t)(g + 3) * kSliceBytes, wave);
        cur_off = cur_off + kStageI == (uint32_t)kSmemI ? 0u : cur_off + kStageI;
    }
    // epilogue: C = acc * (x32_A * x32_B), straight from the registers.  acc[r] of a 32 x 32 block is row
    // 8 (r / 4) + 4 kb + r % 4, column li: a wave-wide store covers 2 rows x 32 consecutive columns.
    const float ts = (*a_ts) * (*b_ts);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t col = n0 + wn * 64 + j * 32 + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * kb + (r & 3);
                if (row < M && col < N) {
                    const float v = acc[i][j][r] * ts;
                    if (kBf16Out) reinterpret_cast<uint16_t *>(Cout)[row * ldc + col] = f32_to_bf16_bits(v);
                    else reinterpret_cast<float *>(Cout)[row * ldc + col] = v;
                }
            }
        }
}

}  // namespace

size_t gemm_inexact_workspace_bytes(int64_t M, int64_t N, int64_t K, int variant)
{
    const int slice = 64;
    (void)variant;
    if (K % slice != 0) return 0;
    const int64_t tm = (M + 255) / 256, tn = (N + 255) / 256;
    return (size_t)((tm + tn) * (K / slice) * (kImgBytes + kImgScales));
}

template <int kFmt>
static hipError_t launch_inexact(const qii_nvfp4 &A, const qii_nvfp4 &B, void *C, int c_is_bf16, int64_t ldc, void *ws,
                                 hipStream_t s)
{
    using F = Fmt<kFmt>;
    const int64_t M = A.rows, N = B.rows, K = A.cols;
    const int64_t tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256, nsl = K / F::kSliceK, sgroups = (nsl + 7) / 8;
    uint8_t *a_img = reinterpret_cast<uint8_t *>(ws);
    uint8_t *b_img = a_img + tiles_m * nsl * (kImgBytes + kImgScales);
    const int64_t blocks_a = tiles_m * 8 * sgroups, blocks_b = tiles_n * 8 * sgroups;
    hipLaunchKernelGGL(prepare_inexact_kernel<kFmt>, dim3((unsigned)(blocks_a + blocks_b)), dim3(256), 0, s, A.codes, A.scales,
                       a_img, M, B.codes, B.scales, b_img, N, K, blocks_a);
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(512);
    hipError_t e;
    if (c_is_bf16) {
        e = allow_dynamic_lds(gemm_inexact_kernel<kFmt, true>, kSmemI);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((gemm_inexact_kernel<kFmt, true>), grid, block, kSmemI, s, a_img, A.tensor_scale, b_img,
                           B.tensor_scale, M, N, K, C, ldc, (int)tiles_m, (int)tiles_n);
    } else {
        e = allow_dynamic_lds(gemm_inexact_kernel<kFmt, false>, kSmemI);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((gemm_inexact_kernel<kFmt, false>), grid, block, kSmemI, s, a_img, A.tensor_scale, b_img,
                           B.tensor_scale, M, N, K, C, ldc, (int)tiles_m, (int)tiles_n);
    }
    return hipGetLastError();
}

hipError_t launch_gemm_inexact(const qii_nvfp4 &A, const qii_nvfp4 &B, void *C, int c_is_bf16, int64_t ldc, int variant,
                               void *ws, hipStream_t s)
{
    if (A.rows == 0 || B.rows == 0) return hipSuccess;
    if (variant == QII_INEXACT_FP8) return launch_inexact<0>(A, B, C, c_is_bf16, ldc, ws, s);
    return launch_inexact<4>(A, B, C, c_is_bf16, ldc, ws, s);
}

}  // namespace qii
