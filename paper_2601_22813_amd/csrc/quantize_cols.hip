// Tuned quantizer / abs-max kernels for dense row-major sources quantized along their
// COLUMNS (the transposed case: Q(E^T), whose scale groups and rotation chunks run down the
// rows of x while memory is contiguous along its columns), and for the backward pass's
// re-quantization of a saved NVFP4 tensor with transposition (Q(W^T), Q(X^T)), where the
// source element is dequantized on load: (e2m1 * e4m3) * tensor_scale.
//
// Layout of the work: a lane owns one column j of x, i.e. one output row, and one whole
// 128-chunk of it: 128 registers.  A wave reads, for each of the 128 rows of the chunk, 64
// adjacent elements (one 128-byte line of bf16), so global loads stay coalesced without a
// transpose through LDS; all seven butterfly stages of the rotation, the eight group maxima
// and dot products are in-lane and the rotation signs are wave-uniform scalars.  A lane
// writes 64 contiguous bytes of codes and 8 scale bytes per chunk; the 4 waves of a block
// take 4 consecutive chunks of the same columns, so a block writes 256 contiguous bytes of
// every output row.  The scale-rounding draws follow the library-wide rule (one Philox call
// feeds rows 4q..4q+3 of one column group): the 4 lanes of a quad compute two calls each
// and hand the words round with quad broadcasts.
#include "qii_device.h"
#include "qii_internal.h"
#include "quantize_core.h"

namespace qii {
namespace {

constexpr float kInvSqrt128 = 0x1.6a09e6p-4f;  // binary32 nearest to 2^-3.5

struct ColsArgs {
    const void *x;       // f32 / bf16 data, or the FP4 codes of an NVFP4 source
    const uint8_t *in_scales;  // NVFP4 source only
    const float *in_ts;        // NVFP4 source only
    int64_t ld;          // elements (stored columns for an NVFP4 source)
    int64_t R, C;        // logical shape: R = columns of x (output rows), C = rows of x
    uint32_t sign[4];
    uint64_t seed_sr;
    const float *amax;
    uint8_t *codes;
    uint8_t *scales;
    float *tensor_scale;
    uint32_t *amax_out;
};

// load the 128 rows of one chunk of column j, widen to f32, apply the rotation signs.
// `chunk` is wave-uniform (scalar registers), so each row's address is a scalar base plus the
// lane's 32-bit column offset; j is clamped into the tensor by the caller, so every lane
// loads from a valid address and out-of-range lanes simply do not store.
template <int kSrc, bool kRht>
__device__ __forceinline__ void load_chunk(float v[128], const ColsArgs &a, int64_t chunk, uint32_t j)
{
    if (kSrc == kSrcNVFP4) {
        // two lanes share a code byte, sixteen a scale byte; batches of 32 rows bound the
        // number of loads (and registers) in flight
        const int64_t cstride = a.ld / 2, sstride = a.ld / 16;
        const uint8_t *pc = (const uint8_t *)a.x + (chunk * 128) * cstride;
        const uint8_t *ps = a.in_scales + (chunk * 128) * sstride;
        const uint32_t jc = j / 2, js = j / 16;
        const uint32_t shift = (j & 1u) * 4u;
        const float x32 = *a.in_ts;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            uint32_t rc[32], rs[32];
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                rc[i] = (pc + (int64_t)(32 * b + i) * cstride)[jc];
                rs[i] = (ps + (int64_t)(32 * b + i) * sstride)[js];
            }
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const int k = 32 * b + i;
                const float2_t c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(rc[i] >> shift, 1.0f, 0);
                const float m = c[0] * e4m3_decode(rs[i]);   // exact
                const uint32_t flip = kRht ? (((a.sign[k >> 5] >> (k & 31)) & 1u) << 31) : 0u;
                v[k] = m * u2f(f2u(x32) ^ flip);
            }
            asm volatile("" ::: "memory");
        }
        return;
    }
    constexpr bool kBf16 = kSrc == kSrcBF16;
    constexpr int esz = kBf16 ? 2 : 4;
    const char *base = (const char *)a.x + (chunk * 128) * a.ld * esz;
    const uint32_t off = j * esz;
    uint32_t raw[128];
#pragma unroll
    for (int i = 0; i < 128; ++i) {
        const char *rowp = base + (int64_t)i * a.ld * esz;
        raw[i] = kBf16 ? (uint32_t)*reinterpret_cast<const uint16_t *>(rowp + off)
                       : *reinterpret_cast<const uint32_t *>(rowp + off);
        // keep the loads in issue order in batches, so that address registers are recycled
        if ((i & 15) == 15) __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < 128; ++i) {
        uint32_t u = kBf16 ? (raw[i] << 16) : raw[i];
        if (kRht) u ^= ((a.sign[i >> 5] >> (i & 31)) & 1u) << 31;
        v[i] = u2f(u);
    }
}

// y = H v / sqrt(128) in registers: stages over index bits 0..6 in order
__device__ __forceinline__ void fwht128(float v[128])
{
#pragma unroll
    for (int len = 1; len < 128; len <<= 1)
#pragma unroll
        for (int i = 0; i < 128; ++i)
            if ((i & len) == 0) {
                const float x = v[i], y = v[i + len];
                v[i] = x + y;
                v[i + len] = x - y;
            }
#pragma unroll
    for (int i = 0; i < 128; ++i) v[i] = __builtin_fmaf(v[i], kInvSqrt128, 0.0f);  // +0 for exact zeros
}

template <int kSrcLane>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kSrcLane * 0x55, 0xF, 0xF, true);
}

// draws of the 8 groups (column groups 8*chunk .. 8*chunk+7) of output row j.
// Lane m of a quad computes the calls of column groups 2m and 2m+1 of the chunk; every lane
// then takes word (j mod 4) of each call.
__device__ __forceinline__ void quad_draws(uint32_t draw[8], uint64_t seed_sr, int64_t chunk, int64_t j)
{
    const int m = threadIdx.x & 3;
    const U4 wa = philox_seeded(seed_sr, (uint32_t)(chunk * 8 + 2 * m), (uint32_t)(j >> 2), 0, kStreamScale);
    const U4 wb = philox_seeded(seed_sr, (uint32_t)(chunk * 8 + 2 * m + 1), (uint32_t)(j >> 2), 0, kStreamScale);
#define QII_PICK(GI, SRC, W)                                                                      \
    do {                                                                                          \
        const uint32_t x = quad_bcast<SRC>(W.x), y = quad_bcast<SRC>(W.y);                        \
        const uint32_t z = quad_bcast<SRC>(W.z), w = quad_bcast<SRC>(W.w);                        \
        draw[GI] = (m == 0 ? x : m == 1 ? y : m == 2 ? z : w) >> 12;                              \
    } while (0)
    QII_PICK(0, 0, wa); QII_PICK(1, 0, wb); QII_PICK(2, 1, wa); QII_PICK(3, 1, wb);
    QII_PICK(4, 2, wa); QII_PICK(5, 2, wb); QII_PICK(6, 3, wa); QII_PICK(7, 3, wb);
#undef QII_PICK
}

template <int kSrc, int kMode, bool kRht>
__global__ __launch_bounds__(256, 2) void quantize_cols_kernel(ColsArgs a)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t chunk = (int64_t)blockIdx.x * 4 + wave;   // wave-uniform
    const int64_t j = (int64_t)blockIdx.y * 64 + lane;
    const TensorConsts tc = tensor_consts(kMode, *a.amax);
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *a.tensor_scale = tc.x32;
    if (chunk * 128 >= a.C) return;
    const bool ok = j < a.R;
    uint4 *pc = reinterpret_cast<uint4 *>(a.codes + j * (a.C / 2) + chunk * 64);
    uint2 *psc = reinterpret_cast<uint2 *>(a.scales + j * (a.C / 16) + chunk * 8);
    if (tc.zero) {  // uniform: an all-zero tensor is emitted as zero bytes
        if (ok) {
#pragma unroll
            for (int i = 0; i < 4; ++i) pc[i] = make_uint4(0u, 0u, 0u, 0u);
            *psc = make_uint2(0u, 0u);
        }
        return;
    }
    float v[128];
    load_chunk<kSrc, kRht>(v, a, chunk, (uint32_t)(ok ? j : a.R - 1));
    if (kRht) fwht128(v);
    uint32_t draw[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
    if (kMode == QII_MS_EDEN) quad_draws(draw, a.seed_sr, chunk, j);
    uint32_t sc[2] = {0u, 0u};
#pragma unroll
    for (int gp = 0; gp < 4; ++gp) {   // two groups = 16 bytes of codes per store
        uint32_t codes[4];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int gi = 2 * gp + h;
            const uint32_t b = quantize_group16<kMode>(v + 16 * gi, tc, draw[gi], a.seed_sr, j, chunk * 8 + gi, codes + 2 * h);
            sc[gi >> 2] |= b << (8 * (gi & 3));
        }
        if (ok) pc[gp] = make_uint4(codes[0], codes[1], codes[2], codes[3]);
    }
    if (ok) *psc = make_uint2(sc[0], sc[1]);
}

template <int kSrc, bool kRht>
__global__ __launch_bounds__(256, 2) void absmax_cols_kernel(ColsArgs a)
{
    __shared__ float wave_m[4];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t chunk = (int64_t)blockIdx.x * 4 + wave;   // wave-uniform
    const int64_t j = (int64_t)blockIdx.y * 64 + lane;
    float m = 0.0f;
    if (chunk * 128 < a.C) {
        float v[128];
        // a clamped duplicate of a real column cannot change the maximum
        load_chunk<kSrc, kRht>(v, a, chunk, (uint32_t)(j < a.R ? j : a.R - 1));
        if (kRht) fwht128(v);
#pragma unroll
        for (int gi = 0; gi < 8; ++gi) m = fmaxf(m, group_absmax(v + 16 * gi));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if (lane == 0) wave_m[wave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = fmaxf(fmaxf(wave_m[0], wave_m[1]), fmaxf(wave_m[2], wave_m[3]));
        // the running maximum only grows, so a stale read can only cause a redundant atomic
        if (f2u(m) > __atomic_load_n(a.amax_out, __ATOMIC_RELAXED)) atomicMax(a.amax_out, f2u(m));
    }
}

ColsArgs make_args(const Source &src, int64_t R, int64_t C, uint64_t seed_rht, uint64_t seed_sr)
{
    ColsArgs a;
    a.x = src.x; a.in_scales = src.scales; a.in_ts = src.ts; a.ld = src.ld; a.R = R; a.C = C;
    const U4 w = philox_seeded(seed_rht, 0, 0, 0, kStreamRht);
    a.sign[0] = w.x; a.sign[1] = w.y; a.sign[2] = w.z; a.sign[3] = w.w;
    a.seed_sr = seed_sr;
    a.amax = nullptr; a.codes = nullptr; a.scales = nullptr; a.tensor_scale = nullptr; a.amax_out = nullptr;
    return a;
}

dim3 cols_grid(int64_t R, int64_t C)
{
    return dim3((unsigned)((C / 128 + 3) / 4), (unsigned)((R + 63) / 64));
}

}  // namespace

bool cols_kernels_apply(const Source &src, int64_t R, int64_t C)
{
    return src.transpose && C % 128 == 0 && (R + 63) / 64 <= 65535;
}

hipError_t launch_absmax_cols(const Source &src, int64_t R, int64_t C, int rht, uint64_t seed_rht,
                              float *amax, hipStream_t s)
{
    ColsArgs a = make_args(src, R, C, seed_rht, 0);
    a.amax_out = reinterpret_cast<uint32_t *>(amax);
    const dim3 grid = cols_grid(R, C), block(256);
#define QII_AMAX(SRC)                                                                             \
    do {                                                                                          \
        if (rht) hipLaunchKernelGGL((absmax_cols_kernel<SRC, true>), grid, block, 0, s, a);       \
        else hipLaunchKernelGGL((absmax_cols_kernel<SRC, false>), grid, block, 0, s, a);          \
    } while (0)
    if (src.kind == kSrcBF16) QII_AMAX(kSrcBF16);
    else if (src.kind == kSrcF32) QII_AMAX(kSrcF32);
    else QII_AMAX(kSrcNVFP4);
#undef QII_AMAX
    return hipGetLastError();
}

hipError_t launch_quantize_cols(const QuantizeArgs &q, hipStream_t s)
{
    ColsArgs a = make_args(q.src, q.R, q.C, q.seed_rht, q.seed_sr);
    a.amax = q.amax; a.codes = q.codes; a.scales = q.scales; a.tensor_scale = q.tensor_scale;
    const dim3 grid = cols_grid(q.R, q.C), block(256);
#define QII_COLS(SRC, MODE, RHT) hipLaunchKernelGGL((quantize_cols_kernel<SRC, MODE, RHT>), grid, block, 0, s, a)
#define QII_COLS_MODE(SRC, RHT)                                   \
    do {                                                          \
        if (q.mode == QII_RTN) QII_COLS(SRC, QII_RTN, RHT);       \
        else if (q.mode == QII_SR) QII_COLS(SRC, QII_SR, RHT);    \
        else QII_COLS(SRC, QII_MS_EDEN, RHT);                     \
    } while (0)
#define QII_COLS_SRC(SRC)                                         \
    do {                                                          \
        if (q.rht) QII_COLS_MODE(SRC, true);                      \
        else QII_COLS_MODE(SRC, false);                           \
    } while (0)
    if (q.src.kind == kSrcBF16) QII_COLS_SRC(kSrcBF16);
    else if (q.src.kind == kSrcF32) QII_COLS_SRC(kSrcF32);
    else QII_COLS_SRC(kSrcNVFP4);
#undef QII_COLS_SRC
#undef QII_COLS_MODE
#undef QII_COLS
    return hipGetLastError();
}

}  // namespace qii
