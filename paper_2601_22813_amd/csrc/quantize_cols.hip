// Tuned quantizer / abs-max kernels for dense row-major sources quantized along their
// COLUMNS (the transposed case: Q(E^T), whose scale groups and rotation chunks run down the
// rows of x while memory is contiguous along its columns), and for the backward pass's
// re-quantization of a saved NVFP4 tensor with transposition (Q(W^T), Q(X^T)), where the
// source element is dequantized on load: (e2m1 * e4m3) * tensor_scale.
//
// Layout of the work: two neighbouring lanes own one column j of x (= one output row) and one
// 128-chunk of it, 64 values each (lane parity p holds rows 64p .. 64p+63 of the chunk), so a
// wave covers 32 columns and, for each of its 64 load instructions, two 64-byte row pieces:
// global loads stay coalesced without a transpose through LDS.  Butterfly stages over index
// bits 0..5 are in-lane, the last stage pairs the two lanes with one v_fmac_f32_dpp (the odd
// lane carries -(a - b), undone by the sign of its scaling constant, as in the row kernels).
// A lane owns four whole scale groups, so group maxima and dot products never leave it; it
// writes 32 contiguous bytes of codes and 4 scale bytes, a lane pair 64 + 8, and the 4 waves
// of a block take 4 consecutive chunks of the same columns (256 contiguous bytes per output
// row).  The scale-rounding draws follow the library-wide rule (one Philox call feeds rows
// 4q..4q+3 of one column group): the 8 lanes that own columns 4q..4q+3 compute one call each
// (column groups 0..7 of the chunk) and fetch the words they need with ds_bpermute.
#include "qii_device.h"
#include "qii_internal.h"
#include "quantize_core.h"

namespace qii {
namespace {

constexpr float kInvSqrt128 = 0x1.6a09e6p-4f;  // binary32 nearest to 2^-3.5
// a block's 4 waves: kColHalves neighbouring 32-column ranges x kChunksPerBlock chunks
constexpr int kColHalves = 1, kChunksPerBlock = 4;

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

// load this lane's 64 rows (rows 64p .. 64p+63 of the chunk) of column j, widen to f32 and
// apply the rotation signs.  `chunk` is wave-uniform; j is clamped into the tensor by the
// caller, so every lane loads from a valid address and out-of-range lanes do not store.
template <int kSrc, bool kRht>
__device__ __forceinline__ void load_half_chunk(float v[64], const ColsArgs &a, int64_t chunk, uint32_t j, int p)
{
    // rotation sign bits of this lane's 64 elements: words 2p and 2p+1
    const uint32_t s0 = p ? a.sign[2] : a.sign[0], s1 = p ? a.sign[3] : a.sign[1];
    if (kSrc == kSrcNVFP4) {
        // two columns share a code byte, sixteen a scale byte
        const int64_t cstride = a.ld / 2, sstride = a.ld / 16;
        const uint8_t *pc = (const uint8_t *)a.x + (chunk * 128 + 64 * p) * cstride + j / 2;
        const uint8_t *ps = a.in_scales + (chunk * 128 + 64 * p) * sstride + j / 16;
        const uint32_t shift = (j & 1u) * 4u;
        const float x32 = *a.in_ts;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            uint32_t rc[32], rs[32];
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                rc[i] = pc[(int64_t)(32 * b + i) * cstride];
                rs[i] = ps[(int64_t)(32 * b + i) * sstride];
            }
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const int k = 32 * b + i;
                const float2_t c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(rc[i] >> shift, 1.0f, 0);
                const float m = c[0] * e4m3_decode(rs[i]);   // exact
                const uint32_t flip = kRht ? ((((k < 32 ? s0 : s1) >> (k & 31)) & 1u) << 31) : 0u;
                v[k] = u2f(f2u(m * x32) ^ flip);
            }
        }
        return;
    }
    constexpr bool kBf16 = kSrc == kSrcBF16;
    constexpr int esz = kBf16 ? 2 : 4;
    const char *base = (const char *)a.x + ((chunk * 128 + 64 * p) * a.ld + j) * esz;
    uint32_t raw[64];
#pragma unroll
    for (int i = 0; i < 64; ++i) {
        const char *rowp = base + (int64_t)i * a.ld * esz;
        raw[i] = kBf16 ? (uint32_t)*reinterpret_cast<const uint16_t *>(rowp) : *reinterpret_cast<const uint32_t *>(rowp);
    }
#pragma unroll
    for (int i = 0; i < 64; ++i) {
        uint32_t u = kBf16 ? (raw[i] << 16) : raw[i];
        if (kRht) u ^= (((i < 32 ? s0 : s1) >> (i & 31)) & 1u) << 31;
        v[i] = u2f(u);
    }
}

// one cross-lane butterfly stage on 16 registers: v[k] += partner(v[k]) * s, partner = lane xor 1
__device__ __forceinline__ void dpp_pair_stage16(float *v, float s)
{
    asm volatile("s_nop 1\n"
                 "v_fmac_f32_dpp %0, %0, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %1, %1, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %2, %2, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %3, %3, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %4, %4, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %5, %5, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %6, %6, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %7, %7, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %8, %8, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %9, %9, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %10, %10, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %11, %11, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %12, %12, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %13, %13, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %14, %14, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 "v_fmac_f32_dpp %15, %15, %16 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
                 : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]),
                   "+v"(v[6]), "+v"(v[7]), "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]),
                   "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15])
                 : "v"(s));
}

// y = H v / sqrt(128) over the 128 values held by a lane pair: stages over index bits 0..5
// in-lane, bit 6 across the pair, then the scaling (the odd lane's constant is negative)
__device__ __forceinline__ void fwht128_pair(float v[64], int p)
{
#pragma unroll
    for (int len = 1; len < 64; len <<= 1)
#pragma unroll
        for (int i = 0; i < 64; ++i)
            if ((i & len) == 0) {
                const float x = v[i], y = v[i + len];
                v[i] = x + y;
                v[i + len] = x - y;
            }
    const float s = p ? -1.0f : 1.0f;
    dpp_pair_stage16(v, s);
    dpp_pair_stage16(v + 16, s);
    dpp_pair_stage16(v + 32, s);
    dpp_pair_stage16(v + 48, s);
    const float c = p ? -kInvSqrt128 : kInvSqrt128;
#pragma unroll
    for (int i = 0; i < 64; ++i) v[i] = __builtin_fmaf(v[i], c, 0.0f);  // +0 for exact zeros
}

// draws of this lane's 4 groups (column groups 8*chunk + 4p .. +3) of output row j.
// Lane o of an octet (the 8 lanes that own columns 4q..4q+3) computes the call of column
// group 8*chunk + o; a lane then takes word (j mod 4) of the calls of its own four groups.
__device__ __forceinline__ void octet_draws(uint32_t draw[4], uint64_t seed_sr, int64_t chunk, int64_t j, int p)
{
    const int lane = threadIdx.x & 63, o = lane & 7, word = (lane >> 1) & 3;
    const U4 w = philox_seeded(seed_sr, (uint32_t)(chunk * 8 + o), (uint32_t)(j >> 2), 0, kStreamScale);
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
        const int src = ((lane & ~7) | (4 * p + gi)) * 4;
        const uint32_t x = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)w.x);
        const uint32_t y = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)w.y);
        const uint32_t z = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)w.z);
        const uint32_t q = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)w.w);
        draw[gi] = (word == 0 ? x : word == 1 ? y : word == 2 ? z : q) >> 12;
    }
}

template <int kSrc, int kMode, bool kRht>
__global__ __launch_bounds__(256) void quantize_cols_kernel(ColsArgs a)
{
    const int lane = threadIdx.x & 63, p = lane & 1;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t chunk = (int64_t)blockIdx.x * kChunksPerBlock + (wave / kColHalves);   // wave-uniform
    const int64_t j = ((int64_t)blockIdx.y * kColHalves + (wave % kColHalves)) * 32 + (lane >> 1);
    const TensorConsts tc = tensor_consts(kMode, *a.amax);
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *a.tensor_scale = tc.x32;
    if (chunk * 128 >= a.C) return;
    const bool ok = j < a.R;
    uint4 *pc = reinterpret_cast<uint4 *>(a.codes + j * (a.C / 2) + chunk * 64 + 32 * p);
    uint32_t *psc = reinterpret_cast<uint32_t *>(a.scales + j * (a.C / 16) + chunk * 8 + 4 * p);
    if (tc.zero) {  // uniform: an all-zero tensor is emitted as zero bytes
        if (ok) {
            pc[0] = make_uint4(0u, 0u, 0u, 0u);
            pc[1] = make_uint4(0u, 0u, 0u, 0u);
            *psc = 0u;
        }
        return;
    }
    float v[64];
    load_half_chunk<kSrc, kRht>(v, a, chunk, (uint32_t)(ok ? j : a.R - 1), p);
    if (kRht) fwht128_pair(v, p);
    uint32_t draw[4] = {0u, 0u, 0u, 0u};
    if (kMode == QII_MS_EDEN) octet_draws(draw, a.seed_sr, chunk, j, p);
    uint32_t sc = 0u;
#pragma unroll
    for (int gp = 0; gp < 2; ++gp) {   // two groups = 16 bytes of codes per store
        uint32_t codes[4];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int gi = 2 * gp + h;
            const uint32_t b = quantize_group16<kMode>(v + 16 * gi, tc, draw[gi], a.seed_sr, j,
                                                       chunk * 8 + 4 * p + gi, codes + 2 * h);
            sc |= b << (8 * gi);
        }
        if (ok) pc[gp] = make_uint4(codes[0], codes[1], codes[2], codes[3]);
    }
    if (ok) *psc = sc;
}

template <int kSrc, bool kRht>
__global__ __launch_bounds__(256) void absmax_cols_kernel(ColsArgs a)
{
    __shared__ float wave_m[4];
    const int lane = threadIdx.x & 63, p = lane & 1;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t chunk = (int64_t)blockIdx.x * kChunksPerBlock + (wave / kColHalves);   // wave-uniform
    const int64_t j = ((int64_t)blockIdx.y * kColHalves + (wave % kColHalves)) * 32 + (lane >> 1);
    float m = 0.0f;
    if (chunk * 128 < a.C) {
        float v[64];
        // a clamped duplicate of a real column cannot change the maximum
        load_half_chunk<kSrc, kRht>(v, a, chunk, (uint32_t)(j < a.R ? j : a.R - 1), p);
        if (kRht) fwht128_pair(v, p);
#pragma unroll
        for (int gi = 0; gi < 4; ++gi) m = fmaxf(m, group_absmax(v + 16 * gi));
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
    return dim3((unsigned)((C / 128 + kChunksPerBlock - 1) / kChunksPerBlock),
                (unsigned)((R + 32 * kColHalves - 1) / (32 * kColHalves)));
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
