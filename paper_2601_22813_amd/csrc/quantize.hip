// Quantizer kernels of libqii: rotated abs-max, stand-alone RHT, and the NVFP4
// quantizers RTN / SR / MS-EDEN (paper Sec. 3.1, Sec. 3.3 Algorithm 1, Table 1).
//
// Work decomposition ("one lane = one scale group"):
//   a lane owns the 16 consecutive elements of one NVFP4 scale group, so the group
//   max, the two EDEN dot products and the 8 code bytes never leave the lane;
//   8 neighbouring lanes (an octet) own one 128-chunk of the rotation.  The first four
//   butterfly stages of the Hadamard transform are in-lane, the last three exchange
//   registers with lanes xor 1, xor 2 and xor 7 through DPP (quad_perm, quad_perm,
//   row_half_mirror); lanes 4..7 of an octet hold the 16-blocks of the chunk in
//   reverse order so that "xor 7" pairs blocks that differ in index bit 2.
//   An octet processes 4 consecutive rows of the same chunk, which lets one
//   Philox4x32 call feed the four scale roundings of a lane.
#include "qii_device.h"
#include "qii_internal.h"
#include "quantize_core.h"

namespace qii {
namespace {

constexpr float kInvSqrt128 = 0x1.6a09e6p-4f;  // binary32 nearest to 2^-3.5

// ------------------------------------------------------------------ loaders
// Each loader fills v[0..15] with logical elements (row, col0 .. col0+15) as f32.
struct LoadContigBF16 {
    const uint16_t *x; int64_t ld;
    __device__ __forceinline__ void operator()(int64_t row, int64_t col0, float v[16]) const {
        const uint4 *p = reinterpret_cast<const uint4 *>(x + row * ld + col0);
        const uint4 a = p[0], b = p[1];
        const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) { v[2 * i] = bf16_lo(w[i]); v[2 * i + 1] = bf16_hi(w[i]); }
    }
};
struct LoadContigF32 {
    const float *x; int64_t ld;
    __device__ __forceinline__ void operator()(int64_t row, int64_t col0, float v[16]) const {
        const float4 *p = reinterpret_cast<const float4 *>(x + row * ld + col0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 t = p[i];
            v[4 * i] = t.x; v[4 * i + 1] = t.y; v[4 * i + 2] = t.z; v[4 * i + 3] = t.w;
        }
    }
};
struct LoadTransBF16 {
    const uint16_t *x; int64_t ld;
    __device__ __forceinline__ void operator()(int64_t row, int64_t col0, float v[16]) const {
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = u2f((uint32_t)x[(col0 + k) * ld + row] << 16);
    }
};
struct LoadTransF32 {
    const float *x; int64_t ld;
    __device__ __forceinline__ void operator()(int64_t row, int64_t col0, float v[16]) const {
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = x[(col0 + k) * ld + row];
    }
};
// dequantized NVFP4: x_hat = (e2m1 * e4m3) * tensor_scale (first product exact)
struct LoadContigNVFP4 {
    const uint8_t *codes; const uint8_t *scales; const float *ts; int64_t cols;
    __device__ __forceinline__ void operator()(int64_t row, int64_t col0, float v[16]) const {
        const uint2 c = *reinterpret_cast<const uint2 *>(codes + (row * cols + col0) / 2);
        const float x8 = e4m3_decode(scales[row * (cols / 16) + col0 / 16]);
        const float x32 = *ts;
        const uint32_t w[2] = {c.x, c.y};
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const uint32_t code = (w[k >> 3] >> (4 * (k & 7))) & 15u;
            const float m = e2m1_decode_mag(code & 7u) * x8;
            v[k] = u2f(f2u(m * x32) ^ ((code & 8u) << 28));
        }
    }
};
struct LoadTransNVFP4 {
    const uint8_t *codes; const uint8_t *scales; const float *ts; int64_t cols;  // stored cols
    __device__ __forceinline__ void operator()(int64_t row, int64_t col0, float v[16]) const {
        const float x32 = *ts;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int64_t sr = col0 + k, sc = row;  // stored (row, col)
            const uint32_t byte = codes[(sr * cols + sc) / 2];
            const uint32_t code = (sc & 1) ? (byte >> 4) : (byte & 15u);
            const float x8 = e4m3_decode(scales[sr * (cols / 16) + sc / 16]);
            const float m = e2m1_decode_mag(code & 7u) * x8;
            v[k] = u2f(f2u(m * x32) ^ ((code & 8u) << 28));
        }
    }
};

// ------------------------------------------------------------------ lane geometry
struct Lane {
    int64_t quad;   // rows 4*quad .. 4*quad+3
    int64_t g;      // scale-group index within the row
    int blk;        // 16-block of the 128-chunk owned by this lane (0..7)
    bool in_range;  // g < groups per row and quad within the tensor
};

__device__ __forceinline__ Lane lane_geometry(int64_t R, int64_t G)
{
    const int sub = threadIdx.x & 7;
    const int blk = (sub & 4) ? (sub ^ 3) : sub;
    const int64_t nch = (G + 7) / 8;
    const int64_t oct = (int64_t)blockIdx.x * (blockDim.x / 8) + (threadIdx.x >> 3);
    Lane L;
    L.quad = oct / nch;
    L.g = (oct % nch) * 8 + blk;
    L.blk = blk;
    L.in_range = (L.g < G) && (L.quad * 4 < R);
    return L;
}

__host__ inline int64_t grid_for(int64_t R, int64_t C, int threads)
{
    const int64_t G = C / 16, nch = (G + 7) / 8, quads = (R + 3) / 4;
    const int64_t octs = nch * quads, per_block = threads / 8;
    return (octs + per_block - 1) / per_block;
}

// ------------------------------------------------------------------ RHT on 16 regs x 8 lanes
// y = H (d .* v) / sqrt(128), H Sylvester, stages over index bits 0..6 in order.
__device__ __forceinline__ void rht128(float v[16], uint32_t sign16, int blk)
{
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = u2f(f2u(v[k]) ^ (((sign16 >> k) & 1u) << 31));
#pragma unroll
    for (int len = 1; len < 16; len <<= 1)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if ((i & len) == 0) {
                const float a = v[i], b = v[i + len];
                v[i] = a + b;
                v[i + len] = a - b;
            }
    // lane holding the block with the stage bit clear gets a + b, the other a - b:
    // fma(own, +-1, partner) is p + v or p - v with a single rounding.
    const float s16 = (blk & 1) ? -1.0f : 1.0f;
    const float s32 = (blk & 2) ? -1.0f : 1.0f;
    const float s64 = (blk & 4) ? -1.0f : 1.0f;
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = __builtin_fmaf(v[k], s16, dpp_f<kDppXor1>(v[k]));
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = __builtin_fmaf(v[k], s32, dpp_f<kDppXor2>(v[k]));
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = __builtin_fmaf(v[k], s64, dpp_f<kDppHalfMirror>(v[k]));
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = __builtin_fmaf(v[k], kInvSqrt128, 0.0f);  // +0 for exact zeros
}

__device__ __forceinline__ uint32_t lane_sign16(uint64_t seed_rht, int blk)
{
    const U4 w = philox_seeded(seed_rht, 0, 0, 0, kStreamRht);
    const uint32_t words[4] = {w.x, w.y, w.z, w.w};
    return (words[blk >> 1] >> ((blk & 1) * 16)) & 0xFFFFu;
}

__device__ __forceinline__ float wave_max(float m)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    return m;
}

// block-wide maximum into a global running maximum (non-negative floats order like their
// bit patterns).  The running maximum only grows, so a stale read can only cause a
// redundant atomic.  Must be reached by every thread of the block.
__device__ __forceinline__ void block_max_to_global(float m, uint32_t *amax_bits)
{
    __shared__ float wave_m[4];
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) wave_m[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = fmaxf(fmaxf(wave_m[0], wave_m[1]), fmaxf(wave_m[2], wave_m[3]));
        if (f2u(m) > __atomic_load_n(amax_bits, __ATOMIC_RELAXED)) atomicMax(amax_bits, f2u(m));
    }
}

// ------------------------------------------------------------------ kernels
// one word per thread, `stride` words apart (the abs-max slots of a layer pass in one launch)
__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, int stride) { p[threadIdx.x * stride] = v; }

template <class Loader, bool kRht>
__global__ __launch_bounds__(256) void absmax_kernel(Loader load, int64_t R, int64_t C,
                                                     uint64_t seed_rht, uint32_t *amax_bits)
{
    const int64_t G = C / 16;
    const Lane L = lane_geometry(R, G);
    const uint32_t sign16 = kRht ? lane_sign16(seed_rht, L.blk) : 0u;
    float m = 0.0f;
#pragma unroll 1
    for (int it = 0; it < 4; ++it) {
        const int64_t row = L.quad * 4 + it;
        const bool ok = L.in_range && row < R;
        float v[16];
        if (ok) load(row, L.g * 16, v);
        else {
#pragma unroll
            for (int k = 0; k < 16; ++k) v[k] = 0.0f;
        }
        if (kRht) rht128(v, sign16, L.blk);
#pragma unroll
        for (int k = 0; k < 16; ++k) m = fmaxf(m, fabsf(v[k]));
    }
    block_max_to_global(m, amax_bits);
}

template <class Loader>
__global__ __launch_bounds__(256) void rht_kernel(Loader load, int64_t R, int64_t C,
                                                  uint64_t seed_rht, float *y, uint32_t *amax_bits)
{
    const int64_t G = C / 16;
    const Lane L = lane_geometry(R, G);
    const uint32_t sign16 = lane_sign16(seed_rht, L.blk);
    float m = 0.0f;
#pragma unroll 1
    for (int it = 0; it < 4; ++it) {
        const int64_t row = L.quad * 4 + it;
        const bool ok = L.in_range && row < R;
        float v[16];
        if (ok) load(row, L.g * 16, v);
        else {
#pragma unroll
            for (int k = 0; k < 16; ++k) v[k] = 0.0f;
        }
        rht128(v, sign16, L.blk);
        if (ok) {
            float4 *o = reinterpret_cast<float4 *>(y + row * C + L.g * 16);
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = make_float4(v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]);
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) m = fmaxf(m, fabsf(v[k]));
    }
    if (amax_bits) block_max_to_global(m, amax_bits);
}

template <class Loader, int kMode, bool kRht>
__global__ __launch_bounds__(256) void quantize_kernel(Loader load, int64_t R, int64_t C,
                                                       uint64_t seed_rht, uint64_t seed_sr,
                                                       const float *amax_ptr, uint8_t *codes,
                                                       uint8_t *scales, float *tensor_scale,
                                                       float *tbuf, uint32_t *amax_accum)
{
    const int64_t G = C / 16;
    const Lane L = lane_geometry(R, G);
    // (the heavy pass of the post hoc scheme knows no tensor maximum: tc stays unused there)
    const TensorConsts tc = kMode == QII_MS_EDEN_PH ? TensorConsts{} : tensor_consts(kMode, *amax_ptr);
    if (kMode != QII_MS_EDEN_PH && blockIdx.x == 0 && threadIdx.x == 0) *tensor_scale = tc.x32;
    float m = 0.0f;
    const uint32_t sign16 = kRht ? lane_sign16(seed_rht, L.blk) : 0u;
    uint32_t draw[4] = {0, 0, 0, 0};
    if (kMode == QII_MS_EDEN) {
        const U4 w = philox_seeded(seed_sr, (uint32_t)L.g, (uint32_t)L.quad, 0, kStreamScale);
        draw[0] = w.x >> 12; draw[1] = w.y >> 12; draw[2] = w.z >> 12; draw[3] = w.w >> 12;
    }
#pragma unroll 1
    for (int it = 0; it < 4; ++it) {
        const int64_t row = L.quad * 4 + it;
        const bool ok = L.in_range && row < R;
        float v[16];
        if (ok && !tc.zero) load(row, L.g * 16, v);
        else {
#pragma unroll
            for (int k = 0; k < 16; ++k) v[k] = 0.0f;
        }
        if (kRht) rht128(v, sign16, L.blk);
        // the per-group arithmetic of all schemes (an all-zero group gives scale byte 0, zero codes)
        uint32_t packed[2];
        if (kMode == QII_MS_EDEN_PH) {
            float gmax;
            const float t = posthoc_group16(v, packed, gmax);
            if (ok) {
                *reinterpret_cast<uint2 *>(codes + (row * C + L.g * 16) / 2) = make_uint2(packed[0], packed[1]);
                tbuf[row * G + L.g] = t;
                m = fmaxf(m, gmax);
            }
            continue;
        }
        const uint32_t b = quantize_group16<kMode>(v, tc, it == 0 ? draw[0] : it == 1 ? draw[1] : it == 2 ? draw[2] : draw[3],
                                                   seed_sr, row, L.g, packed);
        if (ok) {
            *reinterpret_cast<uint2 *>(codes + (row * C + L.g * 16) / 2) = make_uint2(packed[0], packed[1]);
            scales[row * G + L.g] = (uint8_t)b;
        }
    }
    if (kMode == QII_MS_EDEN_PH && amax_accum) {   // the running maximum is spread over the slot's words
        m = wave_max(m);
        if ((threadIdx.x & 63) == 0) max_to_global(m, amax_spread_word(amax_accum, blockIdx.x));
    }
}

// Second pass of the post hoc scheme (Sec. 7): scales only.  x^FP32 = max|x| / (s * 256); the
// byte of group (row, g) is SR_E4M3(t / x^FP32) with the 20-bit draw of (seed, row, g), the one
// Algorithm 1 uses.  One thread takes 4 rows x 4 groups: four Philox calls (a call serves the
// four rows of one group) and, when whole, one 16-byte load and one 4-byte store per row.
__global__ __launch_bounds__(256) void posthoc_scales_kernel(const float *__restrict__ tbuf,
                                                             const float *__restrict__ amax_ptr, int n_amax,
                                                             int64_t R, int64_t G, uint64_t seed_sr,
                                                             uint8_t *__restrict__ scales,
                                                             float *__restrict__ tensor_scale, int64_t tiled_ksn)
{
    // the tensor maximum: one word supplied by the caller, or the maximum of the words the heavy
    // pass spread its running maximum over
    __shared__ float amax_s;
    if (threadIdx.x < 64) {
        const float m = wave_max((int)threadIdx.x < n_amax ? amax_ptr[threadIdx.x * kAmaxStrideWords] : 0.0f);
        if (threadIdx.x == 0) amax_s = m;
    }
    __syncthreads();
    const float amax = amax_s;
    const float s = (float)(96.0 / 17.0 / 0.93);
    const float x32 = amax > 0.0f ? amax / (s * 256.0f) : 1.0f;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx == 0) *tensor_scale = x32;
    const int64_t gq = (G + 3) / 4;
    if (idx >= ((R + 3) / 4) * gq) return;
    const int64_t quad = idx / gq, g0 = (idx % gq) * 4;
    uint32_t draw[4][4];   // [group][row]
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const U4 w = philox_seeded(seed_sr, (uint32_t)(g0 + j), (uint32_t)quad, 0, kStreamScale);
        draw[j][0] = w.x >> 12; draw[j][1] = w.y >> 12; draw[j][2] = w.z >> 12; draw[j][3] = w.w >> 12;
    }
    const bool whole = (G % 4 == 0);
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int64_t row = quad * 4 + it;
        if (row >= R) break;
        if (whole) {
            const float4 t = *reinterpret_cast<const float4 *>(tbuf + row * G + g0);
            const uint32_t b = e4m3_sr(t.x / x32, draw[0][it]) | (e4m3_sr(t.y / x32, draw[1][it]) << 8) |
                               (e4m3_sr(t.z / x32, draw[2][it]) << 16) | (e4m3_sr(t.w / x32, draw[3][it]) << 24);
            // tiled_ksn != 0 (G a multiple of 16): the layout the main GEMM kernel reads, 16 bytes per
            // (row, 256 columns), [row / 256][column / 256][row % 256]
            uint8_t *dst = tiled_ksn ? scales + (((row >> 8) * tiled_ksn + (g0 >> 4)) * 256 + (row & 255)) * 16 + (g0 & 15)
                                     : scales + row * G + g0;
            *reinterpret_cast<uint32_t *>(dst) = b;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (g0 + j < G) scales[row * G + g0 + j] = (uint8_t)e4m3_sr(tbuf[row * G + g0 + j] / x32, draw[j][it]);
        }
    }
}

__global__ void dequantize_kernel(const uint8_t *codes, const uint8_t *scales, const float *ts,
                                  int64_t rows, int64_t cols, float *y)
{
    const int64_t G = cols / 16;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // one scale group each
    if (idx >= rows * G) return;
    const uint2 c = *reinterpret_cast<const uint2 *>(codes + idx * 8);
    const float x8 = e4m3_decode(scales[idx]);
    const float x32 = *ts;
    const uint32_t w[2] = {c.x, c.y};
    float4 *o = reinterpret_cast<float4 *>(y + idx * 16);
    float v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const uint32_t code = (w[k >> 3] >> (4 * (k & 7))) & 15u;
        const float m = e2m1_decode_mag(code & 7u) * x8;
        v[k] = u2f(f2u(m * x32) ^ ((code & 8u) << 28));
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = make_float4(v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]);
}

// ------------------------------------------------------------------ dispatch helpers
template <class F>
hipError_t with_loader(const Source &src, F &&f)
{
    if (src.kind == kSrcBF16) {
        if (src.transpose) return f(LoadTransBF16{(const uint16_t *)src.x, src.ld});
        return f(LoadContigBF16{(const uint16_t *)src.x, src.ld});
    }
    if (src.kind == kSrcF32) {
        if (src.transpose) return f(LoadTransF32{(const float *)src.x, src.ld});
        return f(LoadContigF32{(const float *)src.x, src.ld});
    }
    if (src.transpose) return f(LoadTransNVFP4{(const uint8_t *)src.x, src.scales, src.ts, src.ld});
    return f(LoadContigNVFP4{(const uint8_t *)src.x, src.scales, src.ts, src.ld});
}

}  // namespace

hipError_t launch_fill_u32(uint32_t *p, uint32_t v, int count, int stride_words, hipStream_t s)
{
    hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(count), 0, s, p, v, stride_words);
    return hipGetLastError();
}

hipError_t launch_absmax(const Source &src, int64_t R, int64_t C, int rht, uint64_t seed_rht,
                         float *amax, hipStream_t s)
{
    if (R == 0 || C == 0) return hipSuccess;
    if (rows_kernels_apply(src, R, C)) return launch_absmax_rows(src, R, C, rht, seed_rht, amax, s);
    if (cols_kernels_apply(src, R, C)) return launch_absmax_cols(src, R, C, rht, seed_rht, amax, s);
    const dim3 grid((unsigned)grid_for(R, C, 256)), block(256);
    return with_loader(src, [&](auto load) {
        using L = decltype(load);
        if (rht) hipLaunchKernelGGL((absmax_kernel<L, true>), grid, block, 0, s, load, R, C, seed_rht, (uint32_t *)amax);
        else hipLaunchKernelGGL((absmax_kernel<L, false>), grid, block, 0, s, load, R, C, seed_rht, (uint32_t *)amax);
        return hipGetLastError();
    });
}

hipError_t launch_rht(const Source &src, int64_t R, int64_t C, uint64_t seed_rht, float *y,
                      float *amax, hipStream_t s)
{
    if (R == 0 || C == 0) return hipSuccess;
    const dim3 grid((unsigned)grid_for(R, C, 256)), block(256);
    return with_loader(src, [&](auto load) {
        using L = decltype(load);
        hipLaunchKernelGGL((rht_kernel<L>), grid, block, 0, s, load, R, C, seed_rht, y, (uint32_t *)amax);
        return hipGetLastError();
    });
}

hipError_t launch_quantize(const QuantizeArgs &a, hipStream_t s)
{
    if (a.R == 0 || a.C == 0) return hipSuccess;
    if (rows_kernels_apply(a.src, a.R, a.C)) return launch_quantize_rows(a, s);
    if (a.scales_tiled) return hipErrorInvalidValue;   // only the rows kernels write the tiled copy
    if (cols_kernels_apply(a.src, a.R, a.C)) return launch_quantize_cols(a, s);
    const dim3 grid((unsigned)grid_for(a.R, a.C, 256)), block(256);
    return with_loader(a.src, [&](auto load) {
        using L = decltype(load);
#define QII_LAUNCH(MODE, RHT)                                                                     \
    hipLaunchKernelGGL((quantize_kernel<L, MODE, RHT>), grid, block, 0, s, load, a.R, a.C,        \
                       a.seed_rht, a.seed_sr, a.amax, a.codes, a.scales, a.tensor_scale, a.tbuf,  \
                       a.amax_accum)
        if (a.mode == QII_RTN) { if (a.rht) QII_LAUNCH(QII_RTN, true); else QII_LAUNCH(QII_RTN, false); }
        else if (a.mode == QII_RTN_46) { if (a.rht) QII_LAUNCH(QII_RTN_46, true); else QII_LAUNCH(QII_RTN_46, false); }
        else if (a.mode == QII_MS_EDEN_PH) { if (a.rht) QII_LAUNCH(QII_MS_EDEN_PH, true); else QII_LAUNCH(QII_MS_EDEN_PH, false); }
        else if (a.mode == QII_SR) { if (a.rht) QII_LAUNCH(QII_SR, true); else QII_LAUNCH(QII_SR, false); }
        else { if (a.rht) QII_LAUNCH(QII_MS_EDEN, true); else QII_LAUNCH(QII_MS_EDEN, false); }
#undef QII_LAUNCH
        return hipGetLastError();
    });
}

hipError_t launch_posthoc_scales(const float *tbuf, const float *amax, int n_amax, int64_t R, int64_t C,
                                 uint64_t seed_sr, uint8_t *scales, float *tensor_scale, hipStream_t s, bool tiled)
{
    const int64_t G = C / 16, threads = ((R + 3) / 4) * ((G + 3) / 4);
    if (threads == 0) return hipSuccess;
    if (tiled && C % 256 != 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(posthoc_scales_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, tbuf,
                       amax, n_amax, R, G, seed_sr, scales, tensor_scale, tiled ? C / 256 : (int64_t)0);
    return hipGetLastError();
}

hipError_t launch_dequantize(const uint8_t *codes, const uint8_t *scales, const float *ts,
                             int64_t rows, int64_t cols, float *y, hipStream_t s)
{
    const int64_t groups = rows * (cols / 16);
    if (groups == 0) return hipSuccess;
    hipLaunchKernelGGL(dequantize_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, s,
                       codes, scales, ts, rows, cols, y);
    return hipGetLastError();
}

}  // namespace qii
