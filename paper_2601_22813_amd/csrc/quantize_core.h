// Per-group arithmetic of the NVFP4 quantizers, shared by the tuned kernels.
// One call quantizes the 16 (already rotated) values of one scale group held by one lane.
//
// The conversions use gfx950's converters where their results were checked, exhaustively
// over all binary32 inputs, to equal the value-space rules of the arithmetic contract:
//   v_cvt_scalef32_pk_fp4_f32 (scale 1.0) = round to nearest E2M1, ties to the even code,
//       saturating at 6, sign kept (also on results that round to zero);
//   v_cvt_pk_fp8_f32 on [0, 448]          = round to nearest E4M3, ties to even;
//   v_cvt_scalef32_pk_f32_fp4             = exact E2M1 decode.
#pragma once
#include "../../include/qii.h"
#include "qii_device.h"

namespace qii {

typedef float float2_t __attribute__((ext_vector_type(2)));

// a register whose content does not matter (no instruction is spent on initialising it)
__device__ __forceinline__ void undefined_word(uint32_t &w) { asm volatile("" : "=v"(w)); }

struct TensorConsts {
    float x32;   // x^FP32 = amax / (s * cap)
    float d;     // x^FP32 * s, the divisor of the group-scale equation
    float rd;    // 1 / d, correctly rounded
    float d4;    // x^FP32 * 4 and its reciprocal: the second candidate of the 4/6 choice
    float rd4;
    bool zero;   // amax == 0: emit zeros
    bool fast;   // magnitudes far from the denormal range: the short division sequences
                 // below equal IEEE division bit for bit
};

__device__ __forceinline__ TensorConsts tensor_consts(int mode, float amax)
{
    float s, cap;
    if (mode == QII_RTN) { s = 6.0f; cap = 448.0f; }
    else if (mode == QII_RTN_46) { s = 6.0f; cap = 256.0f; }
    else if (mode == QII_SR) { s = (float)(96.0 / 17.0); cap = 448.0f; }
    else { s = (float)(96.0 / 17.0 / 0.93); cap = 256.0f; }
    TensorConsts tc;
    tc.zero = !(amax > 0.0f);
    tc.x32 = tc.zero ? 1.0f : amax / (s * cap);
    tc.d = tc.x32 * s;
    tc.rd = 1.0f / tc.d;
    tc.d4 = tc.x32 * 4.0f;
    tc.rd4 = 1.0f / tc.d4;
    tc.fast = amax > 0x1p-20f && amax < 0x1p20f;
    return tc;
}

// a / d rounded to nearest: with rd = RN(1/d), two residual corrections of a * rd give the
// correctly rounded quotient when nothing under- or overflows (the same refinement a
// compiler-generated IEEE division ends with); otherwise fall back to the division.
__device__ __forceinline__ float div_by_const(float a, float d, float rd, bool fast)
{
    if (!fast) return a / d;
    const float q0 = a * rd;
    const float e0 = __builtin_fmaf(-d, q0, a);
    const float q1 = __builtin_fmaf(e0, rd, q0);
    const float e1 = __builtin_fmaf(-d, q1, a);
    return __builtin_fmaf(e1, rd, q1);
}

// Which division forms a caller uses: kFast = 1 the short sequences (the caller has branched on
// tc.fast once, outside its loops), 0 the full IEEE divisions, -1 decide here from tc.fast.
template <int kFast>
__device__ __forceinline__ bool use_fast(const TensorConsts &tc)
{
    return kFast < 0 ? tc.fast : kFast != 0;
}

template <int kFast = -1>
__device__ __forceinline__ float div_by_tensor_const(float a, const TensorConsts &tc)
{
    return div_by_const(a, tc.d, tc.rd, use_fast<kFast>(tc));
}

// a / b rounded to nearest for operands far from the denormal and overflow ranges: the
// Newton-Raphson sequence of a compiler-generated IEEE binary32 division (reciprocal
// estimate, one refinement of it, quotient, two residual corrections) without the operand
// pre-scaling and the special-case fix-up, which are identities in that range.
__device__ __forceinline__ float div_safe_range(float a, float b)
{
    const float r0 = __builtin_amdgcn_rcpf(b);
    const float f0 = __builtin_fmaf(-b, r0, 1.0f);
    const float r1 = __builtin_fmaf(f0, r0, r0);
    const float m = a * r1;
    const float f2 = __builtin_fmaf(-b, m, a);
    const float f3 = __builtin_fmaf(f2, r1, m);
    const float f4 = __builtin_fmaf(-b, f3, a);
    return __builtin_fmaf(f4, r1, f3);
}

template <int kFast = -1>
__device__ __forceinline__ float div_ieee(float a, float b, const TensorConsts &tc)
{
    return use_fast<kFast>(tc) ? div_safe_range(a, b) : a / b;
}

__device__ __forceinline__ float group_absmax(const float y[16])
{
    float m0 = fmaxf(fabsf(y[0]), fabsf(y[1])), m1 = fmaxf(fabsf(y[2]), fabsf(y[3]));
#pragma unroll
    for (int k = 4; k < 16; k += 4) {
        m0 = fmaxf(fmaxf(m0, fabsf(y[k])), fabsf(y[k + 1]));
        m1 = fmaxf(fmaxf(m1, fabsf(y[k + 2])), fabsf(y[k + 3]));
    }
    return fmaxf(m0, m1);
}

// The reciprocal 1 / (x^FP8 * x^FP32) only depends on the scale byte once the tensor scale is
// known: a block fills a 128-entry table in LDS with full IEEE divisions at its start and every
// group then reads its reciprocal instead of decoding the byte and dividing.  Entry 0 is unused.
__device__ __forceinline__ void fill_inv_table(float *inv_tab, const TensorConsts &tc)
{
    for (uint32_t b = threadIdx.x; b < 128u; b += blockDim.x) {
        const float p = e4m3_decode(b) * tc.x32;
        inv_tab[b] = b == 0u ? 0.0f : 1.0f / p;
    }
    __syncthreads();
}

// (without a table a zero byte takes a stand-in divisor; its results are dropped by the caller)
template <int kFast = -1, bool kTab = false>
__device__ __forceinline__ float group_inv(uint32_t b, const TensorConsts &tc, const float *inv_tab)
{
    if (kTab) return inv_tab[b];
    return div_ieee<kFast>(1.0f, b == 0u ? 1.0f : e4m3_decode(b) * tc.x32, tc);
}

// e4m3_sr for the lanes with `use` set, with the rare range below 2^-6 behind a wave-uniform
// branch.  A NaN (0/0 when both dot products of a group underflow, far outside the value range
// of real tensors) takes the small branch and gives byte 0, as "not greater than zero" does in
// the value-space rule.  Lanes without `use` get an unspecified byte.
__device__ __forceinline__ uint32_t e4m3_sr_wave(float t, uint32_t r20, bool use = true)
{
    const uint32_t bn = ((f2u(t) + r20) >> 20) - 960u;
    uint32_t b = bn > 0x7Eu ? 0x7Eu : bn;
    const bool small = use && !(t >= 0x1p-6f);
    if (__builtin_amdgcn_ballot_w64(small) != 0ull) {
        asm volatile("" : "+v"(t));   // keeps the arithmetic of the rare case inside its branch
        const uint32_t bs = ((uint32_t)(t * 0x1p29f) + r20) >> 20;
        b = small ? bs : b;
    }
    return b;
}

// One candidate of the 4/6 choice (Sec. 4.1): round the group to nearest with the scale byte
// RTN_FP8(r), r = group maximum / (x^FP32 * level).  Fills packed[2]; err = sum of
// (x_i - c_i * (x^FP8 * x^FP32))^2, each difference one fused multiply-add, summed as a fused
// multiply-add chain in index order.  A scale byte of 0 gives zero codes and err = <x, x>.
template <int kFast = -1, bool kTab = false>
__device__ __forceinline__ uint32_t rtn_candidate(const float y[16], float r, const TensorConsts &tc,
                                                  const float *inv_tab, uint32_t packed[2], float &err)
{
    const uint32_t b = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(fminf(r, 448.0f), 0.0f, 0, false) & 0xFFu;
    // with b == 0 the arithmetic below runs on a stand-in scale and its results are dropped
    const float p = b == 0u ? 1.0f : e4m3_decode(b) * tc.x32;
    const float inv = kTab ? inv_tab[b] : div_ieee<kFast>(1.0f, p, tc);   // (entry 0: results are dropped)
    packed[0] = 0u;
    packed[1] = 0u;
#define QII_ENC(H, I)                                                                             \
    packed[H] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed[H], y[8 * H + 2 * I] * inv,       \
                                                         y[8 * H + 2 * I + 1] * inv, 1.0f, I)
    QII_ENC(0, 0); QII_ENC(0, 1); QII_ENC(0, 2); QII_ENC(0, 3);
    QII_ENC(1, 0); QII_ENC(1, 1); QII_ENC(1, 2); QII_ENC(1, 3);
#undef QII_ENC
    if (b == 0u) { packed[0] = 0u; packed[1] = 0u; }
    float e = 0.0f;
#define QII_ERR(H, I)                                                                             \
    do {                                                                                          \
        const float2_t c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(packed[H], 1.0f, I);          \
        const float d0 = __builtin_fmaf(-c[0], p, y[8 * H + 2 * I]);                              \
        e = __builtin_fmaf(d0, d0, e);                                                            \
        const float d1 = __builtin_fmaf(-c[1], p, y[8 * H + 2 * I + 1]);                          \
        e = __builtin_fmaf(d1, d1, e);                                                            \
    } while (0)
    QII_ERR(0, 0); QII_ERR(0, 1); QII_ERR(0, 2); QII_ERR(0, 3);
    QII_ERR(1, 0); QII_ERR(1, 1); QII_ERR(1, 2); QII_ERR(1, 3);
#undef QII_ERR
    err = e;
    return b;
}

// Internal mode number of MS-EDEN with post hoc range alignment (QII_MS_EDEN_PH of the C ABI).
// E8M3 (Sec. 7): a non-negative binary32 rounded to three mantissa bits, nearest even.
__device__ __forceinline__ float e8m3_rtn(float u)
{
    const uint32_t b = f2u(u);
    return u2f((b + 0x7FFFFu + ((b >> 20) & 1u)) & 0xFFF00000u);
}

// Heavy pass of the post hoc scheme (Sec. 7) for one group; needs no tensor maximum.
// Pseudo-scale p = RTN_E8M3(gmax / s), codes RTN_FP4(y_i / p), returns the corrected
// pseudo-scale t = <y,y> / <y, codes> (p cancels; t = p when the denominator is not positive,
// 0 for an all-zero group).  The three divisions take the short exact sequences when every
// lane of the wave has its group maximum in (2^-20, 2^20) or zero (then all operands are far
// from the denormal and overflow ranges), else full IEEE divisions.  Call with all lanes active.
__device__ __forceinline__ float posthoc_group16(const float y[16], uint32_t packed[2], float &gmax)
{
    constexpr float kS = (float)(96.0 / 17.0 / 0.93), kRs = (float)(1.0 / (double)kS);
    packed[0] = 0u;
    packed[1] = 0u;
    gmax = group_absmax(y);
    const bool odd = !(gmax == 0.0f || (gmax > 0x1p-20f && gmax < 0x1p20f));
    const bool fast = __builtin_amdgcn_ballot_w64(odd) == 0ull;   // wave-uniform
    const float p = e8m3_rtn(div_by_const(gmax, kS, kRs, fast));
    // an all-zero group (or a maximum that rounds to nothing) runs the arithmetic below on a
    // stand-in pseudo-scale and drops the results: no divergent branch
    const bool live = p > 0.0f;
    const float ps = live ? p : 1.0f;
    const float inv = fast ? div_safe_range(1.0f, ps) : 1.0f / ps;
#define QII_ENC(H, I)                                                                             \
    packed[H] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed[H], y[8 * H + 2 * I] * inv,       \
                                                         y[8 * H + 2 * I + 1] * inv, 1.0f, I)
    QII_ENC(0, 0); QII_ENC(0, 1); QII_ENC(0, 2); QII_ENC(0, 3);
    QII_ENC(1, 0); QII_ENC(1, 1); QII_ENC(1, 2); QII_ENC(1, 3);
#undef QII_ENC
    float num = 0.0f, den = 0.0f;
#define QII_DOT(H, I)                                                                             \
    do {                                                                                          \
        const float2_t c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(packed[H], 1.0f, I);          \
        const float y0 = y[8 * H + 2 * I], y1 = y[8 * H + 2 * I + 1];                             \
        num = __builtin_fmaf(y0, y0, num);                                                        \
        den = __builtin_fmaf(y0, c[0], den);                                                      \
        num = __builtin_fmaf(y1, y1, num);                                                        \
        den = __builtin_fmaf(y1, c[1], den);                                                      \
    } while (0)
    QII_DOT(0, 0); QII_DOT(0, 1); QII_DOT(0, 2); QII_DOT(0, 3);
    QII_DOT(1, 0); QII_DOT(1, 1); QII_DOT(1, 2); QII_DOT(1, 3);
#undef QII_DOT
    const bool pos = den > 0.0f;
    const float dd = pos ? den : 1.0f;
    const float t = fast ? div_safe_range(num, dd) : num / dd;
    packed[0] = live ? packed[0] : 0u;
    packed[1] = live ? packed[1] : 0u;
    return live ? (pos ? t : p) : 0.0f;
}

// a wave's maximum into the global running maximum (non-negative floats order like their bits)
__device__ __forceinline__ float wave_max(float m)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    return m;
}

// The heavy pass of the post hoc scheme folds block maxima into a running maximum.  A device-wide
// atomic on one address costs about 4 ns however many compute units issue it (the eight L2 caches
// of the chip are not coherent with one another, so such atomics are resolved on the memory side
// one after the other): thousands of blocks updating one word took 18 us.  The running maximum
// is therefore kept as kAmaxSpread words, 256 bytes apart (different memory channels), that blocks
// pick by their index; the scales pass takes the maximum of the words.
constexpr uint32_t kAmaxSpread = 64;
constexpr uint32_t kAmaxStrideWords = 64;
constexpr size_t kAmaxRegionBytes = (size_t)kAmaxSpread * kAmaxStrideWords * 4;   // 16 KiB

__device__ __forceinline__ uint32_t *amax_spread_word(uint32_t *region, uint32_t block_index)
{
    return region + (block_index & (kAmaxSpread - 1)) * kAmaxStrideWords;
}

__device__ __forceinline__ void max_to_global(float m, uint32_t *amax_bits)
{
    // the running maximum only grows, so a stale read can only cause a redundant atomic
    if (f2u(m) > __atomic_load_n(amax_bits, __ATOMIC_RELAXED)) atomicMax(amax_bits, f2u(m));
}

// Quantize one group.  y: rotated values; draw20: the 20 scale-rounding bits of this group
// (MS-EDEN); (seed_sr, row, g): identify the element draws (SR).  Returns the scale byte and
// fills packed[2] with the 16 codes (element 2j in the low nibble of byte j).
// kTab: the caller passes the block's reciprocal table (inv_tab is then not null)
template <int kMode, int kFast = -1, bool kTab = false>
__device__ __forceinline__ uint32_t quantize_group16(const float y[16], const TensorConsts &tc,
                                                     uint32_t draw20, uint64_t seed_sr, int64_t row,
                                                     int64_t g, uint32_t packed[2],
                                                     const float *inv_tab = nullptr)
{
    if (kMode == QII_RTN_46) {
        // both candidates, then the one with the lower error; the mapping to 6 wins ties
        const float gmax = group_absmax(y);
        uint32_t p6[2], p4[2];
        float e6, e4;
        const bool fast = use_fast<kFast>(tc);
        const uint32_t b6 = rtn_candidate<kFast, kTab>(y, div_by_const(gmax, tc.d, tc.rd, fast), tc, inv_tab, p6, e6);
        const uint32_t b4 = rtn_candidate<kFast, kTab>(y, div_by_const(gmax, tc.d4, tc.rd4, fast), tc, inv_tab, p4, e4);
        const bool use4 = e4 < e6;
        packed[0] = use4 ? p4[0] : p6[0];
        packed[1] = use4 ? p4[1] : p6[1];
        return use4 ? b4 : b6;
    }
    // x^FP8_g = RTN_FP8( max_g |x| / (x^FP32 * s) ), saturating at 448 (the quotient is >= 0; the
    // conversion writes bytes 0 and 1 of a zero word: byte 1 is the code of 0.0)
    const float r = div_by_tensor_const<kFast>(group_absmax(y), tc);
    const uint32_t b_rtn = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(__builtin_amdgcn_fmed3f(r, 0.0f, 448.0f), 0.0f, 0, false);
    if (kMode == QII_SR) {
        packed[0] = 0u;
        packed[1] = 0u;
        if (b_rtn == 0u) return 0u;
        const float inv = group_inv<kFast, kTab>(b_rtn, tc, inv_tab);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const U4 w = philox_seeded(seed_sr, (uint32_t)(g * 2 + h), (uint32_t)row, 0, kStreamElem);
            const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float q = y[h * 8 + j] * inv;
                const uint32_t r16 = (j & 1) ? (ww[j >> 1] >> 16) : (ww[j >> 1] & 0xFFFFu);
                const uint32_t code = e2m1_sr_code(fabsf(q), r16) | ((f2u(q) >> 28) & 8u);
                packed[h] |= code << (4 * j);
            }
        }
        return b_rtn;
    }
    // A group whose scale byte is 0 has zero codes.  It runs the arithmetic below like any other
    // group (reciprocal table entry 0 is 0) and its results are dropped at the end: no divergent
    // branch in the common path.
    const float inv = group_inv<kFast, kTab>(b_rtn, tc, inv_tab);
    // x^FP4_i = RTN_FP4( x_i * inv ): two elements per conversion, packed in place (the four
    // conversions of a word write all of its bytes, so it needs no initial value)
    undefined_word(packed[0]);
    undefined_word(packed[1]);
#define QII_ENC(H, I)                                                                             \
    packed[H] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed[H], y[8 * H + 2 * I] * inv,       \
                                                         y[8 * H + 2 * I + 1] * inv, 1.0f, I)
    QII_ENC(0, 0); QII_ENC(0, 1); QII_ENC(0, 2); QII_ENC(0, 3);
    QII_ENC(1, 0); QII_ENC(1, 1); QII_ENC(1, 2); QII_ENC(1, 3);
#undef QII_ENC
    uint32_t b = b_rtn;
    if (kMode == QII_MS_EDEN) {
        // S_g * x^FP8_g = <x,x> / (<x, x^FP4> * x^FP32); dot products as fma chains in index order
        float num = 0.0f, den = 0.0f;
#define QII_DOT(H, I)                                                                             \
    do {                                                                                          \
        const float2_t c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(packed[H], 1.0f, I);          \
        const float y0 = y[8 * H + 2 * I], y1 = y[8 * H + 2 * I + 1];                             \
        num = __builtin_fmaf(y0, y0, num);                                                        \
        den = __builtin_fmaf(y0, c[0], den);                                                      \
        num = __builtin_fmaf(y1, y1, num);                                                        \
        den = __builtin_fmaf(y1, c[1], den);                                                      \
    } while (0)
        QII_DOT(0, 0); QII_DOT(0, 1); QII_DOT(0, 2); QII_DOT(0, 3);
        QII_DOT(1, 0); QII_DOT(1, 1); QII_DOT(1, 2); QII_DOT(1, 3);
#undef QII_DOT
        // the corrected scale replaces the byte where the group is live and the denominator positive
        const bool use = b_rtn != 0u && den > 0.0f;
        const uint32_t bs = e4m3_sr_wave(div_ieee<kFast>(num, (use ? den : 1.0f) * tc.x32, tc), draw20, use);
        b = use ? bs : b_rtn;
    }
    packed[0] = b_rtn != 0u ? packed[0] : 0u;
    packed[1] = b_rtn != 0u ? packed[1] : 0u;
    return b;
}

}  // namespace qii
