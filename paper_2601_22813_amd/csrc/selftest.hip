// Device self-test of the hardware conversions and short division sequences that the tuned
// kernels rely on.  The quantizers' arithmetic contract is stated as value-space rules
// (qii_device.h: e2m1_round_mag, e4m3_rtn, e2m1_decode_mag; IEEE binary32 division); the tuned
// kernels replace them by gfx950 instructions and by Newton sequences without range scaling.
// Each sweep below counts the inputs on which such a replacement differs from its rule; a
// compiler or firmware change that alters one of them shows up as a non-zero count.
#include "qii_device.h"
#include "qii_internal.h"
#include "quantize_core.h"

namespace qii {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__global__ void fill_u64_zero_kernel(unsigned long long *p) { p[threadIdx.x] = 0ull; }

__device__ __forceinline__ void count(unsigned long long *slot, unsigned long long n)
{
    // one atomic per wave
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) n += __shfl_xor(n, off);
    if ((threadIdx.x & 63) == 0 && n) atomicAdd(slot, n);
}

// [0] v_cvt_scalef32_pk_fp4_f32 (scale 1) against "round to nearest E2M1, ties to the even code,
// saturating at 6, sign bit kept": every finite binary32, two per conversion.
__global__ __launch_bounds__(256) void sweep_fp4_encode(unsigned long long *counts)
{
    unsigned long long bad = 0;
    const uint64_t n = 1ull << 31, stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint32_t u0 = (uint32_t)(2 * i), u1 = u0 + 1u;
        if ((u0 & 0x7F800000u) == 0x7F800000u) continue;   // infinities and NaNs are outside the contract
        const float a = u2f(u0), b = u2f(u1);
        const uint32_t hw = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, a, b, 1.0f, 0) & 0xFFu;
        const uint32_t ra = e2m1_mag_code(e2m1_round_mag(fabsf(a))) | ((u0 >> 28) & 8u);
        const uint32_t rb = e2m1_mag_code(e2m1_round_mag(fabsf(b))) | ((u1 >> 28) & 8u);
        bad += hw != (ra | (rb << 4));
    }
    count(counts + 0, bad);
}

// [1] v_cvt_pk_fp8_f32 on [0, 448] against e4m3_rtn (nearest, ties to even): every binary32 there.
__global__ __launch_bounds__(256) void sweep_fp8_encode(unsigned long long *counts)
{
    unsigned long long bad = 0;
    const uint64_t n = 0x43E00000ull + 1, stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const float r = u2f((uint32_t)i);
        const uint32_t hw = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(r, 0.0f, 0, false);   // bytes 1..3 must read 0
        bad += hw != e4m3_rtn(r);
    }
    count(counts + 1, bad);
}

// [2] v_cvt_scalef32_pk_f32_fp4 (scale 1) against the exact E2M1 decode: all byte values, all four
//     byte positions.
// [3] the GEMM's dequantization, v_cvt_scalef32_pk_f16_fp4 with scale 2^8 times the scale byte in
//     f16 position (= e4m3 * 2^-8): all 16 codes x 127 scale bytes against e2m1 * e4m3 in f32.
// [6] e4m3_decode (one multiplication by 2^120) against the bit-field definition.
__global__ __launch_bounds__(256) void sweep_decodes(unsigned long long *counts)
{
    unsigned long long bad2 = 0, bad3 = 0, bad6 = 0;
    const uint32_t byte = threadIdx.x;   // 256 threads
    const float lo = e2m1_decode_mag(byte & 7u) * ((byte & 8u) ? -1.0f : 1.0f);
    const float hi = e2m1_decode_mag((byte >> 4) & 7u) * ((byte & 0x80u) ? -1.0f : 1.0f);
    const uint32_t word = byte * 0x01010101u;
#define QII_CHECK_POS(P)                                                                          \
    do {                                                                                          \
        const float2_t c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(word, 1.0f, P);               \
        bad2 += f2u(c[0]) != f2u(lo) || f2u(c[1]) != f2u(hi);                                     \
    } while (0)
    QII_CHECK_POS(0); QII_CHECK_POS(1); QII_CHECK_POS(2); QII_CHECK_POS(3);
#undef QII_CHECK_POS
    for (uint32_t sb = 0; sb < 127; ++sb) {
        const uint32_t s16 = (sb << 7) | (sb << 23);
        const half2_t s2 = __builtin_bit_cast(half2_t, s16);
        const half2_t h = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(word, 256.0f, 0) * s2;
        // the value the contract assigns: e4m3 by its bit fields, times the code
        const int e = (int)(sb >> 3), m = (int)(sb & 7u);
        const float x8 = e == 0 ? ldexpf((float)m * 0.125f, -6) : ldexpf(1.0f + (float)m * 0.125f, e - 7);
        bad3 += (float)h[0] != lo * x8 || (float)h[1] != hi * x8;
        if (byte == 0) bad6 += f2u(e4m3_decode(sb)) != f2u(x8);
    }
    count(counts + 2, bad2);
    count(counts + 3, bad3);
    count(counts + 6, bad6);
}

__device__ __forceinline__ uint32_t mix(uint32_t x)
{
    x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
    return x;
}

// [4] div_by_const (a * RN(1/d) with two residual corrections) and [5] div_safe_range (reciprocal
// estimate, refinement, quotient, two corrections) against IEEE division, on pseudo-random pairs
// whose exponents span the range the kernels use them in: a, d in [2^-40, 2^40] (quotients and
// residuals far from the denormal and overflow ranges).
__global__ __launch_bounds__(256) void sweep_divisions(unsigned long long *counts, uint64_t pairs)
{
    unsigned long long bad4 = 0, bad5 = 0;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < pairs; i += stride) {
        const uint32_t h0 = mix((uint32_t)i * 2u + 1u), h1 = mix((uint32_t)(i >> 11) ^ h0 ^ 0x9E3779B9u);
        const uint32_t h2 = mix(h1 + (uint32_t)i);
        // exponent fields 87..167 (2^-40 .. 2^40), random mantissas
        const float a = u2f(((87u + h2 % 81u) << 23) | (h0 & 0x7FFFFFu));
        const float d = u2f(((87u + (h2 >> 8) % 81u) << 23) | (h1 & 0x7FFFFFu));
        const float q = a / d;
        const float rd = 1.0f / d;
        bad4 += f2u(div_by_const(a, d, rd, true)) != f2u(q);
        bad5 += f2u(div_safe_range(a, d)) != f2u(q);
    }
    count(counts + 4, bad4);
    count(counts + 5, bad5);
}

// [7] the reciprocal of every product e4m3 * x^FP32 (the per-group divisor 1 / (x^FP8 * x^FP32)) by
// div_safe_range against IEEE division, for tensor scales x^FP32 over 80 binades
__global__ __launch_bounds__(256) void sweep_reciprocals(unsigned long long *counts)
{
    unsigned long long bad = 0;
    const uint64_t n = (uint64_t)81 << 23, stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const float x = u2f((uint32_t)(((uint64_t)87 << 23) + i));
        bad += f2u(div_safe_range(1.0f, x)) != f2u(1.0f / x);
    }
    count(counts + 7, bad);
}

}  // namespace

hipError_t launch_selftest_conversions(unsigned long long *counts, hipStream_t s)
{
    hipLaunchKernelGGL(fill_u64_zero_kernel, dim3(1), dim3(8), 0, s, counts);
    hipLaunchKernelGGL(sweep_fp4_encode, dim3(4096), dim3(256), 0, s, counts);
    hipLaunchKernelGGL(sweep_fp8_encode, dim3(4096), dim3(256), 0, s, counts);
    hipLaunchKernelGGL(sweep_decodes, dim3(1), dim3(256), 0, s, counts);
    hipLaunchKernelGGL(sweep_divisions, dim3(4096), dim3(256), 0, s, counts, (uint64_t)1 << 30);
    hipLaunchKernelGGL(sweep_reciprocals, dim3(4096), dim3(256), 0, s, counts);
    return hipGetLastError();
}

}  // namespace qii
