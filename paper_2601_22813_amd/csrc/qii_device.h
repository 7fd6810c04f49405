// Device-side building blocks shared by the libqii kernels (gfx950 only).
//
// Arithmetic contract: every quantizer decision is taken in IEEE binary32 with one
// rounding per written operation (the library is built with -ffp-contract=off and
// fp32 denormals enabled); fused multiply-adds appear only where written as
// __builtin_fmaf.  The bit manipulations below are exact restatements of value-space
// rounding rules; each comment states the rule.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qii {

constexpr uint32_t kStreamRht = 0x52485400u;
constexpr uint32_t kStreamScale = 0x53434C00u;
constexpr uint32_t kStreamElem = 0x454C4D00u;
constexpr uint32_t kStreamDerive = 0x44525600u;

// ---------------------------------------------------------------- Philox4x32-10
struct U4 { uint32_t x, y, z, w; };

__host__ __device__ inline U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return U4{c0, c1, c2, c3};
}

__host__ __device__ inline U4 philox_seeded(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2,
                                            uint32_t c3)
{
    return philox4x32_10(c0, c1, c2, c3, (uint32_t)seed, (uint32_t)(seed >> 32));
}

// ---------------------------------------------------------------- streaming stores
// 16 bytes of codes: written once by a quantizer and not read again by it, so a non-temporal store
// (the lines do not linger dirty in L2, where the next kernel's traffic would have to push them out)
typedef uint32_t qii_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_codes16(uint8_t *dst, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3)
{
    __builtin_nontemporal_store(qii_u32x4{c0, c1, c2, c3}, reinterpret_cast<qii_u32x4 *>(dst));
}

// ---------------------------------------------------------------- bit casts
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }

// ---------------------------------------------------------------- E4M3 (scales, >= 0)
// decode: the byte placed in bits 27..20 of a binary32 is the same number with
// exponent bias 127 instead of 7 (subnormals included), so one exact scaling by 2^120
// gives the value.
__device__ __forceinline__ float e4m3_decode(uint32_t b)
{
    return u2f(b << 20) * 0x1p120f;
}

// round to nearest even, saturating at 448 (byte 0x7E); r >= 0 finite.
// normal range: RNE of the binary32 mantissa to 3 bits = add half-ulp-minus-one plus
// the kept lsb, then truncate; re-bias by (127-7)<<3.  below 2^-6 the grid is uniform
// with step 2^-9, so the byte is rint(r * 2^9).
__device__ __forceinline__ uint32_t e4m3_rtn(float r)
{
    if (r < 0x1p-6f) return (uint32_t)__builtin_rintf(r * 512.0f);
    const uint32_t u = f2u(r);
    const uint32_t v = (u + 0x7FFFFu + ((u >> 20) & 1u)) >> 20;
    const uint32_t b = v - 960u;
    return b > 0x7Eu ? 0x7Eu : b;
}

// stochastic rounding with 20 random bits R: up iff R + d >= 2^20 where d is the
// position of t between its E4M3 neighbours scaled to 2^20.  In the normal range d is
// the 20 discarded mantissa bits; below 2^-6 it is frac(t * 2^9) * 2^20, and comparing
// with its floor is the same test because R is an integer.
__device__ __forceinline__ uint32_t e4m3_sr(float t, uint32_t r20)
{
    if (!(t >= 0x1p-6f)) return ((uint32_t)(t * 0x1p29f) + r20) >> 20;   // (a NaN gives byte 0)
    const uint32_t b = ((f2u(t) + r20) >> 20) - 960u;
    return b > 0x7Eu ? 0x7Eu : b;
}

// ---------------------------------------------------------------- E2M1 (elements)
// Round |q| to the E2M1 grid {0,.5,1,1.5,2,3,4,6} (nearest even, saturating) and
// return the rounded magnitude as a float; the code follows from its bits.
__device__ __forceinline__ float e2m1_round_mag(float a)
{
    if (a < 1.0f) return __builtin_rintf(a * 2.0f) * 0.5f;
    const uint32_t u = f2u(a);
    const float c = u2f((u + 0x1FFFFFu + ((u >> 22) & 1u)) & 0xFFC00000u);
    return c > 6.0f ? 6.0f : c;
}

// magnitude (an exact grid value) -> 3-bit code
__device__ __forceinline__ uint32_t e2m1_mag_code(float c)
{
    return c < 1.0f ? (uint32_t)(c * 2.0f) : (f2u(c) >> 22) - 252u;
}

// stochastic rounding of |q| with 16 random bits R: up iff R + d >= 2^16, d the
// position between the neighbours scaled to 2^16; returns the 3-bit code.
__device__ __forceinline__ uint32_t e2m1_sr_code(float a, uint32_t r16)
{
    if (a < 1.0f) return ((uint32_t)(a * 0x1p17f) + r16) >> 16;
    if (a >= 6.0f) return 7u;
    const uint32_t m = ((f2u(a) + (r16 << 6)) >> 22) - 252u;
    return m > 7u ? 7u : m;
}

__device__ __forceinline__ float e2m1_decode_mag(uint32_t m)
{
    return m < 2u ? (float)m * 0.5f : u2f((m + 252u) << 22);
}

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return u2f(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return u2f(packed & 0xFFFF0000u); }

// f32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    const uint32_t u = f2u(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// ---------------------------------------------------------------- lane exchange (DPP)
// value of the lane whose index differs by `xor 1`, `xor 2`, `xor 7` within a row of 16
template <int kCtrl>
__device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane -> 7 - lane within each 8 (= xor 7)
constexpr int kDppRor8 = 0x128;       // row_ror:8 (= xor 8 within a row of 16)

}  // namespace qii
