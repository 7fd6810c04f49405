// Lane-level building blocks shared by the tuned quantizer kernels: the two register layouts of a
// 128-chunk and what goes with them (rotation, rotation-sign masks, scale-rounding draws, gathering
// of scale bytes).
//
// "Octet" layout (groups along the contiguous dimension): a lane owns one 16-element scale group,
// 8 neighbouring lanes one 128-chunk; lanes 4..7 of an octet hold the 16-blocks in reverse order so
// that the xor-7 lane exchange pairs blocks that differ in index bit 2.
// "Quad" layout (groups along the strided dimension): the 4 lanes of a quad own one 128-chunk of two
// adjacent columns, 32 rows each.
//
// Rotation (Algorithm 1, first loop): butterfly stages over the index bits that live inside a lane
// are plain add/sub; stages that pair lanes use one v_fmac_f32_dpp: own += partner * (+1 | -1).  The
// lane whose block has the stage bit set thereby holds -(a - b) instead of (a - b); the sign flip
// commutes with the later stages and is undone exactly by the sign of the lane's final 2^-3.5
// scaling constant.  Only the sign of exactly-zero intermediates can differ from the plain
// butterfly, and the final fma(v, c, +0) maps every zero result to +0, as the arithmetic contract
// states.
#pragma once
#include "qii_device.h"
#include "quantize_core.h"

namespace qii {

constexpr float kInvSqrt128 = 0x1.6a09e6p-4f;  // binary32 nearest to 2^-3.5

// ---------------------------------------------------------------- octet layout
struct OctetLane {
    int blk;              // 16-block of the chunk owned by this lane
    float s16, s32, s64;  // +-1 multipliers of the three cross-lane stages
    float cfin;           // +-2^-3.5
    uint32_t sign16;      // rotation sign bits of this lane's 16 elements
};

// sign: the 128 rotation signs, bit j of word j / 32
__device__ __forceinline__ OctetLane octet_lane(int lane, const uint32_t sign[4])
{
    OctetLane L;
    const int sub = lane & 7;
    L.blk = (sub & 4) ? (sub ^ 3) : sub;
    L.s16 = (L.blk & 1) ? -1.0f : 1.0f;
    L.s32 = (L.blk & 2) ? -1.0f : 1.0f;
    L.s64 = (L.blk & 4) ? -1.0f : 1.0f;
    L.cfin = (__builtin_popcount(L.blk) & 1) ? -kInvSqrt128 : kInvSqrt128;
    const uint32_t w = (L.blk >> 1) == 0 ? sign[0] : (L.blk >> 1) == 1 ? sign[1] : (L.blk >> 1) == 2 ? sign[2] : sign[3];
    L.sign16 = (w >> ((L.blk & 1) * 16)) & 0xFFFFu;
    return L;
}

// one cross-lane butterfly stage on all 16 registers: v[k] += partner(v[k]) * s
#define QII_DPP_STAGE(CTRL)                                                                       \
    asm volatile("s_nop 1\n"                                                                      \
                 "v_fmac_f32_dpp %0, %0, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"               \
                 "v_fmac_f32_dpp %1, %1, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"               \
                 "v_fmac_f32_dpp %2, %2, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"               \
                 "v_fmac_f32_dpp %3, %3, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"               \
                 "v_fmac_f32_dpp %4, %4, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"               \
                 "v_fmac_f32_dpp %5, %5, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"               \
                 "v_fmac_f32_dpp %6, %6, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"               \
                 "v_fmac_f32_dpp %7, %7, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"               \
                 "v_fmac_f32_dpp %8, %8, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"               \
                 "v_fmac_f32_dpp %9, %9, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"               \
                 "v_fmac_f32_dpp %10, %10, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"             \
                 "v_fmac_f32_dpp %11, %11, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"             \
                 "v_fmac_f32_dpp %12, %12, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"             \
                 "v_fmac_f32_dpp %13, %13, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"             \
                 "v_fmac_f32_dpp %14, %14, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"             \
                 "v_fmac_f32_dpp %15, %15, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"             \
                 : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]),        \
                   "+v"(v[6]), "+v"(v[7]), "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]),      \
                   "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15])                             \
                 : "v"(s))

__device__ __forceinline__ void dpp_stage_xor1(float v[16], float s) { QII_DPP_STAGE("quad_perm:[1,0,3,2]"); }
__device__ __forceinline__ void dpp_stage_xor2(float v[16], float s) { QII_DPP_STAGE("quad_perm:[2,3,0,1]"); }
__device__ __forceinline__ void dpp_stage_xor7(float v[16], float s) { QII_DPP_STAGE("row_half_mirror"); }

// stages over index bits 0..3 (in-lane) then 4..6 (cross-lane), then the scaling
// kScale = false leaves out the final scaling: for the abs-max pass, where rounding is monotone
// and symmetric, max |fma(v, c, 0)| = fma(max |v|, |c|, 0), so one scaling of the maximum does
template <bool kScale = true>
__device__ __forceinline__ void rht128_lane(float v[16], const OctetLane &L)
{
#pragma unroll
    for (int len = 1; len < 16; len <<= 1)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if ((i & len) == 0) {
                const float a = v[i], b = v[i + len];
                v[i] = a + b;
                v[i + len] = a - b;
            }
    dpp_stage_xor1(v, L.s16);
    dpp_stage_xor2(v, L.s32);
    dpp_stage_xor7(v, L.s64);
    if (kScale)
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = __builtin_fmaf(v[k], L.cfin, 0.0f);  // +0 for exact zeros
}

// The 8 scale bytes of an octet's chunk are consecutive in memory; single-byte stores are
// slow, so they are gathered into the lane holding block 0, which stores them as one 8-byte
// word: each lane shifts its byte to position (blk mod 4), two DPP ORs merge a quad, and the
// half-mirror brings the upper quad's word (blocks 4..7 sit in lane 7 - blk) to the lower one.
__device__ __forceinline__ uint2 gather_scale_bytes(uint32_t b, int blk)
{
    uint32_t t = b << (8 * (blk & 3));
    t |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)t, kDppXor1, 0xF, 0xF, true);
    t |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)t, kDppXor2, 0xF, 0xF, true);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)t, kDppHalfMirror, 0xF, 0xF, true);
    return make_uint2(t, hi);
}

// sign masks of a lane's 16 elements, positioned for packed bf16 words (two elements per word) or
// for f32 words
template <bool kBf16>
__device__ __forceinline__ void make_masks(uint32_t sign16, uint32_t mask[kBf16 ? 8 : 16])
{
    if (kBf16) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            mask[i] = (((sign16 >> (2 * i)) & 1u) << 15) | (((sign16 >> (2 * i + 1)) & 1u) << 31);
    } else {
#pragma unroll
        for (int k = 0; k < 16; ++k) mask[k] = ((sign16 >> k) & 1u) << 31;
    }
}

// 16 bf16 (8 words) -> f32 with the rotation signs applied
template <bool kRht>
__device__ __forceinline__ void unpack_bf16x16(const uint32_t w[8], float v[16], const uint32_t mask[8])
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t s = kRht ? (w[i] ^ mask[i]) : w[i];
        v[2 * i] = bf16_lo(s);
        v[2 * i + 1] = bf16_hi(s);
    }
}

// ---------------------------------------------------------------- quad layout
// one cross-lane butterfly stage on 16 registers: v[k] += partner(v[k]) * s
#define QII_PAIR_STAGE(NAME, CTRL)                                                                \
    __device__ __forceinline__ void NAME(float *v, float s)                                       \
    {                                                                                             \
        asm volatile("s_nop 1\n"                                                                  \
                     "v_fmac_f32_dpp %0, %0, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"           \
                     "v_fmac_f32_dpp %1, %1, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"           \
                     "v_fmac_f32_dpp %2, %2, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"           \
                     "v_fmac_f32_dpp %3, %3, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"           \
                     "v_fmac_f32_dpp %4, %4, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"           \
                     "v_fmac_f32_dpp %5, %5, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"           \
                     "v_fmac_f32_dpp %6, %6, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"           \
                     "v_fmac_f32_dpp %7, %7, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"           \
                     "v_fmac_f32_dpp %8, %8, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"           \
                     "v_fmac_f32_dpp %9, %9, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"           \
                     "v_fmac_f32_dpp %10, %10, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"         \
                     "v_fmac_f32_dpp %11, %11, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"         \
                     "v_fmac_f32_dpp %12, %12, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"         \
                     "v_fmac_f32_dpp %13, %13, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"         \
                     "v_fmac_f32_dpp %14, %14, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"         \
                     "v_fmac_f32_dpp %15, %15, %16 " CTRL " row_mask:0xf bank_mask:0xf\n"         \
                     : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]),    \
                       "+v"(v[6]), "+v"(v[7]), "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]),  \
                       "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15])                         \
                     : "v"(s));                                                                   \
    }
QII_PAIR_STAGE(dpp_xor1_stage16, "quad_perm:[1,0,3,2]")
QII_PAIR_STAGE(dpp_xor2_stage16, "quad_perm:[2,3,0,1]")
#undef QII_PAIR_STAGE

// y = H v / sqrt(128) over the 128 values of one column held by a lane quad: stages over
// index bits 0..4 in-lane, bits 5 and 6 across the quad, then the scaling (kScale = false: left
// to the caller; the abs-max pass scales its maximum once, which is the same number because
// rounding is monotone and symmetric)
template <bool kScale = true>
__device__ __forceinline__ void fwht128_quad(float v[32], int q)
{
#pragma unroll
    for (int len = 1; len < 32; len <<= 1)
#pragma unroll
        for (int i = 0; i < 32; ++i)
            if ((i & len) == 0) {
                const float x = v[i], y = v[i + len];
                v[i] = x + y;
                v[i + len] = x - y;
            }
    const float s5 = (q & 1) ? -1.0f : 1.0f, s6 = (q & 2) ? -1.0f : 1.0f;
    dpp_xor1_stage16(v, s5);
    dpp_xor1_stage16(v + 16, s5);
    dpp_xor2_stage16(v, s6);
    dpp_xor2_stage16(v + 16, s6);
    const float c = (q == 1 || q == 2) ? -kInvSqrt128 : kInvSqrt128;
    if (kScale)
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = __builtin_fmaf(v[i], c, 0.0f);  // +0 for exact zeros
}

// draws of this lane's groups: draw[e][h] for column j0+e, column group 8*chunk + 2q + h.
// Lane o of an octet (the 8 lanes that own columns 4j..4j+3) computes the call of column
// group 8*chunk + o; a lane then takes the words of its two columns from its two calls.
__device__ __forceinline__ void octet_draws(uint32_t draw[2][2], uint64_t seed_sr, int64_t chunk, int64_t j0, int q)
{
    const int lane = threadIdx.x & 63, o = lane & 7, upper = (lane >> 2) & 1;   // upper: columns 2,3 of the four
    const U4 w = philox_seeded(seed_sr, (uint32_t)(chunk * 8 + o), (uint32_t)(j0 >> 2), 0, kStreamScale);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int src = ((lane & ~7) | (2 * q + h)) * 4;
        const uint32_t x = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)w.x);
        const uint32_t y = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)w.y);
        const uint32_t z = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)w.z);
        const uint32_t t = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)w.w);
        draw[0][h] = (upper ? z : x) >> 12;
        draw[1][h] = (upper ? t : y) >> 12;
    }
}

// the 8 scale bytes of a (column, chunk): lane q contributes bytes 2q, 2q+1; lane 0 of the quad
// ends up with all of them
__device__ __forceinline__ uint2 gather_quad_scales(uint32_t two_bytes, int q)
{
    uint32_t t = two_bytes << (16 * (q & 1));
    t |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)t, kDppXor1, 0xF, 0xF, true);
    const uint32_t other = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)t, kDppXor2, 0xF, 0xF, true);
    return make_uint2(t, other);
}

}  // namespace qii
