// Tuned quantizer / abs-max kernels for dense row-major sources quantized along their rows
// (the contiguous case: Q(E), and the forward-pass RTN of X and W).
//
// Layout of the work: a lane owns one 16-element scale group, 8 lanes one 128-chunk, a wave
// 8 consecutive chunks of a row (1024 elements, 2 KiB of bf16), a block 4 waves: side by
// side on wide tensors, or, when a row needs fewer than 4 waves, 2 or 4 row quads at once.
// blockIdx.y selects the column range, blockIdx.x strides over row quads, so the
// per-thread set-up (lane constants, sign masks) is paid once for many groups.  The four
// rows of a quad are loaded together (32 B per lane and row) before any arithmetic.
//
// Rotation: butterfly stages over index bits 0..3 are plain in-lane add/sub; stages over
// bits 4..6 pair lanes (xor 1, xor 2, xor 7 via DPP) with a single v_fmac_f32_dpp:
// own += partner * (+1 | -1).  The lane whose block has the stage bit set thereby holds
// -(a - b) instead of (a - b); the sign flip commutes with the later stages and is
// undone exactly by the sign of the lane's final 2^-3.5 scaling constant.  Only the sign
// of exactly-zero intermediates can differ from the plain butterfly, and the final
// fma(v, c, +0) maps every zero result to +0, as the arithmetic contract states.
#include "qii_device.h"
#include "qii_internal.h"
#include "quantize_core.h"

namespace qii {
namespace {

constexpr float kInvSqrt128 = 0x1.6a09e6p-4f;  // binary32 nearest to 2^-3.5

struct RowsArgs {
    const void *x;
    int64_t ld;          // elements
    int64_t R, C;
    uint32_t sign[4];    // the 128 rotation signs (host-side Philox), bit j of word j/32
    uint64_t seed_sr;
    const float *amax;
    uint8_t *codes;
    uint8_t *scales;
    float *tensor_scale;
    uint32_t *amax_out;  // abs-max kernel, and the heavy pass of the post hoc scheme (nullable there)
    float *tbuf;         // post hoc scheme: corrected pseudo-scales [R][C/16]
    int wpr;             // waves of a block that sit side by side on a row: 1, 2 or 4
};

struct LaneSetup {
    int blk;              // 16-block of the chunk owned by this lane
    int64_t first, step;  // this wave's first row quad and its stride (quads)
    int64_t g;            // scale group within the row
    bool col_ok;
    float s16, s32, s64;  // +-1 multipliers of the three cross-lane stages
    float cfin;           // +-2^-3.5
    uint32_t sign16;      // rotation sign bits of this lane's 16 elements
};

__device__ __forceinline__ LaneSetup lane_setup(const RowsArgs &a, int64_t G)
{
    LaneSetup L;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane & 7;
    L.blk = (sub & 4) ? (sub ^ 3) : sub;
    // wpr waves side by side, 4 / wpr row quads per block
    const int wcol = wave & (a.wpr - 1), wq = wave / a.wpr, qpb = 4 / a.wpr;
    L.first = (int64_t)blockIdx.x * qpb + wq;
    L.step = (int64_t)gridDim.x * qpb;
    const int64_t chunk = ((int64_t)blockIdx.y * a.wpr + wcol) * 8 + (lane >> 3);
    L.g = chunk * 8 + L.blk;
    L.col_ok = L.g < G;
    L.s16 = (L.blk & 1) ? -1.0f : 1.0f;
    L.s32 = (L.blk & 2) ? -1.0f : 1.0f;
    L.s64 = (L.blk & 4) ? -1.0f : 1.0f;
    L.cfin = (__builtin_popcount(L.blk) & 1) ? -kInvSqrt128 : kInvSqrt128;
    const uint32_t w = (L.blk >> 1) == 0 ? a.sign[0] : (L.blk >> 1) == 1 ? a.sign[1] : (L.blk >> 1) == 2 ? a.sign[2] : a.sign[3];
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
__device__ __forceinline__ void rht128_lane(float v[16], const LaneSetup &L)
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

// raw row data of one lane: 16 elements
template <bool kBf16>
struct Raw {
    uint4 q[kBf16 ? 2 : 4];
};

// rows and groups are clamped into the tensor, so every lane always loads from a valid
// address and no exec-masked branch is needed; out-of-range lanes simply do not store
template <bool kBf16>
__device__ __forceinline__ void load_raw(Raw<kBf16> &r, const RowsArgs &a, int64_t row, int64_t g)
{
    constexpr int n = kBf16 ? 2 : 4;
    const uint4 *p = kBf16 ? reinterpret_cast<const uint4 *>((const uint16_t *)a.x + row * a.ld + g * 16)
                           : reinterpret_cast<const uint4 *>((const float *)a.x + row * a.ld + g * 16);
#pragma unroll
    for (int i = 0; i < n; ++i) r.q[i] = p[i];
}

template <bool kBf16>
__device__ __forceinline__ void load_quad(Raw<kBf16> raw[4], const RowsArgs &a, int64_t quad, int64_t g)
{
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        int64_t row = quad * 4 + it;
        row = row < a.R ? row : a.R - 1;
        load_raw<kBf16>(raw[it], a, row, g);
    }
}

// widen to f32 and apply the rotation signs (sign masks are lane constants)
template <bool kBf16, bool kRht>
__device__ __forceinline__ void unpack_signed(const Raw<kBf16> &r, float v[16], const uint32_t mask[kBf16 ? 8 : 16])
{
    if (kBf16) {
        const uint32_t w[8] = {r.q[0].x, r.q[0].y, r.q[0].z, r.q[0].w, r.q[1].x, r.q[1].y, r.q[1].z, r.q[1].w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t s = kRht ? (w[i] ^ mask[i]) : w[i];
            v[2 * i] = bf16_lo(s);
            v[2 * i + 1] = bf16_hi(s);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t w[4] = {r.q[i].x, r.q[i].y, r.q[i].z, r.q[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) v[4 * i + j] = u2f(kRht ? (w[j] ^ mask[4 * i + j]) : w[j]);
        }
    }
}

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

// One quad of rows for one lane.  Once a row's raw words are unpacked its slot is free, so with
// kPrefetch the same row of the block's next quad (qn) is fetched right away, four rows of
// arithmetic ahead of its use; the block's last quad runs the copy without the loads.
template <bool kBf16, int kMode, bool kRht, bool kPrefetch>
__device__ __forceinline__ void quantize_quad(const RowsArgs &a, const LaneSetup &L, const TensorConsts &tc,
                                              const uint32_t *mask, Raw<kBf16> raw[4], int64_t quad,
                                              int64_t qn, int64_t G, int64_t gc, float &m,
                                              const float *inv_tab)
{
    uint32_t draw[4] = {0u, 0u, 0u, 0u};
    if (kMode == QII_MS_EDEN) {
        const U4 w = philox_seeded(a.seed_sr, (uint32_t)L.g, (uint32_t)quad, 0, kStreamScale);
        draw[0] = w.x >> 12; draw[1] = w.y >> 12; draw[2] = w.z >> 12; draw[3] = w.w >> 12;
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int64_t row = quad * 4 + it;
        float v[16];
        unpack_signed<kBf16, kRht>(raw[it], v, mask);
        if (kPrefetch) {
            const int64_t rn = qn * 4 + it;
            load_raw<kBf16>(raw[it], a, rn < a.R ? rn : a.R - 1, gc);
        }
        if (kRht) rht128_lane(v, L);
        uint32_t packed[2];
        if (kMode == QII_MS_EDEN_PH) {
            // heavy pass of the post hoc scheme: codes, corrected pseudo-scale, running maximum
            float gmax;
            const float t = posthoc_group16(v, packed, gmax);
            if (L.col_ok && row < a.R) {
                *reinterpret_cast<uint2 *>(a.codes + row * (a.C / 2) + (uint32_t)L.g * 8u) = make_uint2(packed[0], packed[1]);
                (a.tbuf + row * G)[(uint32_t)L.g] = t;
                m = fmaxf(m, gmax);
            }
            continue;
        }
        const uint32_t b = quantize_group16<kMode>(v, tc, draw[it], a.seed_sr, row, L.g, packed, inv_tab);
        // row base pointers are wave-uniform (scalar registers); the lane adds a 32-bit offset
        uint8_t *crow = a.codes + row * (a.C / 2), *srow = a.scales + row * G;
        const uint32_t goff = (uint32_t)L.g;
        if (L.col_ok && row < a.R)
            *reinterpret_cast<uint2 *>(crow + goff * 8u) = make_uint2(packed[0], packed[1]);
        if (G % 8 == 0) {   // whole octets: one 8-byte store per chunk
            const uint2 sc = gather_scale_bytes(b, L.blk);
            if (L.col_ok && row < a.R && L.blk == 0)
                *reinterpret_cast<uint2 *>(srow + goff) = sc;
        } else if (L.col_ok && row < a.R) {
            srow[goff] = (uint8_t)b;
        }
    }
}

template <bool kBf16, int kMode, bool kRht>
__global__ __launch_bounds__(256) void quantize_rows_kernel(RowsArgs a)
{
    const int64_t G = a.C / 16;
    const LaneSetup L = lane_setup(a, G);
    // (the heavy pass of the post hoc scheme knows no tensor maximum: tc stays unused there)
    const TensorConsts tc = kMode == QII_MS_EDEN_PH ? TensorConsts{} : tensor_consts(kMode, *a.amax);
    if (kMode != QII_MS_EDEN_PH && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *a.tensor_scale = tc.x32;
    const int64_t quads = (a.R + 3) / 4;
    if (tc.zero) {  // uniform: an all-zero tensor is emitted as zero bytes
        for (int64_t quad = L.first; quad < quads; quad += L.step)
            for (int it = 0; it < 4; ++it) {
                const int64_t row = quad * 4 + it;
                if (L.col_ok && row < a.R) {
                    *reinterpret_cast<uint2 *>(a.codes + (row * a.C + L.g * 16) / 2) = make_uint2(0u, 0u);
                    a.scales[row * G + L.g] = 0;
                }
            }
        return;
    }
    __shared__ float inv_tab[128];
    if (kMode != QII_MS_EDEN_PH) fill_inv_table(inv_tab, tc);
    uint32_t mask[kBf16 ? 8 : 16];
    make_masks<kBf16>(L.sign16, mask);
    const int64_t gc = L.col_ok ? L.g : G - 1;
    Raw<kBf16> raw[4];
    int64_t quad = L.first;   // (a wave whose first quad lies beyond the tensor stores nothing)
    load_quad<kBf16>(raw, a, quad, gc);
    float m = 0.0f;
    for (; quad + L.step < quads; quad += L.step)
        quantize_quad<kBf16, kMode, kRht, true>(a, L, tc, mask, raw, quad, quad + L.step, G, gc, m, inv_tab);
    quantize_quad<kBf16, kMode, kRht, false>(a, L, tc, mask, raw, quad, quad, G, gc, m, inv_tab);
    if (kMode == QII_MS_EDEN_PH && a.amax_out) {   // one atomic per wave at most; a wave covers many quads
        m = wave_max(m);
        if ((threadIdx.x & 63) == 0) max_to_global(m, a.amax_out);
    }
}

template <bool kBf16, bool kRht>
__global__ __launch_bounds__(256, 4) void absmax_rows_kernel(RowsArgs a)
{
    __shared__ float wave_m[4];
    const int64_t G = a.C / 16;
    const LaneSetup L = lane_setup(a, G);
    uint32_t mask[kBf16 ? 8 : 16];
    make_masks<kBf16>(L.sign16, mask);
    const int64_t quads = (a.R + 3) / 4;
    const int64_t gc = L.col_ok ? L.g : G - 1;
    float m = 0.0f;
    Raw<kBf16> raw[4];
    load_quad<kBf16>(raw, a, L.first, gc);
    for (int64_t quad = L.first; quad < quads; quad += L.step) {
        Raw<kBf16> nxt[4];
        const int64_t qn = quad + L.step;
        load_quad<kBf16>(nxt, a, qn < quads ? qn : quad, gc);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            float v[16];
            unpack_signed<kBf16, kRht>(raw[it], v, mask);
            if (kRht) rht128_lane<false>(v, L);
            // a clamped duplicate of a real row cannot change the maximum; lanes beyond the
            // last column hold a made-up chunk and are left out
            if (L.col_ok) m = fmaxf(m, group_absmax(v));
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) raw[it] = nxt[it];
    }
    if (kRht) m = __builtin_fmaf(m, kInvSqrt128, 0.0f);   // the scaling the rotation left out
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0) wave_m[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = fmaxf(fmaxf(wave_m[0], wave_m[1]), fmaxf(wave_m[2], wave_m[3]));
        // the running maximum only grows, so a stale read can only cause a redundant atomic
        if (f2u(m) > __atomic_load_n(a.amax_out, __ATOMIC_RELAXED)) atomicMax(a.amax_out, f2u(m));
    }
}

// waves of a block side by side on a row: as many as the row needs, at most 4
int rows_wpr(int64_t C)
{
    const int64_t nch = (C / 16 + 7) / 8;   // 128-chunks per row; a wave takes 8
    return nch <= 8 ? 1 : nch <= 16 ? 2 : 4;
}

// blocks: as many as stay resident at once (4 per CU), with the row quads split evenly
dim3 rows_grid(int64_t R, int64_t C)
{
    const int64_t G = C / 16, nch = (G + 7) / 8;
    const int wpr = rows_wpr(C);
    const int64_t gy = (nch + 8 * wpr - 1) / (8 * wpr);
    const int64_t quads = (R + 3) / 4, qpb = 4 / wpr, bquads = (quads + qpb - 1) / qpb;
    int64_t cap = (256 * 4) / gy;                  // 256 CUs x 4 resident blocks
    if (cap < 1) cap = 1;
    const int64_t iters = (bquads + cap - 1) / cap; // iterations per block
    int64_t gx = (bquads + iters - 1) / iters;      // even split
    if (gx < 1) gx = 1;
    return dim3((unsigned)gx, (unsigned)gy);
}

RowsArgs make_args(const Source &src, int64_t R, int64_t C, uint64_t seed_rht, uint64_t seed_sr)
{
    RowsArgs a;
    a.x = src.x; a.ld = src.ld; a.R = R; a.C = C;
    const U4 w = philox_seeded(seed_rht, 0, 0, 0, kStreamRht);
    a.sign[0] = w.x; a.sign[1] = w.y; a.sign[2] = w.z; a.sign[3] = w.w;
    a.seed_sr = seed_sr;
    a.amax = nullptr; a.codes = nullptr; a.scales = nullptr; a.tensor_scale = nullptr; a.amax_out = nullptr;
    a.tbuf = nullptr;
    a.wpr = rows_wpr(C);
    return a;
}

}  // namespace

bool rows_kernels_apply(const Source &src)
{
    return !src.transpose && (src.kind == kSrcBF16 || src.kind == kSrcF32);
}

hipError_t launch_absmax_rows(const Source &src, int64_t R, int64_t C, int rht, uint64_t seed_rht,
                              float *amax, hipStream_t s)
{
    RowsArgs a = make_args(src, R, C, seed_rht, 0);
    a.amax_out = reinterpret_cast<uint32_t *>(amax);
    const dim3 grid = rows_grid(R, C), block(256);
    const bool bf = src.kind == kSrcBF16;
    if (bf) { if (rht) hipLaunchKernelGGL((absmax_rows_kernel<true, true>), grid, block, 0, s, a); else hipLaunchKernelGGL((absmax_rows_kernel<true, false>), grid, block, 0, s, a); }
    else { if (rht) hipLaunchKernelGGL((absmax_rows_kernel<false, true>), grid, block, 0, s, a); else hipLaunchKernelGGL((absmax_rows_kernel<false, false>), grid, block, 0, s, a); }
    return hipGetLastError();
}

hipError_t launch_quantize_rows(const QuantizeArgs &q, hipStream_t s)
{
    RowsArgs a = make_args(q.src, q.R, q.C, q.seed_rht, q.seed_sr);
    a.amax = q.amax; a.codes = q.codes; a.scales = q.scales; a.tensor_scale = q.tensor_scale;
    a.tbuf = q.tbuf; a.amax_out = q.amax_accum;
    const dim3 grid = rows_grid(q.R, q.C), block(256);
    const bool bf = q.src.kind == kSrcBF16;
#define QII_ROWS(BF, MODE, RHT) hipLaunchKernelGGL((quantize_rows_kernel<BF, MODE, RHT>), grid, block, 0, s, a)
#define QII_ROWS_MODE(BF, RHT)                                   \
    do {                                                         \
        if (q.mode == QII_RTN) QII_ROWS(BF, QII_RTN, RHT);       \
        else if (q.mode == QII_SR) QII_ROWS(BF, QII_SR, RHT);    \
        else if (q.mode == QII_RTN_46) QII_ROWS(BF, QII_RTN_46, RHT); \
        else if (q.mode == QII_MS_EDEN_PH) QII_ROWS(BF, QII_MS_EDEN_PH, RHT); \
        else QII_ROWS(BF, QII_MS_EDEN, RHT);                     \
    } while (0)
    if (bf) { if (q.rht) QII_ROWS_MODE(true, true); else QII_ROWS_MODE(true, false); }
    else { if (q.rht) QII_ROWS_MODE(false, true); else QII_ROWS_MODE(false, false); }
#undef QII_ROWS_MODE
#undef QII_ROWS
    return hipGetLastError();
}

}  // namespace qii
