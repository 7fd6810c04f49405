// Tuned quantizer / abs-max kernels for dense row-major sources quantized along their rows
// (the contiguous case: Q(E), and the forward-pass RTN of X and W).
//
// Layout of the work: a lane owns one 16-element scale group, 8 lanes one 128-chunk, a wave
// 8 consecutive chunks of a row (1024 elements, 2 KiB of bf16) of one quad of 4 rows (one
// scale-rounding draw call serves the 4 rows of a group), a block 4 waves: side by side on
// wide tensors, or, when a row needs fewer than 4 waves, 2 or 4 row quads.  blockIdx.y selects
// the column range, blockIdx.x the row quads.  The four rows of a quad are requested together
// (32 B per lane and row) before anything else happens in the kernel.
// The octet register layout and its rotation are in quantize_lanes.h.
#include "qii_device.h"
#include "qii_internal.h"
#include "quantize_core.h"
#include "quantize_lanes.h"

namespace qii {
namespace {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

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
    uint32_t *amax_out;  // abs-max kernel (one word), and the heavy pass of the post hoc scheme
                         // (kAmaxSpread words, nullable there)
    float *tbuf;         // post hoc scheme: corrected pseudo-scales [R][C/16]
    uint8_t *tiled;      // nullable: a second copy of the scale bytes, [row / 256][C / 256][row % 256][16]
    int wpr;             // waves of a block that sit side by side on a row: 1, 2 or 4
    int gy;              // blocks side by side on a row; the grid is one-dimensional, columns fastest
};

struct LaneSetup : OctetLane {
    int quad;             // this wave's row quad (rows 4 quad .. 4 quad + 3); wave-uniform
    int64_t g;            // scale group within the row
    bool col_ok;
};

// kQuadsPerWave: row quads a wave takes (the quantizers: 1; the abs-max pass: 2)
template <int kQuadsPerWave>
__device__ __forceinline__ LaneSetup lane_setup(const RowsArgs &a, int64_t G)
{
    LaneSetup L;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept in a scalar register
    static_cast<OctetLane &>(L) = octet_lane(lane, a.sign);
    // wpr waves side by side, 4 / wpr waves below one another
    const int wcol = wave & (a.wpr - 1), wq = wave / a.wpr, qpb = 4 / a.wpr;
    // consecutive blocks walk along a row first, then down the rows: blocks that run at the same
    // time read one contiguous region of the tensor
    const int bx = (int)blockIdx.x / a.gy, by = (int)blockIdx.x - bx * a.gy;
    L.quad = (bx * qpb + wq) * kQuadsPerWave;
    const int64_t chunk = ((int64_t)by * a.wpr + wcol) * 8 + (lane >> 3);
    L.g = chunk * 8 + L.blk;
    L.col_ok = L.g < G;
    return L;
}

// raw row data of one lane: 16 elements
template <bool kBf16>
struct Raw {
    u32x4 q[kBf16 ? 2 : 4];
};

// All row addressing is wave-uniform (a wave works on whole rows): the row's base address sits
// in scalar registers inside a buffer descriptor that covers exactly the row's C elements, and a
// lane only contributes a 32-bit byte offset that never changes.  A row beyond the tensor gets an
// empty descriptor, a lane beyond the last column an offset beyond the descriptor: such loads
// return 0 and such stores are dropped by the hardware, so neither needs a branch or a mask.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_rsrc(const void *base, int64_t row_bytes_offset, bool row_ok, int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(reinterpret_cast<const char *>(base) + row_bytes_offset), 0,
                                             row_ok ? bytes : 0, 0x00020000);
}

constexpr uint32_t kNoStore = 0xFFFFFFF0u;   // a lane offset beyond every descriptor
// Cache policy of the code stores.  With rotation (the backward pass's quantizers) they are
// non-temporal: the lines do not linger dirty in L2, where the next kernel's traffic would have to
// push them out (-1 % and -3 % on the two 8192 x 8192 kernels, and the kernel that follows starts
// on a clean cache).  Without rotation (the forward pass) the GEMM reads the codes right away and
// ran 1.2 % slower when they had to come back from memory, so those stores stay ordinary.
template <bool kRht>
constexpr int code_store_policy() { return kRht ? 2 : 0; }

template <bool kBf16>
__device__ __forceinline__ void load_raw(Raw<kBf16> &r, const RowsArgs &a, int row, uint32_t voff)
{
    constexpr int n = kBf16 ? 2 : 4, esz = kBf16 ? 2 : 4;
    const __amdgpu_buffer_rsrc_t rs = row_rsrc(a.x, (int64_t)row * a.ld * esz, row < (int)a.R, (int)(a.C * esz));
#pragma unroll
    for (int i = 0; i < n; ++i) r.q[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + 16u * i, 0, 0);
}

template <bool kBf16>
__device__ __forceinline__ void load_quad(Raw<kBf16> raw[4], const RowsArgs &a, int quad, uint32_t voff)
{
#pragma unroll
    for (int it = 0; it < 4; ++it) load_raw<kBf16>(raw[it], a, quad * 4 + it, voff);
}

// widen to f32 and apply the rotation signs (sign masks are lane constants)
template <bool kBf16, bool kRht>
__device__ __forceinline__ void unpack_signed(const Raw<kBf16> &r, float v[16], const uint32_t mask[kBf16 ? 8 : 16])
{
    if (kBf16) {
        const uint32_t w[8] = {r.q[0][0], r.q[0][1], r.q[0][2], r.q[0][3], r.q[1][0], r.q[1][1], r.q[1][2], r.q[1][3]};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t s = kRht ? (w[i] ^ mask[i]) : w[i];
            v[2 * i] = bf16_lo(s);
            v[2 * i + 1] = bf16_hi(s);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) v[4 * i + j] = u2f(kRht ? (r.q[i][j] ^ mask[4 * i + j]) : r.q[i][j]);
    }
}

// per-lane store offsets (bytes within a row of the output)
struct StoreOffsets {
    uint32_t codes;    // 8 bytes of codes per group
    uint32_t scale8;   // the gathered 8 scale bytes of a chunk: the lane holding block 0 stores them
    uint32_t scale1;   // one scale byte per lane (rows whose group count is not a multiple of 8)
    uint32_t t4;       // post hoc scheme: one f32 per group
    uint32_t tiled8;   // the chunk's 8 scale bytes within the tiled copy, relative to (row tile, row)
};

// One quad of rows for one lane: the four rows' raw words are in registers (requested at the very
// start of the kernel).
template <bool kBf16, int kMode, bool kRht, int kFast>
__device__ __forceinline__ void quantize_quad(const RowsArgs &a, const LaneSetup &L, const TensorConsts &tc,
                                              const uint32_t *mask, Raw<kBf16> raw[4], int64_t G,
                                              const StoreOffsets &so, float &m, const float *inv_tab)
{
    uint32_t draw[4] = {0u, 0u, 0u, 0u};
    if (kMode == QII_MS_EDEN) {
        const U4 w = philox_seeded(a.seed_sr, (uint32_t)L.g, (uint32_t)L.quad, 0, kStreamScale);
        draw[0] = w.x >> 12; draw[1] = w.y >> 12; draw[2] = w.z >> 12; draw[3] = w.w >> 12;
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int row = L.quad * 4 + it;   // wave-uniform
        float v[16];
        unpack_signed<kBf16, kRht>(raw[it], v, mask);
        if (kRht) rht128_lane(v, L);
        const bool row_ok = row < (int)a.R;
        const __amdgpu_buffer_rsrc_t rc = row_rsrc(a.codes, (int64_t)row * (a.C / 2), row_ok, (int)(a.C / 2));
        uint32_t packed[2];
        if (kMode == QII_MS_EDEN_PH) {
            // heavy pass of the post hoc scheme: codes, corrected pseudo-scale, running maximum
            float gmax;
            const float t = posthoc_group16(v, packed, gmax);
            __builtin_amdgcn_raw_buffer_store_b64(u32x2{packed[0], packed[1]}, rc, so.codes, 0, code_store_policy<kRht>());
            __builtin_amdgcn_raw_buffer_store_b32(f2u(t), row_rsrc(a.tbuf, (int64_t)row * G * 4, row_ok, (int)(G * 4)), so.t4, 0, 0);
            if (L.col_ok && row_ok) m = fmaxf(m, gmax);
            continue;
        }
        const uint32_t b = quantize_group16<kMode, kFast, true>(v, tc, draw[it], a.seed_sr, row, L.g, packed, inv_tab);
        __builtin_amdgcn_raw_buffer_store_b64(u32x2{packed[0], packed[1]}, rc, so.codes, 0, code_store_policy<kRht>());
        const __amdgpu_buffer_rsrc_t rs = row_rsrc(a.scales, (int64_t)row * G, row_ok, (int)G);
        if (kRht || G % 8 == 0) {   // whole octets (always so with rotation): one 8-byte store per chunk
            const uint2 sc = gather_scale_bytes(b, L.blk);
            __builtin_amdgcn_raw_buffer_store_b64(u32x2{sc.x, sc.y}, rs, so.scale8, 0, 0);
            if (!kRht && a.tiled) {   // uniform: the forward pass's copy for the GEMM (C a multiple of 256)
                const int64_t ksn = a.C / 256;
                const __amdgpu_buffer_rsrc_t rt = row_rsrc(a.tiled, ((int64_t)(row >> 8) * ksn * 256 + (row & 255)) * 16, row_ok,
                                                           (int)(ksn * 4096 - (row & 255) * 16));
                __builtin_amdgcn_raw_buffer_store_b64(u32x2{sc.x, sc.y}, rt, so.tiled8, 0, 0);
            }
        } else {
            __builtin_amdgcn_raw_buffer_store_b8((uint8_t)b, rs, so.scale1, 0, 0);
        }
    }
}

// One wave = one quad of rows x 1024 columns, one block = 4 such pieces; the grid covers the tensor.
// Blocks are short-lived on purpose: many independent blocks that start and finish at different
// times keep the memory traffic of the chip smooth, where long-lived waves marching in step (a
// grid-stride loop with prefetch was measured) load and compute in bursts and ran 10 % slower.
template <bool kBf16, int kMode, bool kRht>
__global__ __launch_bounds__(256) void quantize_rows_kernel(RowsArgs a)
{
    constexpr int esz = kBf16 ? 2 : 4;
    const int64_t G = a.C / 16;
    const LaneSetup L = lane_setup<1>(a, G);
    // the rows are requested before anything else: the loads do not depend on the tensor
    // constants, whose set-up (a dependent load, divisions, the table) then overlaps them
    const uint32_t voff = (uint32_t)L.g * (16u * esz);   // (beyond the row for lanes beyond the last column)
    Raw<kBf16> raw[4];
    load_quad<kBf16>(raw, a, L.quad, voff);
    // (the heavy pass of the post hoc scheme knows no tensor maximum: tc stays unused there)
    const TensorConsts tc = kMode == QII_MS_EDEN_PH ? TensorConsts{} : tensor_consts(kMode, *a.amax);
    if (kMode != QII_MS_EDEN_PH && blockIdx.x == 0 && threadIdx.x == 0) *a.tensor_scale = tc.x32;
    StoreOffsets so;
    so.codes = L.col_ok ? (uint32_t)L.g * 8u : kNoStore;
    so.scale8 = (L.col_ok && L.blk == 0) ? (uint32_t)L.g : kNoStore;
    so.scale1 = L.col_ok ? (uint32_t)L.g : kNoStore;
    so.t4 = L.col_ok ? (uint32_t)L.g * 4u : kNoStore;
    so.tiled8 = (L.col_ok && L.blk == 0) ? (uint32_t)(L.g >> 4) * 4096u + (uint32_t)((L.g >> 3) & 1) * 8u : kNoStore;
    if (tc.zero) {  // uniform: an all-zero tensor is emitted as zero bytes
        for (int it = 0; it < 4; ++it) {
            const int64_t row = (int64_t)L.quad * 4 + it;
            if (L.col_ok && row < a.R) {
                *reinterpret_cast<uint2 *>(a.codes + (row * a.C + L.g * 16) / 2) = make_uint2(0u, 0u);
                a.scales[row * G + L.g] = 0;
                if (!kRht && a.tiled) a.tiled[(((row >> 8) * (a.C / 256) + (L.g >> 4)) * 256 + (row & 255)) * 16 + (L.g & 15)] = 0;
            }
        }
        return;
    }
    __shared__ float inv_tab[128];
    __shared__ float wave_m[4];
    if (kMode != QII_MS_EDEN_PH) fill_inv_table(inv_tab, tc);
    uint32_t mask[kBf16 ? 8 : 16];
    make_masks<kBf16>(L.sign16, mask);
    float m = 0.0f;
    if (kMode == QII_MS_EDEN_PH || tc.fast)   // uniform: one branch for the whole kernel
        quantize_quad<kBf16, kMode, kRht, 1>(a, L, tc, mask, raw, G, so, m, inv_tab);
    else
        quantize_quad<kBf16, kMode, kRht, 0>(a, L, tc, mask, raw, G, so, m, inv_tab);
    if (kMode == QII_MS_EDEN_PH && a.amax_out) {   // uniform: one update per block, spread over the slot's words
        m = wave_max(m);
        if ((threadIdx.x & 63) == 0) wave_m[threadIdx.x >> 6] = m;
        __syncthreads();
        if (threadIdx.x == 0)
            max_to_global(fmaxf(fmaxf(wave_m[0], wave_m[1]), fmaxf(wave_m[2], wave_m[3])),
                          amax_spread_word(a.amax_out, blockIdx.x));
    }
}

// Abs-max pass.  Its result is one word that every block has to fold its maximum into, and such
// device-wide atomics on one address are resolved one after the other (about 4 ns each), so this
// kernel runs as few, long-lived blocks (two per compute unit) that stride over the row quads with
// the next quad's loads in flight, and issue one atomic each at the very end.
template <bool kBf16, bool kRht>
__global__ __launch_bounds__(256) void absmax_rows_kernel(RowsArgs a)
{
    constexpr int esz = kBf16 ? 2 : 4;
    __shared__ float wave_m[4];
    const int64_t G = a.C / 16;
    const LaneSetup L = lane_setup<1>(a, G);
    const int quads = (int)((a.R + 3) / 4);
    const int step = ((int)gridDim.x / a.gy) * (4 / a.wpr);
    const uint32_t voff = (uint32_t)L.g * (16u * esz);
    uint32_t mask[kBf16 ? 8 : 16];
    make_masks<kBf16>(L.sign16, mask);
    float m = 0.0f;
    Raw<kBf16> raw[4];
    load_quad<kBf16>(raw, a, L.quad, voff);   // (rows and columns beyond the tensor read as 0 and cannot change the maximum)
    for (int quad = L.quad; quad < quads; quad += step) {
        Raw<kBf16> nxt[4];
        load_quad<kBf16>(nxt, a, quad + step, voff);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            float v[16];
            unpack_signed<kBf16, kRht>(raw[it], v, mask);
            if (kRht) rht128_lane<false>(v, L);
            m = fmaxf(m, group_absmax(v));
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) raw[it] = nxt[it];
    }
    if (kRht) m = __builtin_fmaf(m, kInvSqrt128, 0.0f);   // the scaling the rotation left out
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) wave_m[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) max_to_global(fmaxf(fmaxf(wave_m[0], wave_m[1]), fmaxf(wave_m[2], wave_m[3])), a.amax_out);
}

// waves of a block side by side on a row: as many as the row needs, at most 4
int rows_wpr(int64_t C)
{
    const int64_t nch = (C / 16 + 7) / 8;   // 128-chunks per row; a wave takes 8
    return nch <= 8 ? 1 : nch <= 16 ? 2 : 4;
}

// one wave per row quad x 1024 columns; max_block_rows > 0 caps the number of blocks below one
// another (the abs-max pass then strides over the rest)
dim3 rows_grid(int64_t R, int64_t C, int64_t max_block_rows)
{
    const int64_t G = C / 16, nch = (G + 7) / 8;
    const int wpr = rows_wpr(C);
    const int64_t gy = (nch + 8 * wpr - 1) / (8 * wpr);
    const int64_t quads = (R + 3) / 4, qpb = 4 / wpr;
    int64_t gx = (quads + qpb - 1) / qpb;
    if (max_block_rows > 0 && gx > max_block_rows) {
        const int64_t iters = (gx + max_block_rows - 1) / max_block_rows;
        gx = (gx + iters - 1) / iters;   // even split
    }
    return dim3((unsigned)((gx < 1 ? 1 : gx) * gy), 1u);
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
    a.tiled = nullptr;
    a.wpr = rows_wpr(C);
    const int64_t nch = (C / 16 + 7) / 8;
    a.gy = (int)((nch + 8 * a.wpr - 1) / (8 * a.wpr));
    return a;
}

}  // namespace

// (a row of the source and of every output is addressed through a 32-bit buffer descriptor)
bool rows_kernels_apply(const Source &src, int64_t R, int64_t C)
{
    return !src.transpose && (src.kind == kSrcBF16 || src.kind == kSrcF32) && C <= ((int64_t)1 << 28) &&
           R < ((int64_t)1 << 31) - 8;   // row indices are 32-bit in the kernels
}

hipError_t launch_absmax_rows(const Source &src, int64_t R, int64_t C, int rht, uint64_t seed_rht,
                              float *amax, hipStream_t s)
{
    RowsArgs a = make_args(src, R, C, seed_rht, 0);
    a.amax_out = reinterpret_cast<uint32_t *>(amax);
    const int64_t gy_ = a.gy;
    const dim3 grid = rows_grid(R, C, 512 / gy_ > 0 ? 512 / gy_ : 1), block(256);   // two blocks per compute unit
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
    if (q.scales_tiled) {
        if (q.rht || q.C % 256 != 0 || q.mode == QII_MS_EDEN_PH) return hipErrorInvalidValue;
        a.tiled = q.scales_tiled;
    }
    const dim3 grid = rows_grid(q.R, q.C, 0), block(256);
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
