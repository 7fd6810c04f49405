// Tuned quantizer / abs-max kernels for dense row-major sources quantized along their
// COLUMNS (the transposed case: Q(E^T), whose scale groups and rotation chunks run down the
// rows of x while memory is contiguous along its columns), and for the backward pass's
// re-quantization of a saved NVFP4 tensor with transposition (Q(W^T), Q(X^T)), where the
// source element is dequantized on load: (e2m1 * e4m3) * tensor_scale.
//
// Layout of the work: the 4 lanes of a quad own two adjacent columns of x (= two output rows)
// and one 128-chunk of them, 32 rows each (lane q holds rows 32q .. 32q+31 of the chunk, for
// both columns): one 4-byte load fetches a row's two bf16 columns, so a wave covers 32 columns
// with 32 load instructions of four 64-byte row pieces each, coalesced without a transpose
// through LDS.  Butterfly stages over index bits 0..4 are in-lane, bits 5 and 6 pair lanes
// xor 1 and xor 2 with one v_fmac_f32_dpp each (lanes with the stage bit set carry -(a - b),
// undone by the sign of their scaling constant, as in the row kernels).  A lane owns two whole
// scale groups per column, so group maxima and dot products never leave it; it writes 16
// contiguous bytes of codes per column, a quad 64, and the 4 waves of a block take 4
// consecutive chunks of the same columns (256 contiguous bytes per output row); the 8 scale
// bytes of a (column, chunk) are gathered with DPP into one store.  The scale-rounding draws
// follow the library-wide rule (one Philox call feeds rows 4j..4j+3 of one column group): the
// 8 lanes that own columns 4j..4j+3 compute one call each (column groups 0..7 of the chunk)
// and fetch the words they need with ds_bpermute.  An NVFP4 source (re-quantization with
// transposition) is dequantized on load; there one byte holds a row's two columns.
#include "qii_device.h"
#include "qii_internal.h"
#include "quantize_core.h"
#include "quantize_lanes.h"

namespace qii {
namespace {

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
    uint32_t *amax_out;  // abs-max kernel (one word), and the heavy pass of the post hoc scheme (kAmaxSpread words, nullable there)
    float *tbuf;         // post hoc scheme: corrected pseudo-scales [R][C/16]
};

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Buffer descriptor of the 128 source rows of one chunk: the loads below then take their
// wave-uniform part (base, row offset) from scalar registers and only a 32-bit lane offset from
// a vector register, with no per-lane 64-bit address arithmetic.  `bytes` covers exactly the
// rows and columns a chunk reads; an offset beyond it would read 0, never fault.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t chunk_rsrc(const void *base, int64_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// Raw words of this lane's 32 rows (rows 32q .. 32q+31 of the chunk) of columns j0 and j0+1
// (j0 even): one word per row (two bf16, or two FP4 codes plus their scale byte), two for f32.
template <int kSrc>
struct RawCols {
    uint32_t a[32];
    uint32_t b[kSrc == kSrcBF16 ? 1 : 32];   // f32: second column; NVFP4: scale bytes
};

// issue the loads; `chunk` is wave-uniform, j0 is clamped into the tensor by the caller, so every
// lane loads from a valid address
template <int kSrc>
__device__ __forceinline__ void load_quarter_chunk_raw(RawCols<kSrc> &r, const ColsArgs &a, int64_t chunk, uint32_t j0, int q)
{
    if (kSrc == kSrcNVFP4) {
        // buffer loads: wave-uniform base and row offset in scalar registers, 32-bit lane offset
        const int64_t cstride = a.ld / 2, sstride = a.ld / 16;
        const __amdgpu_buffer_rsrc_t rc_rsrc = chunk_rsrc((const uint8_t *)a.x + chunk * 128 * cstride, 127 * cstride + a.R / 2);
        const __amdgpu_buffer_rsrc_t rs_rsrc = chunk_rsrc(a.in_scales + chunk * 128 * sstride, 127 * sstride + a.R / 16);
        const int oc = (int)(32 * q * cstride + j0 / 2), os = (int)(32 * q * sstride + j0 / 16);
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            r.a[i] = __builtin_amdgcn_raw_buffer_load_b8(rc_rsrc, oc, (int)(i * cstride), 0);
            r.b[i] = __builtin_amdgcn_raw_buffer_load_b8(rs_rsrc, os, (int)(i * sstride), 0);
        }
    } else if (kSrc == kSrcBF16) {
        const __amdgpu_buffer_rsrc_t rsrc = chunk_rsrc((const char *)a.x + chunk * 128 * a.ld * 2, (127 * a.ld + a.R) * 2);
        const int off = (int)((32 * q * a.ld + j0) * 2);
#pragma unroll
        for (int i = 0; i < 32; ++i) r.a[i] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, off, (int)(i * a.ld * 2), 0);
    } else {
        const __amdgpu_buffer_rsrc_t rsrc = chunk_rsrc((const char *)a.x + chunk * 128 * a.ld * 4, (127 * a.ld + a.R) * 4);
        const int off = (int)((32 * q * a.ld + j0) * 4);
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(rsrc, off, (int)(i * a.ld * 4), 0);
            r.a[i] = w[0];
            r.b[i] = w[1];
        }
    }
}

// widen to f32 (an NVFP4 source is dequantized: (e2m1 * e4m3) * tensor scale, first product exact)
// and apply the rotation signs
template <int kSrc, bool kRht>
__device__ __forceinline__ void unpack_quarter_chunk(float v[2][32], const RawCols<kSrc> &r, const ColsArgs &a, int q)
{
    const uint32_t sw = q == 0 ? a.sign[0] : q == 1 ? a.sign[1] : q == 2 ? a.sign[2] : a.sign[3];
    const float x32 = kSrc == kSrcNVFP4 ? *a.in_ts : 0.0f;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const uint32_t flip = kRht ? (((sw >> i) & 1u) << 31) : 0u;
        if (kSrc == kSrcNVFP4) {
            const float2_t c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(r.a[i], 1.0f, 0);
            const float x8 = e4m3_decode(r.b[i]);
            v[0][i] = u2f(f2u((c[0] * x8) * x32) ^ flip);
            v[1][i] = u2f(f2u((c[1] * x8) * x32) ^ flip);
        } else if (kSrc == kSrcBF16) {
            v[0][i] = u2f((r.a[i] << 16) ^ flip);
            v[1][i] = u2f((r.a[i] & 0xFFFF0000u) ^ flip);
        } else {
            v[0][i] = u2f(r.a[i] ^ flip);
            v[1][i] = u2f(r.b[i] ^ flip);
        }
    }
}

template <int kSrc, bool kRht>
__device__ __forceinline__ void load_quarter_chunk(float v[2][32], const ColsArgs &a, int64_t chunk, uint32_t j0, int q)
{
    RawCols<kSrc> r;
    load_quarter_chunk_raw<kSrc>(r, a, chunk, j0, q);
    unpack_quarter_chunk<kSrc, kRht>(v, r, a, q);
}

// the four scale groups of a lane (two per column), their stores
template <int kMode, int kFast>
__device__ __forceinline__ void quantize_tile_groups(const ColsArgs &a, float v[2][32], const TensorConsts &tc,
                                                     const uint32_t draw[2][2], int64_t chunk, int64_t j0, int q,
                                                     const float *inv_tab)
{
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        uint32_t codes[4];
        uint32_t sc = 0u;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t b = quantize_group16<kMode, kFast, true>(v[e] + 16 * h, tc, draw[e][h], a.seed_sr, j0 + e,
                                                                    chunk * 8 + 2 * q + h, codes + 2 * h, inv_tab);
            sc |= b << (8 * h);
        }
        const uint2 s8 = gather_quad_scales(sc, q);
        if (j0 + e < a.R) {
            store_codes16(a.codes + (j0 + e) * (a.C / 2) + chunk * 64 + 16 * q, codes[0], codes[1], codes[2], codes[3]);
            if (q == 0) *reinterpret_cast<uint2 *>(a.scales + (j0 + e) * (a.C / 16) + chunk * 8) = s8;
        }
    }
}

template <int kSrc, int kMode, bool kRht>
__global__ __launch_bounds__(256) void quantize_cols_kernel(ColsArgs a)
{
    const int lane = threadIdx.x & 63, q = lane & 3;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Blocks are dispatched x fastest and go to the 8 dies round robin.  Where the grid allows it, die k
    // takes stripes of 32 column blocks (2 KiB of a source row) and walks each stripe column blocks
    // fastest, so that the pieces of one source row inside a stripe are fetched at about the same
    // time and through one L2.
    uint32_t bx = blockIdx.x, by = blockIdx.y;
    if ((gridDim.y & 255u) == 0u) {
        const uint32_t id = by * gridDim.x + bx, xcd = id & 7u, slot = id >> 3, per = 32u * gridDim.x;
        const uint32_t stripe = (slot / per) * 8u + xcd, r = slot % per;
        by = 32u * stripe + (r & 31u);
        bx = r >> 5;
    }
    const int64_t chunk = (int64_t)bx * 4 + wave;   // wave-uniform
    const int64_t j0 = (int64_t)by * 32 + 2 * (lane >> 2);
    // R is even whenever this kernel is chosen, so a pair of columns is in range or not as a whole
    const bool live = chunk * 128 < a.C;   // wave-uniform
    const int64_t jc = j0 < a.R ? j0 : a.R - 2;
    // the tile's loads are issued before anything else: they do not depend on the tensor constants,
    // whose set-up (a dependent load, divisions, the table and its barrier) then overlaps them
    RawCols<kSrc> raw;
    if (kMode != QII_MS_EDEN_PH && live) load_quarter_chunk_raw<kSrc>(raw, a, chunk, (uint32_t)jc, q);
    // (the heavy pass of the post hoc scheme knows no tensor maximum: tc stays unused there)
    const TensorConsts tc = kMode == QII_MS_EDEN_PH ? TensorConsts{} : tensor_consts(kMode, *a.amax);
    if (kMode != QII_MS_EDEN_PH && bx == 0 && by == 0 && threadIdx.x == 0) *a.tensor_scale = tc.x32;
    if (kMode == QII_MS_EDEN_PH) {
        // heavy pass of the post hoc scheme: codes, corrected pseudo-scales, and the block's
        // maximum into the running maximum (a wave does one tile only, so the four waves of a
        // block are combined first; waves beyond the last chunk take part with 0)
        __shared__ float wave_m[4];
        float m = 0.0f;
        if (chunk * 128 < a.C) {
            float v[2][32];
            load_quarter_chunk<kSrc, kRht>(v, a, chunk, (uint32_t)(j0 < a.R ? j0 : a.R - 2), q);
            if (kRht) {
                fwht128_quad(v[0], q);
                fwht128_quad(v[1], q);
            }
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                uint32_t codes[4];
                float t[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float gmax;
                    t[h] = posthoc_group16(v[e] + 16 * h, codes + 2 * h, gmax);
                    if (j0 + e < a.R) m = fmaxf(m, gmax);
                }
                if (j0 + e < a.R) {
                    // (an ordinary store: the non-temporal one of the other modes made this kernel 5 % slower)
                    *reinterpret_cast<uint4 *>(a.codes + (j0 + e) * (a.C / 2) + chunk * 64 + 16 * q) =
                        make_uint4(codes[0], codes[1], codes[2], codes[3]);
                    *reinterpret_cast<float2 *>(a.tbuf + (j0 + e) * (a.C / 16) + chunk * 8 + 2 * q) = make_float2(t[0], t[1]);
                }
            }
        }
        if (a.amax_out) {   // uniform
            m = wave_max(m);
            if (lane == 0) wave_m[wave] = m;
            __syncthreads();
            if (threadIdx.x == 0)
                max_to_global(fmaxf(fmaxf(wave_m[0], wave_m[1]), fmaxf(wave_m[2], wave_m[3])),
                              amax_spread_word(a.amax_out, blockIdx.x + gridDim.x * blockIdx.y));
        }
        return;
    }
    __shared__ float inv_tab[128];
    fill_inv_table(inv_tab, tc);   // before any wave leaves: it ends in a block-wide barrier
    if (!live) return;
    if (tc.zero) {  // uniform: an all-zero tensor is emitted as zero bytes
#pragma unroll
        for (int e = 0; e < 2; ++e)
            if (j0 + e < a.R) {
                *reinterpret_cast<uint4 *>(a.codes + (j0 + e) * (a.C / 2) + chunk * 64 + 16 * q) = make_uint4(0u, 0u, 0u, 0u);
                if (q == 0) *reinterpret_cast<uint2 *>(a.scales + (j0 + e) * (a.C / 16) + chunk * 8) = make_uint2(0u, 0u);
            }
        return;
    }
    float v[2][32];
    unpack_quarter_chunk<kSrc, kRht>(v, raw, a, q);
    if (kRht) {
        fwht128_quad(v[0], q);
        fwht128_quad(v[1], q);
    }
    uint32_t draw[2][2] = {{0u, 0u}, {0u, 0u}};
    if (kMode == QII_MS_EDEN) octet_draws(draw, a.seed_sr, chunk, j0, q);
    if (tc.fast) quantize_tile_groups<kMode, 1>(a, v, tc, draw, chunk, j0, q, inv_tab);   // uniform: one branch per tile
    else quantize_tile_groups<kMode, 0>(a, v, tc, draw, chunk, j0, q, inv_tab);
}

// Abs-max pass: few long-lived blocks (two per compute unit) that stride over the tiles and fold
// their maximum into the result with one atomic each at the very end (device-wide atomics on one
// address are resolved one after the other, about 10 ns each).  A block requests its next tile
// before it works on the current one.  Tile order as in the quantizer where the shape allows it:
// the blocks of one die walk that die's stripes of 32 column blocks, column blocks fastest.
template <int kSrc, bool kRht>
__global__ __launch_bounds__(256) void absmax_cols_kernel(ColsArgs a, int64_t tiles_x, int64_t tiles)
{
    __shared__ float wave_m[4];
    const int lane = threadIdx.x & 63, q = lane & 3;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t tiles_y = tiles / tiles_x;
    const bool striped = (tiles_y & 255) == 0 && (gridDim.x & 7u) == 0u;   // uniform
    // the k-th tile of this block: (row block bx, column block by), or none
    auto tile_of = [&](int64_t k, int64_t &bx, int64_t &by) -> bool {
        if (striped) {
            const int64_t slot = (int64_t)(blockIdx.x >> 3) + k * (gridDim.x >> 3), per = 32 * tiles_x;
            if (slot >= tiles / 8) return false;
            const int64_t stripe = (slot / per) * 8 + (blockIdx.x & 7u), r = slot % per;
            by = 32 * stripe + (r & 31);
            bx = r >> 5;
        } else {
            const int64_t t = (int64_t)blockIdx.x + k * gridDim.x;
            if (t >= tiles) return false;
            bx = t % tiles_x;
            by = t / tiles_x;
        }
        return true;
    };
    float m = 0.0f;
    RawCols<kSrc> cur, nxt;
    int64_t bx, by;
    bool have = tile_of(0, bx, by);
    bool live = have && (bx * 4 + wave) * 128 < a.C;   // wave-uniform
    // (a clamped duplicate of a real column pair cannot change the maximum)
    if (live) {
        const int64_t j0 = by * 32 + 2 * (lane >> 2);
        load_quarter_chunk_raw<kSrc>(cur, a, bx * 4 + wave, (uint32_t)(j0 < a.R ? j0 : a.R - 2), q);
    }
    for (int64_t k = 1; have; ++k) {
        const bool have_n = tile_of(k, bx, by);
        const bool live_n = have_n && (bx * 4 + wave) * 128 < a.C;
        if (live_n) {
            const int64_t j0 = by * 32 + 2 * (lane >> 2);
            load_quarter_chunk_raw<kSrc>(nxt, a, bx * 4 + wave, (uint32_t)(j0 < a.R ? j0 : a.R - 2), q);
        }
        if (live) {
            float v[2][32];
            unpack_quarter_chunk<kSrc, kRht>(v, cur, a, q);
            if (kRht) {
                fwht128_quad<false>(v[0], q);
                fwht128_quad<false>(v[1], q);
            }
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int h = 0; h < 2; ++h) m = fmaxf(m, group_absmax(v[e] + 16 * h));
        }
        cur = nxt;
        have = have_n;
        live = live_n;
    }
    if (kRht) m = __builtin_fmaf(m, kInvSqrt128, 0.0f);   // the scaling the rotation left out
    m = wave_max(m);
    if (lane == 0) wave_m[wave] = m;
    __syncthreads();
    if (threadIdx.x == 0) max_to_global(fmaxf(fmaxf(wave_m[0], wave_m[1]), fmaxf(wave_m[2], wave_m[3])), a.amax_out);
}

ColsArgs make_args(const Source &src, int64_t R, int64_t C, uint64_t seed_rht, uint64_t seed_sr)
{
    ColsArgs a;
    a.x = src.x; a.in_scales = src.scales; a.in_ts = src.ts; a.ld = src.ld; a.R = R; a.C = C;
    const U4 w = philox_seeded(seed_rht, 0, 0, 0, kStreamRht);
    a.sign[0] = w.x; a.sign[1] = w.y; a.sign[2] = w.z; a.sign[3] = w.w;
    a.seed_sr = seed_sr;
    a.amax = nullptr; a.codes = nullptr; a.scales = nullptr; a.tensor_scale = nullptr; a.amax_out = nullptr;
    a.tbuf = nullptr;
    return a;
}

dim3 cols_grid(int64_t R, int64_t C)
{
    return dim3((unsigned)((C / 128 + 3) / 4), (unsigned)((R + 31) / 32));
}

}  // namespace

// transposed sources whose quantized dimension is a multiple of 128 and whose rows allow the
// two-column loads: an even number of columns and 4-byte (bf16) / 8-byte (f32) aligned pairs
bool cols_kernels_apply(const Source &src, int64_t R, int64_t C)
{
    if (!src.transpose || C % 128 != 0 || R % 2 != 0 || (R + 31) / 32 > 65535) return false;
    if (src.ld > (int64_t)1 << 21) return false;   // offsets within a chunk (128 rows, in bytes) stay below 2^31
    const uintptr_t p = reinterpret_cast<uintptr_t>(src.x);
    if (src.kind == kSrcBF16) return src.ld % 2 == 0 && p % 4 == 0;
    if (src.kind == kSrcF32) return src.ld % 2 == 0 && p % 8 == 0;
    return true;   // NVFP4: stored columns are a multiple of 16
}

hipError_t launch_absmax_cols(const Source &src, int64_t R, int64_t C, int rht, uint64_t seed_rht,
                              float *amax, hipStream_t s)
{
    ColsArgs a = make_args(src, R, C, seed_rht, 0);
    a.amax_out = reinterpret_cast<uint32_t *>(amax);
    const dim3 full = cols_grid(R, C), block(256);
    const int64_t tiles_x = full.x, tiles = (int64_t)full.x * full.y;
    const dim3 grid((unsigned)(tiles < 512 ? tiles : 512));   // two blocks per compute unit
#define QII_AMAX(SRC)                                                                             \
    do {                                                                                          \
        if (rht) hipLaunchKernelGGL((absmax_cols_kernel<SRC, true>), grid, block, 0, s, a, tiles_x, tiles);  \
        else hipLaunchKernelGGL((absmax_cols_kernel<SRC, false>), grid, block, 0, s, a, tiles_x, tiles);     \
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
    a.tbuf = q.tbuf; a.amax_out = q.amax_accum;
    const dim3 grid = cols_grid(q.R, q.C), block(256);
#define QII_COLS(SRC, MODE, RHT) hipLaunchKernelGGL((quantize_cols_kernel<SRC, MODE, RHT>), grid, block, 0, s, a)
#define QII_COLS_MODE(SRC, RHT)                                   \
    do {                                                          \
        if (q.mode == QII_RTN) QII_COLS(SRC, QII_RTN, RHT);       \
        else if (q.mode == QII_SR) QII_COLS(SRC, QII_SR, RHT);    \
        else if (q.mode == QII_RTN_46) QII_COLS(SRC, QII_RTN_46, RHT); \
        else if (q.mode == QII_MS_EDEN_PH) QII_COLS(SRC, QII_MS_EDEN_PH, RHT); \
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
