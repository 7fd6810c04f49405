// Host-side interfaces between the translation units of libqii.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/qii.h"

namespace qii {

// Where the quantizer reads its logical R x C matrix from.
//   kind F32 / BF16: element (r, c) = x[r*ld + c]            (transpose == 0)
//                                     x[c*ld + r]            (transpose == 1)
//   kind NVFP4     : element (r, c) = dequantized in[r][c] or in[c][r]; in_cols is the
//                    number of columns of the stored tensor.
enum SourceKind { kSrcF32 = 0, kSrcBF16 = 1, kSrcNVFP4 = 2 };

struct Source {
    int kind;
    int transpose;
    const void *x;           // f32 / bf16 data, or the FP4 codes
    const uint8_t *scales;   // NVFP4 only
    const float *ts;         // NVFP4 only (device scalar)
    int64_t ld;              // elements (f32/bf16) or stored columns (NVFP4)
};

struct QuantizeArgs {
    Source src;
    int64_t R, C;            // logical shape: groups of 16 run along C
    int mode;                // qii_mode
    int rht;                 // 0 or 1
    uint64_t seed_rht, seed_sr;
    const float *amax;       // device scalar: max |rotated tensor|
    uint8_t *codes;
    uint8_t *scales;
    float *tensor_scale;
    // post hoc range alignment only (mode QII_MS_EDEN_PH): the heavy pass writes one f32 per
    // group into tbuf instead of scale bytes and folds the group maxima into the 64 words (256
    // bytes apart, a region of 16 KiB) at amax_accum (nullable: the caller supplies the maximum itself); launch_posthoc_scales finishes
    float *tbuf;
    uint32_t *amax_accum;
    // a second copy of the scale bytes in the main GEMM kernel's tiled layout (nullable; only where
    // rows_kernels_apply, no rotation, C a multiple of 256; room for R rounded up to 256 rows)
    uint8_t *scales_tiled = nullptr;
};

// One read of a dense matrix producing Q(x) (side r: rows x cols) and Q(x^T) (side c: cols x rows),
// mode QII_MS_EDEN (amax of each rotated tensor supplied) or QII_MS_EDEN_PH (heavy pass: tbuf and
// amax_accum as in QuantizeArgs, per side); quantize_pair.hip
struct PairQuantizeArgs {
    Source src;
    int64_t rows, cols;
    int mode;
    struct Side {
        uint64_t seed_rht, seed_sr;
        const float *amax;
        uint8_t *codes;
        uint8_t *scales;
        float *tensor_scale;
        float *tbuf;
        uint32_t *amax_accum;
    } r, c;
};
bool pair_kernel_applies(const Source &src, int64_t rows, int64_t cols);
hipError_t launch_quantize_pair(const PairQuantizeArgs &p, hipStream_t s);

// p[i * stride_words] = v for i < count (count <= 256); a kernel, not a memset node, so that the
// calls can be captured in a HIP graph
hipError_t launch_fill_u32(uint32_t *p, uint32_t v, int count, int stride_words, hipStream_t s);
hipError_t launch_absmax(const Source &src, int64_t R, int64_t C, int rht, uint64_t seed_rht,
                         float *amax /* must hold 0 */, hipStream_t s);
hipError_t launch_rht(const Source &src, int64_t R, int64_t C, uint64_t seed_rht, float *y,
                      float *amax /* nullable, must hold 0 */, hipStream_t s);
hipError_t launch_quantize(const QuantizeArgs &a, hipStream_t s);
// amax: n_amax words, 256 bytes apart (1: a maximum supplied by the caller; 64: the spread running
// maximum of the heavy pass, whose maximum is taken).  tiled (C a multiple of 256): the scale bytes
// go out in the layout the main GEMM kernel reads ([row / 256][C / 256][row % 256][16 bytes]; room for
// the row count rounded up to 256) instead of row-major
hipError_t launch_posthoc_scales(const float *tbuf, const float *amax, int n_amax, int64_t R, int64_t C,
                                 uint64_t seed_sr, uint8_t *scales, float *tensor_scale, hipStream_t s,
                                 bool tiled = false);
hipError_t launch_dequantize(const uint8_t *codes, const uint8_t *scales, const float *ts,
                             int64_t rows, int64_t cols, float *y, hipStream_t s);
// tuned kernels for dense sources quantized along their rows (quantize_rows.hip)
bool rows_kernels_apply(const Source &src, int64_t R, int64_t C);
hipError_t launch_absmax_rows(const Source &src, int64_t R, int64_t C, int rht, uint64_t seed_rht,
                              float *amax, hipStream_t s);
hipError_t launch_quantize_rows(const QuantizeArgs &a, hipStream_t s);
// tuned kernels for dense sources quantized along their columns (quantize_cols.hip)
bool cols_kernels_apply(const Source &src, int64_t R, int64_t C);
hipError_t launch_absmax_cols(const Source &src, int64_t R, int64_t C, int rht, uint64_t seed_rht,
                              float *amax, hipStream_t s);
hipError_t launch_quantize_cols(const QuantizeArgs &a, hipStream_t s);
// ws (nullable): gemm_workspace_bytes(M, N, K) bytes, 16-byte aligned, for the re-tiled scale
// bytes of the fast kernel; without it a slower kernel reads the row-major scales directly
size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
// amax_c (nullable): device float that receives max |C| over the values as stored
// pretiled: bit 0 / bit 1 say that A.scales / B.scales already hold the tiled layout (K a multiple
// of 256, see launch_posthoc_scales), bit 2 / bit 3 that A's / B's tiled scale bytes are already in
// their place in ws (QuantizeArgs::scales_tiled); either way that operand's re-tiling is skipped
hipError_t launch_gemm(const qii_nvfp4 &A, const qii_nvfp4 &B, void *C, int c_is_bf16, int64_t ldc,
                       float *amax_c, void *ws, size_t ws_bytes, hipStream_t s, int pretiled = 0);

// host-only test aids for the shared last round of the main GEMM kernel (gemm_sharing_map.h):
// plan = {positions run one block per tile, shared tiles, sharing blocks}; the segments of a
// hardware block id as {block number, shared tile, first K tile, K tiles, slot} (returns their
// number, -1 beyond 4); the first and last partial-tile slot the fix-up kernel adds up for a tile
void gemm_sharing_plan(int64_t M, int64_t N, int64_t K, int32_t plan[3]);
int gemm_sharing_segments(int rem, int ktotal, int grid, int block_id, int32_t *out);
void gemm_sharing_tile_slots(int rem, int ktotal, int grid, int lt, int32_t out[2]);

// sweeps of the hardware conversions and short division sequences against their value-space
// rules; counts[0..7] (device) receive the numbers of mismatches (selftest.hip)
// exploratory non-exact GEMM variants (gemm_inexact.hip); ws as gemm_inexact_workspace_bytes says
size_t gemm_inexact_workspace_bytes(int64_t M, int64_t N, int64_t K, int variant);
hipError_t launch_gemm_inexact(const qii_nvfp4 &A, const qii_nvfp4 &B, void *C, int c_is_bf16, int64_t ldc, int variant,
                               void *ws, hipStream_t s);
hipError_t launch_selftest_conversions(unsigned long long *counts, hipStream_t s);
hipError_t launch_microbench(int kind, void *a, void *b, uint64_t n, int blocks, int iters, hipStream_t s);

}  // namespace qii
