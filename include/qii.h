/*
 * qii.h -- C ABI of libqii: the NVFP4-quantized linear layer of Quartet II on one
 * AMD MI355X (gfx950).
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers (HBM) unless a comment says "host".  The
 *     caller owns every buffer, including the workspace; the library never allocates,
 *     frees or synchronises.  Kernels are enqueued on `stream` (a hipStream_t passed
 *     as void*; NULL = the default stream); outputs are valid once the stream reaches
 *     that point.  Scalars that the device produces (tensor scale, amax) stay on the
 *     device as float*.
 *   - Every function returns a qii_status.  On any status other than QII_OK nothing
 *     has been enqueued.  qii_last_error() (host string, thread local) explains the
 *     last failure.  Nothing throws, aborts or prints.
 *   - Matrices are row-major.  An NVFP4 tensor (Sec. 3.1 of the paper: FP4 E2M1
 *     elements, one FP8 E4M3 scale per 16 consecutive elements of a row, one FP32
 *     scale per tensor) is described by qii_nvfp4.  Its value is
 *         x_hat[r][c] = e2m1(codes[r][c]) * e4m3(scales[r][c/16]) * tensor_scale.
 *   - Randomness (omega_RHT, omega_SR of Algorithm 1) is counter based: outputs are a
 *     pure function of the seeds and the element / group index, never of the launch
 *     geometry.  Generator: Philox4x32-10 keyed by the 64-bit seed.
 *       rotation signs : counter (0, 0, 0, 0x52485400); sign j = bit (j mod 32) of
 *                        word (j div 32); a set bit means -1.
 *       scale rounding : group (row, cg) of the OUTPUT tensor uses counter
 *                        (cg, row div 4, 0, 0x53434C00), word (row mod 4), top 20 bits.
 *       element rounding (mode SR): element (row, col) uses counter
 *                        (col div 8, row, 0, 0x454C4D00), word ((col mod 8) div 2),
 *                        low 16 bits for even col, high 16 bits for odd col.
 *       backward sub-seed i : counter (i, 0, 0, 0x44525600), words 0 (low) and 1 (high).
 *   - Inputs must be finite.  An all-zero tensor quantizes to all-zero bytes with
 *     tensor_scale = 1.
 */
#ifndef QII_H
#define QII_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The enumerations below cross the ABI as 32-bit integers.  A C++ translation unit gives them the
 * fixed underlying type int, so that a value outside the enumerators (which the entry points
 * answer with QII_INVALID_ARG) is an ordinary integer and not undefined behaviour on load.      */
#ifdef __cplusplus
#define QII_ENUM_INT : int
#else
#define QII_ENUM_INT
#endif

typedef enum QII_ENUM_INT {
    QII_OK = 0,
    QII_INVALID_ARG = 1,         /* null pointer, bad enum, misaligned buffer          */
    QII_BAD_SHAPE = 2,           /* a dimension violates the divisibility rules below   */
    QII_UNSUPPORTED = 3,         /* combination not implemented                         */
    QII_WORKSPACE_TOO_SMALL = 4, /* ws_bytes below the matching *_workspace_bytes query */
    QII_HIP_ERROR = 5            /* a launch failed; text in qii_last_error()           */
} qii_status;

/* Rounding scheme of the quantizer.
 *   QII_RTN     round to nearest, grid max 6, scale cap 448 (Table 1, row "RTN 1x16";
 *               the forward pass of Sec. 5 without the 4/6 heuristic).
 *   QII_SR      Q_SR of Sec. 3.1: grid max 6*16/17, cap 448, element-wise stochastic
 *               rounding to FP4; never clips; unbiased.
 *   QII_MS_EDEN Algorithm 1 (Sec. 3.3): Q_RTN(x, s) with s = 6*16/17/0.93 and cap 256,
 *               then the per-16 EDEN factor merged into the E4M3 scale by stochastic
 *               rounding; unbiased after the inverse rotation.
 *   QII_RTN_46  round to nearest with the per-block "4/6" choice of Sec. 4.1 (Table 1,
 *               row "+4/6"; the forward pass of Sec. 5): each group of 16 is quantized
 *               twice, with its maximum mapped to 6 and to 4, and the candidate with the
 *               smaller squared error is kept (ties: 6).  Scale cap 256, so that the 1.5
 *               times larger scale of a block mapped to 4 (at most 384) is an E4M3 value.
 *               Deterministic; biased, hence forward pass only.
 *   QII_MS_EDEN_PH  MS-EDEN with the post hoc range alignment of Sec. 7: one heavy pass that
 *               needs no tensor maximum (group scales rounded to E8M3 = three mantissa bits at
 *               binary32 range, FP4 codes and EDEN factors w.r.t. those pseudo-scales, the
 *               rotated maximum reduced on the way) and one pass over the scales alone
 *               (divide by the tensor scale, stochastic rounding to E4M3 with the draws of
 *               QII_MS_EDEN).  Equal to QII_MS_EDEN bit for bit when the tensor scale is a
 *               power of two, otherwise a different but equally unbiased estimate.  Needs
 *               qii_quantize_posthoc_workspace_bytes of workspace. */
typedef enum QII_ENUM_INT { QII_RTN = 0, QII_SR = 1, QII_MS_EDEN = 2, QII_RTN_46 = 3, QII_MS_EDEN_PH = 4 } qii_mode;

typedef enum QII_ENUM_INT { QII_F32 = 0, QII_BF16 = 1 } qii_dtype;

/* One NVFP4 tensor of `rows` x `cols` (cols % 16 == 0).
 *   codes        rows*cols/2 bytes; element 2j of a row in the low nibble of byte j,
 *                element 2j+1 in the high nibble; 16-byte aligned.
 *   scales       rows*cols/16 bytes, E4M3 (bias 7, no infinities, 0x7F never written),
 *                plain row-major [rows][cols/16]; 8-byte aligned.
 *   tensor_scale one float.                                                           */
typedef struct {
    uint8_t *codes;
    uint8_t *scales;
    float *tensor_scale;
    int64_t rows;
    int64_t cols;
} qii_nvfp4;

/* Randomized Hadamard transform of Algorithm 1 (first loop), as a stand-alone op:
 *   y = RHT(x) or RHT(x^T), in f32, chunks of 128 along the rows of the logical
 *   matrix: y = H (d .* v) / sqrt(128), H[i][j] = (-1)^popcount(i & j), d from seed_rht.
 *   x: rows x cols, leading dimension ld (elements), dtype dt.  transpose != 0 works on
 *   x^T (y is cols x rows, contiguous); the rotated dimension must be a multiple of 128.
 *   amax (nullable): receives max |y| (Sec. 3.3, numerator of x^FP32).                */
qii_status qii_rht(const void *x, qii_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                   int transpose, uint64_t seed_rht, float *y, float *amax, void *stream);

/* max |RHT(x)| (or of x itself when rht_group == 0) into *amax: the global reduction
 * that Sec. 7 ("Fused Re-Quantization Kernel") names as the barrier before any scale
 * can be computed.  Same argument rules as qii_quantize_nvfp4.                        */
qii_status qii_absmax(const void *x, qii_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                      int transpose, int rht_group, uint64_t seed_rht, float *amax, void *stream);

/* Q(x) or Q(x^T) -> NVFP4 (Sec. 3.1 equations for QII_SR, Sec. 3.3 equations and
 * Algorithm 1 for QII_MS_EDEN, Table 1 "RTN 1x16" for QII_RTN, Sec. 4.1 for QII_RTN_46,
 * Sec. 7 "Post Hoc Range Alignment" for QII_MS_EDEN_PH).
 *   x          rows x cols, leading dimension ld >= cols (elements); with transpose == 0
 *              every row must start 16-byte aligned.
 *   transpose  0: quantize x, groups along cols;  out is rows x cols.
 *              1: quantize x^T, groups along rows of x;  out is cols x rows.
 *   rht_group  128: rotate chunks of 128 of the quantized dimension first (it must be
 *              a multiple of 128); 0: no rotation (it must be a multiple of 16).
 *   seed_rht, seed_sr  omega_RHT, omega_SR.  The output lives in ROTATED space and is
 *              meaningful only against a tensor rotated with the same seed_rht on the
 *              same inner dimension (the rotations cancel in the GEMM).
 *   amax_in    nullable.  Non-null: device float holding max|.| of the rotated tensor,
 *              supplied by the caller (App. D assumes this); the tensor is then read
 *              once.  Null: the library measures it first (a second read of x) and
 *              needs 256 bytes of workspace.  With QII_MS_EDEN_PH the tensor is read
 *              once either way (the maximum is reduced during the heavy pass unless
 *              supplied) and ws must hold qii_quantize_posthoc_workspace_bytes(out.rows,
 *              out.cols) bytes, 256-byte aligned.
 *   errors     QII_INVALID_ARG / QII_BAD_SHAPE / QII_WORKSPACE_TOO_SMALL before anything
 *              is launched; the outputs are then untouched.
 *   out        caller-allocated; out.rows/out.cols must equal the shape stated above. */
qii_status qii_quantize_nvfp4(const void *x, qii_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                              int transpose, qii_mode mode, int rht_group, uint64_t seed_rht,
                              uint64_t seed_sr, const float *amax_in, const qii_nvfp4 *out,
                              void *ws, size_t ws_bytes, void *stream);

/* Both orientations of one tensor from a single read (Sec. 5, backward pass: the output gradient
 * E is needed as Q(E) with groups along d_out and as Q(E^T) with groups along the tokens; Sec. 7
 * describes the backward quantizers as fused kernels around one load of their operand):
 *   out_rows = Q(x)    rows x cols, rotation seed_rht_rows, rounding seed_sr_rows
 *   out_cols = Q(x^T)  cols x rows, rotation seed_rht_cols, rounding seed_sr_cols
 * with rotation groups of 128 on both (rows and cols must be multiples of 128), mode QII_MS_EDEN
 * (Algorithm 1: two abs-max passes, then one read for both outputs) or QII_MS_EDEN_PH (one heavy
 * pass that reads x once, then the two scales-only passes).  The bytes are those of the two
 * qii_quantize_nvfp4 calls with the same seeds.  bf16 sources with 16-byte aligned rows take the
 * single-read kernel; anything else falls back to the two separate quantizers.  ws:
 * qii_quantize_pair_workspace_bytes(rows, cols, mode) bytes, 256-byte aligned.               */
qii_status qii_quantize_pair_nvfp4(const void *x, qii_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                                   qii_mode mode, uint64_t seed_rht_rows, uint64_t seed_sr_rows,
                                   uint64_t seed_rht_cols, uint64_t seed_sr_cols, const qii_nvfp4 *out_rows,
                                   const qii_nvfp4 *out_cols, void *ws, size_t ws_bytes, void *stream);

/* qii_quantize_nvfp4 for callers that cannot allocate device memory or bring a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the abs-max
 * scalar and, for QII_MS_EDEN_PH, the per-group f32 buffer live in a buffer of 16 MiB + 16 KiB
 * that the library holds in each GPU's memory from load time to the end of the process.  The
 * tensor's maximum is always measured by the call (there is no amax_in).  Arguments, outputs and
 * errors as qii_quantize_nvfp4; in addition QII_UNSUPPORTED for QII_MS_EDEN_PH on a tensor of more
 * than 4194304 scale groups (8192 x 8192 elements); the other modes take any size.  Allocates
 * nothing.  All calls on one GPU share that GPU's buffer: calls that overlap in time on the same
 * GPU (different streams or threads) race; calls ordered on one stream do not.                 */
qii_status qii_quantize_nvfp4_noalloc(const void *x, qii_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                                      int transpose, qii_mode mode, int rht_group, uint64_t seed_rht,
                                      uint64_t seed_sr, const qii_nvfp4 *out, void *stream);

/* Backward-pass re-quantization of a saved forward tensor (Sec. 5, "Backward Pass"):
 * dequantize `in` ((code*scale)*tensor_scale in f32), optionally transpose, quantize
 * as above.  in and out must not overlap.                                             */
qii_status qii_requantize_nvfp4(const qii_nvfp4 *in, int transpose, qii_mode mode, int rht_group,
                                uint64_t seed_rht, uint64_t seed_sr, const float *amax_in,
                                const qii_nvfp4 *out, void *ws, size_t ws_bytes, void *stream);

/* y[r][c] = (e2m1 * e4m3) * tensor_scale as f32, rows x cols contiguous.              */
qii_status qii_dequantize_nvfp4(const qii_nvfp4 *in, float *y, void *stream);

/* Block-scaled GEMM of Sec. 5:  C = A_hat * B_hat^T  with A (M x K) and B (N x K) both
 * K-contiguous NVFP4, products accumulated in f32.  C is M x N, leading dimension ldc,
 * dtype QII_F32 or QII_BF16 (rounded to nearest even from the f32 accumulator).
 * K = A.cols = B.cols is any multiple of 16 (NVFP4's own rule).  ws (nullable):
 * qii_gemm_workspace_bytes bytes, 16-byte aligned; with it (and K a multiple of 256) the fast
 * kernel runs, which first copies the scale bytes into a tile-contiguous layout and, when the
 * number of 256 x 256 output tiles leaves the last round of the grid mostly idle, shares those
 * tiles between blocks (f32 partial tiles in ws, added in a fixed order: results do not depend on
 * timing).  Without ws a slower kernel is used; with a ws too small for the partial tiles, one
 * block per tile.  Either way every product is formed exactly and accumulated in f32.
 * errors: QII_INVALID_ARG / QII_BAD_SHAPE before anything is launched; C is then untouched. */
qii_status qii_gemm_nvfp4(const qii_nvfp4 *A, const qii_nvfp4 *B, void *C, qii_dtype c_dt,
                          int64_t ldc, void *ws, size_t ws_bytes, void *stream);

/* The same GEMM that also emits max |C| (over the values as stored in C, i.e. after rounding to
 * c_dt) into the device float amax_c: the abs-max the next quantizer of C needs (Sec. 3.1 / 3.3,
 * numerator of x^FP32) comes out of the producing kernel, as App. D assumes, instead of costing
 * one more read of C.  amax_c == NULL gives qii_gemm_nvfp4.  With M * N == 0 it receives 0.   */
qii_status qii_gemm_nvfp4_amax(const qii_nvfp4 *A, const qii_nvfp4 *B, void *C, qii_dtype c_dt,
                               int64_t ldc, float *amax_c, void *ws, size_t ws_bytes, void *stream);

/* Forward pass of one linear layer (Sec. 5): Xq = RTN(X) and Wq = RTN(W) with 1x16
 * scales along d_in and no rotation, Y = Xq * Wq^T.  X is T x d_in, W is d_out x d_in,
 * Y is T x d_out (contiguous, dtype y_dt).  Xq_saved (T x d_in) and Wq_saved
 * (d_out x d_in) are caller-allocated and are the state kept for the backward pass.
 * d_in must be a multiple of 16.  All arguments of the pass (inputs, outputs, descriptors,
 * workspace) are checked before the first launch; on an error nothing has been written.  */
qii_status qii_linear_fwd(const void *X, const void *W, qii_dtype dt, int64_t T, int64_t d_in,
                          int64_t d_out, void *Y, qii_dtype y_dt, const qii_nvfp4 *Xq_saved,
                          const qii_nvfp4 *Wq_saved, void *ws, size_t ws_bytes, void *stream);

/* The same forward pass with the rounding scheme of X and W chosen by the caller:
 * QII_RTN (as qii_linear_fwd) or QII_RTN_46, the forward pass of Sec. 5 with the 4/6
 * choice of Sec. 4.1.  Other modes are rejected (the forward pass is deterministic).
 * amax_x, amax_w (each nullable): device floats holding max|X| and max|W|, for callers
 * that have them from the producing kernel (App. D assumes so); the matching abs-max
 * pass is then skipped.                                                                */
qii_status qii_linear_fwd_mode(const void *X, const void *W, qii_dtype dt, int64_t T, int64_t d_in,
                               int64_t d_out, qii_mode mode, const float *amax_x, const float *amax_w,
                               void *Y, qii_dtype y_dt, const qii_nvfp4 *Xq_saved,
                               const qii_nvfp4 *Wq_saved, void *ws, size_t ws_bytes, void *stream);

/* qii_linear_fwd_mode that also emits max |Y| into the device float amax_y (nullable), from the
 * GEMM's epilogue: a stack of layers passes it as amax_x of the layer that consumes Y, which then
 * needs no abs-max pass over its input (App. D).                                          */
qii_status qii_linear_fwd_amax(const void *X, const void *W, qii_dtype dt, int64_t T, int64_t d_in,
                               int64_t d_out, qii_mode mode, const float *amax_x, const float *amax_w,
                               void *Y, qii_dtype y_dt, float *amax_y, const qii_nvfp4 *Xq_saved,
                               const qii_nvfp4 *Wq_saved, void *ws, size_t ws_bytes, void *stream);

/* Backward pass of one linear layer (Sec. 5): with six sub-seeds derived from `seed`
 * (0: rotation of the dX GEMM, 1: rotation of the dW GEMM, 2..5: rounding seeds of
 * Q(E), Q(W^T), Q(E^T), Q(X^T)), all quantizers MS-EDEN:
 *   dX = Q(E) * Q(W^T)^T   (T x d_in,    inner dimension d_out)
 *   dW = Q(E^T) * Q(X^T)^T (d_out x d_in, inner dimension T)
 * dY is T x d_out (dtype dt).  T and d_out must be multiples of 128 and non-zero.
 * dX, dW contiguous, dtype g_dt.  All arguments of the pass are checked before the first
 * launch; on an error nothing has been written.                                        */
qii_status qii_linear_bwd(const void *dY, qii_dtype dt, const qii_nvfp4 *Xq_saved,
                          const qii_nvfp4 *Wq_saved, uint64_t seed, void *dX, void *dW,
                          qii_dtype g_dt, void *ws, size_t ws_bytes, void *stream);

/* The same backward pass with the scheme of its four quantizers chosen by the caller:
 * QII_MS_EDEN (as qii_linear_bwd: an abs-max pass and a quantize pass per tensor) or
 * QII_MS_EDEN_PH (Sec. 7: one heavy pass and a scales-only pass per tensor).  Workspace:
 * qii_linear_bwd_mode_workspace_bytes.  Other modes are rejected.                       */
qii_status qii_linear_bwd_mode(const void *dY, qii_dtype dt, const qii_nvfp4 *Xq_saved,
                               const qii_nvfp4 *Wq_saved, uint64_t seed, qii_mode mode, void *dX,
                               void *dW, qii_dtype g_dt, void *ws, size_t ws_bytes, void *stream);

/* Workspace sizes in bytes (host computations, no device work).                       */
size_t qii_quantize_workspace_bytes(void);
/* for mode QII_MS_EDEN_PH; rows x cols is the shape of the quantized output            */
size_t qii_quantize_posthoc_workspace_bytes(int64_t rows, int64_t cols);
size_t qii_quantize_pair_workspace_bytes(int64_t rows, int64_t cols, qii_mode mode);
size_t qii_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
size_t qii_linear_fwd_workspace_bytes(int64_t T, int64_t d_in, int64_t d_out);
size_t qii_linear_bwd_workspace_bytes(int64_t T, int64_t d_in, int64_t d_out);
size_t qii_linear_bwd_mode_workspace_bytes(int64_t T, int64_t d_in, int64_t d_out, qii_mode mode);

/* Device self-test (a maintenance aid, not an operation of the paper).  The tuned kernels
 * realise the rounding rules of Sec. 3.1 / Sec. 3.3 with gfx950 conversion instructions and
 * take their divisions as short Newton sequences; this call sweeps them against the rules
 * they stand for and writes the number of disagreeing inputs into counts[0..7] (device):
 *   0 FP4 encode (round to nearest even, saturating, sign kept): every finite binary32
 *   1 E4M3 encode on [0, 448]: every binary32 in the interval
 *   2 FP4 decode: every byte, all four byte positions
 *   3 the GEMM's FP4 x E4M3 -> f16 dequantization: 16 codes x 127 scale bytes, exact products
 *   4 division by a tensor constant, 5 general short division: 2^30 pseudo-random pairs each
 *   6 E4M3 decode: every byte     7 reciprocals over 81 binades: every binary32 there
 * All eight must read 0.  Takes a few hundred milliseconds.                              */
qii_status qii_selftest_conversions(uint64_t *counts, void *stream);

/* Exploratory NON-EXACT variants of qii_gemm_nvfp4 (measurement only; no other entry point of the
 * library reaches them, and their results do not meet the tolerance of the exact GEMM).  They show
 * what gfx950's native block-scaled matrix instruction (one power-of-two scale per 32 elements of
 * K) delivers when NVFP4's numerics (Sec. 5: products of the dequantized operands) are given up:
 *   QII_INEXACT_FP8       operand elements rounded to FP8 E4M3 relative to a power-of-two scale per
 *                         32 elements of K
 *   QII_INEXACT_FP4_POW2  FP4 codes as they are, each group's E4M3 scale rounded to the nearest
 *                         power of two, groups zero-padded to the instruction's 32-element scale
 *                         blocks
 * K must be a multiple of 64.
 * Arguments as qii_gemm_nvfp4; ws: qii_gemm_inexact_workspace_bytes(M, N, K, variant) bytes, 256-byte
 * aligned, required (it receives both operands re-encoded).  Errors as qii_gemm_nvfp4, plus
 * QII_BAD_SHAPE for a K the variant does not take.                                         */
typedef enum QII_ENUM_INT { QII_INEXACT_FP8 = 0, QII_INEXACT_FP4_POW2 = 1 } qii_inexact_variant;
qii_status qii_gemm_nvfp4_inexact(const qii_nvfp4 *A, const qii_nvfp4 *B, void *C, qii_dtype c_dt, int64_t ldc,
                                  qii_inexact_variant variant, void *ws, size_t ws_bytes, void *stream);
size_t qii_gemm_inexact_workspace_bytes(int64_t M, int64_t N, int64_t K, qii_inexact_variant variant);

/* Microbenchmarks of the machine limits the kernels are measured against (a measurement aid,
 * not an operation of the paper): one launch per call, timed by the caller with events.
 *   a, b   device buffers (see the kinds); n bytes, a multiple of 16
 *   blocks grid size in blocks of 256 threads (1..2^20); iters loop trips of the issue-rate kinds
 * Kinds: EMPTY no work (launch floor); COPY a -> b, READ a, WRITE b: n bytes in 16-byte words,
 * grid-stride; QUANT_TRAFFIC the loads and stores of the rows quantizer on an [n/16384][8192] bf16
 * matrix at a without its arithmetic (n a multiple of 262144; b holds n/4 + n/32 bytes; the grid
 * is derived from n); QUANT_TRAFFIC_COLS the same for the columns quantizer on an 8192 x 8192 bf16
 * matrix (n must be 134217728); VALU_FMA 16 independent v_fma_f32 per trip; VALU_RHT one 16-element slice
 * of the 128-point rotation per lane and trip (128 vector instructions); VALU_CVT_FP4 8 FP4
 * conversions per trip; VALU_CVT_F16_FP4 8 FP4 -> f16 conversions, VALU_PK_MUL_F16 16 packed f16
 * products per trip; MFMA_DEQUANT the GEMM's inner loop without its memory side, one wave per SIMD
 * (16 matrix instructions per trip, each followed by a dequantization chunk of 2 conversions
 * and 2 packed products: n = 1 all 16 as in the GEMM, n = 2 the first 8 only, n = 0 none, n = 3 the work that
 * codes packed as E2M3 would need instead, 2 conversions of 32 values and 32 packed products per
 * trip, n = 4 none again but with operands that change from one matrix instruction to the next, as
 * real data does; iters even); VALU_CVT_PK32_F16_FP6 2 conversions of 32 E2M3 values per trip; MFMA_F16 4 v_mfma_f32_32x32x16_f16 per wave and trip; ATOMIC_ONE_WORD one
 * atomic maximum per block on a[0]; ATOMIC_SPREAD the same over 64 words 256 bytes apart (a holds
 * 16 KiB).  Buffers a kind does not name may be NULL.                                    */
typedef enum QII_ENUM_INT {
    QII_MB_EMPTY = 0, QII_MB_COPY = 1, QII_MB_READ = 2, QII_MB_WRITE = 3, QII_MB_QUANT_TRAFFIC = 4,
    QII_MB_VALU_FMA = 5, QII_MB_VALU_RHT = 6, QII_MB_VALU_CVT_FP4 = 7, QII_MB_MFMA_F16 = 8,
    QII_MB_ATOMIC_ONE_WORD = 9, QII_MB_ATOMIC_SPREAD = 10, QII_MB_QUANT_TRAFFIC_COLS = 11,
    QII_MB_VALU_CVT_F16_FP4 = 12, QII_MB_VALU_PK_MUL_F16 = 13, QII_MB_MFMA_DEQUANT = 14,
    QII_MB_VALU_CVT_PK32_F16_FP6 = 15
} qii_microbench_kind;
qii_status qii_microbench(int kind, void *a, void *b, uint64_t n, int blocks, int iters, void *stream);

/* Test aids for the GEMM's shared last round (host computations, no device work): the index
 * arithmetic the kernels use, callable on a CPU so that it can be checked by brute force.
 * qii_gemm_sharing_plan: plan[0] = launch positions run one block per output tile, plan[1] = tiles
 *   after them that are shared between blocks (0: none), plan[2] = number of sharing blocks, for a
 *   GEMM of M x N x K whose workspace has qii_gemm_workspace_bytes.
 * qii_gemm_sharing_segments: the tile segments of the block with hardware id block_id when `grid`
 *   blocks share `rem` tiles of `ktotal` K tiles each; out receives 5 numbers per segment (block
 *   number, shared tile, first K tile, K tiles, partial-tile slot); returns the number of segments
 *   (at most 4 are written; -1 if there would be more; QII-style errors do not apply: arguments must
 *   satisfy 0 < rem, 8 <= ktotal, 0 < grid, 0 <= block_id < grid).
 * qii_gemm_sharing_tile_slots: out[0], out[1] = first and last slot that are added up for shared
 *   tile lt, in this order.                                                               */
void qii_gemm_sharing_plan(int64_t M, int64_t N, int64_t K, int32_t plan[3]);
int qii_gemm_sharing_segments(int rem, int ktotal, int grid, int block_id, int32_t *out);
void qii_gemm_sharing_tile_slots(int rem, int ktotal, int grid, int lt, int32_t out[2]);

/* Host helpers.                                                                        */
uint64_t qii_derive_seed(uint64_t seed, uint32_t i); /* backward sub-seed i (0..5)      */
const char *qii_status_string(qii_status s);
const char *qii_last_error(void);
int qii_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QII_H */
