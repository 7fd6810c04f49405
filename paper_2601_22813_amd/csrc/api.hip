// C ABI of libqii (see include/qii.h): argument validation, workspace carving and the
// kernel sequences of the layer's forward and backward pass (paper Sec. 5).
#include <stdarg.h>
#include <stdio.h>

#include <mutex>

#include "qii_device.h"
#include "qii_internal.h"
#include "quantize_core.h"

namespace {

thread_local char g_err[512] = "";

qii_status fail(qii_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

qii_status hip_fail(hipError_t e, const char *what)
{
    return fail(QII_HIP_ERROR, "%s: %s", what, hipGetErrorString(e));
}

constexpr size_t kSlot = 256;  // bytes reserved per device scalar in a workspace
constexpr size_t kRegion = qii::kAmaxRegionBytes;   // the spread running maximum of the post hoc scheme (16 KiB)
size_t align_up(size_t v) { return (v + kSlot - 1) / kSlot * kSlot; }
bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

qii_status check_nvfp4(const qii_nvfp4 *t, const char *name)
{
    if (!t) return fail(QII_INVALID_ARG, "%s: null descriptor", name);
    if (t->rows < 0 || t->cols < 0 || t->cols % 16 != 0)
        return fail(QII_BAD_SHAPE, "%s: %lld x %lld (cols must be a multiple of 16)", name,
                    (long long)t->rows, (long long)t->cols);
    if (t->rows * t->cols > 0) {
        if (!t->codes || !t->scales || !t->tensor_scale)
            return fail(QII_INVALID_ARG, "%s: null buffer", name);
        if (!aligned(t->codes, 16) || !aligned(t->scales, 8) || !aligned(t->tensor_scale, 4))
            return fail(QII_INVALID_ARG, "%s: misaligned buffer (codes 16, scales 8, tensor_scale 4)", name);
    }
    return QII_OK;
}

// checks the dense source and fills a Source descriptor plus the logical shape
qii_status dense_source(const void *x, qii_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                        int transpose, int rht_group, qii::Source *src, int64_t *R, int64_t *C)
{
    if (dt != QII_F32 && dt != QII_BF16) return fail(QII_INVALID_ARG, "bad dtype %d", (int)dt);
    if (rows < 0 || cols < 0 || ld < cols) return fail(QII_BAD_SHAPE, "rows %lld cols %lld ld %lld", (long long)rows, (long long)cols, (long long)ld);
    if (rht_group != 0 && rht_group != 128) return fail(QII_INVALID_ARG, "rht_group must be 0 or 128");
    *R = transpose ? cols : rows;
    *C = transpose ? rows : cols;
    const int64_t need = rht_group == 128 ? 128 : 16;
    if (*C % need != 0)
        return fail(QII_BAD_SHAPE, "quantized dimension %lld is not a multiple of %lld", (long long)*C, (long long)need);
    if (rows * cols > 0) {
        if (!x) return fail(QII_INVALID_ARG, "null input");
        const size_t esz = dt == QII_F32 ? 4 : 2;
        if (!aligned(x, esz)) return fail(QII_INVALID_ARG, "misaligned input");
        if (!transpose && (!aligned(x, 16) || (ld * esz) % 16 != 0))
            return fail(QII_INVALID_ARG, "input rows must be 16-byte aligned");
    }
    src->kind = dt == QII_F32 ? qii::kSrcF32 : qii::kSrcBF16;
    src->transpose = transpose ? 1 : 0;
    src->x = x;
    src->scales = nullptr;
    src->ts = nullptr;
    src->ld = ld;
    return QII_OK;
}

qii_status nvfp4_source(const qii_nvfp4 *in, int transpose, int rht_group, qii::Source *src,
                        int64_t *R, int64_t *C)
{
    qii_status st = check_nvfp4(in, "in");
    if (st != QII_OK) return st;
    if (rht_group != 0 && rht_group != 128) return fail(QII_INVALID_ARG, "rht_group must be 0 or 128");
    *R = transpose ? in->cols : in->rows;
    *C = transpose ? in->rows : in->cols;
    const int64_t need = rht_group == 128 ? 128 : 16;
    if (*C % need != 0)
        return fail(QII_BAD_SHAPE, "quantized dimension %lld is not a multiple of %lld", (long long)*C, (long long)need);
    src->kind = qii::kSrcNVFP4;
    src->transpose = transpose ? 1 : 0;
    src->x = in->codes;
    src->scales = in->scales;
    src->ts = in->tensor_scale;
    src->ld = in->cols;
    return QII_OK;
}

// measure (if needed) and quantize one logical R x C source
qii_status quantize_source(const qii::Source &src, int64_t R, int64_t C, qii_mode mode, int rht_group,
                           uint64_t seed_rht, uint64_t seed_sr, const float *amax_in,
                           const qii_nvfp4 *out, float *amax_slot, float *tbuf, hipStream_t s,
                           bool slot_zeroed = false, bool tiled_scales = false, uint8_t *tiled_copy = nullptr)
{
    // tiled_copy (modes other than the post hoc scheme, no rotation, a dense source read along its rows,
    // C a multiple of 256): the scale bytes are written there a second time, in the GEMM kernel's layout
    // tiled_scales (post hoc scheme only, C a multiple of 256, out->scales with room for R rounded up
    // to 256 rows): the scale bytes go out in the layout the main GEMM kernel reads
    if (mode != QII_RTN && mode != QII_SR && mode != QII_MS_EDEN && mode != QII_RTN_46 && mode != QII_MS_EDEN_PH)
        return fail(QII_INVALID_ARG, "bad mode %d", (int)mode);
    qii_status st = check_nvfp4(out, "out");
    if (st != QII_OK) return st;
    if (out->rows != R || out->cols != C)
        return fail(QII_BAD_SHAPE, "out is %lld x %lld, expected %lld x %lld", (long long)out->rows,
                    (long long)out->cols, (long long)R, (long long)C);
    if (R * C == 0) return QII_OK;
    if (mode == QII_MS_EDEN_PH) {
        // Sec. 7: heavy pass (codes, corrected pseudo-scales, running maximum), then scales only
        if (!tbuf) return fail(QII_WORKSPACE_TOO_SMALL, "the post hoc scheme needs qii_quantize_posthoc_workspace_bytes of workspace");
        if (!amax_in && !slot_zeroed) {   // the running maximum is spread over 64 words of its region
            hipError_t e = qii::launch_fill_u32(reinterpret_cast<uint32_t *>(amax_slot), 0u, (int)qii::kAmaxSpread, (int)qii::kAmaxStrideWords, s);
            if (e != hipSuccess) return hip_fail(e, "fill");
        }
        qii::QuantizeArgs a;
        a.src = src; a.R = R; a.C = C; a.mode = (int)mode; a.rht = rht_group == 128;
        a.seed_rht = seed_rht; a.seed_sr = seed_sr; a.amax = nullptr;
        a.codes = out->codes; a.scales = out->scales; a.tensor_scale = out->tensor_scale;
        a.tbuf = tbuf; a.amax_accum = amax_in ? nullptr : reinterpret_cast<uint32_t *>(amax_slot);
        hipError_t e = qii::launch_quantize(a, s);
        if (e != hipSuccess) return hip_fail(e, "quantize (heavy pass)");
        e = qii::launch_posthoc_scales(tbuf, amax_in ? amax_in : amax_slot, amax_in ? 1 : (int)qii::kAmaxSpread, R, C, seed_sr,
                                       out->scales, out->tensor_scale, s, tiled_scales);
        if (e != hipSuccess) return hip_fail(e, "quantize (scales pass)");
        return QII_OK;
    }
    if (tiled_scales) return fail(QII_INVALID_ARG, "tiled scales are written by the post hoc scheme only");
    const float *amax = amax_in;
    if (!amax) {
        if (!amax_slot) return fail(QII_WORKSPACE_TOO_SMALL, "workspace needed to measure the abs-max");
        hipError_t e = hipSuccess;
        if (!slot_zeroed) e = qii::launch_fill_u32(reinterpret_cast<uint32_t *>(amax_slot), 0u, 1, 1, s);
        if (e != hipSuccess) return hip_fail(e, "fill");
        e = qii::launch_absmax(src, R, C, rht_group == 128, seed_rht, amax_slot, s);
        if (e != hipSuccess) return hip_fail(e, "absmax");
        amax = amax_slot;
    }
    qii::QuantizeArgs a;
    a.src = src; a.R = R; a.C = C; a.mode = (int)mode; a.rht = rht_group == 128;
    a.seed_rht = seed_rht; a.seed_sr = seed_sr; a.amax = amax;
    a.codes = out->codes; a.scales = out->scales; a.tensor_scale = out->tensor_scale;
    a.tbuf = nullptr; a.amax_accum = nullptr;
    a.scales_tiled = tiled_copy;
    hipError_t e = qii::launch_quantize(a, s);
    if (e != hipSuccess) return hip_fail(e, "quantize");
    return QII_OK;
}

// workspace of one quantizer call: [abs-max slot][post hoc scheme only: one f32 per group]
qii_status carve_quantize_ws(qii_mode mode, const float *amax_in, int64_t R, int64_t C, void *ws,
                             size_t ws_bytes, float **slot, float **tbuf)
{
    *slot = nullptr;
    *tbuf = nullptr;
    if (mode == QII_MS_EDEN_PH) {
        const size_t need = kRegion + align_up((size_t)(R * (C / 16)) * 4);
        if (!ws || ws_bytes < need || !aligned(ws, kSlot))
            return fail(QII_WORKSPACE_TOO_SMALL, "the post hoc scheme needs %zu bytes of 256-byte aligned workspace", need);
        *slot = reinterpret_cast<float *>(ws);
        *tbuf = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(ws) + kRegion);
        return QII_OK;
    }
    if (!amax_in) {
        if (!ws || ws_bytes < kSlot || !aligned(ws, 4))
            return fail(QII_WORKSPACE_TOO_SMALL, "need %zu bytes of workspace without amax_in", kSlot);
        *slot = reinterpret_cast<float *>(ws);
    }
    return QII_OK;
}

// the two quantizer front ends on caller-carved workspace pieces (layer passes: their abs-max
// slots are cleared by one launch for the whole pass)
qii_status quantize_dense(const void *x, qii_dtype dt, int64_t rows, int64_t cols, int64_t ld, int transpose,
                          qii_mode mode, int rht_group, uint64_t seed_rht, uint64_t seed_sr,
                          const float *amax_in, const qii_nvfp4 *out, float *slot, float *tbuf, hipStream_t s,
                          bool slot_zeroed)
{
    qii::Source src;
    int64_t R, C;
    qii_status st = dense_source(x, dt, rows, cols, ld, transpose, rht_group, &src, &R, &C);
    if (st != QII_OK) return st;
    return quantize_source(src, R, C, mode, rht_group, seed_rht, seed_sr, amax_in, out, slot, tbuf, s, slot_zeroed);
}

qii_status requantize_saved(const qii_nvfp4 *in, int transpose, qii_mode mode, int rht_group, uint64_t seed_rht,
                            uint64_t seed_sr, const qii_nvfp4 *out, float *slot, float *tbuf, hipStream_t s,
                            bool slot_zeroed, bool tiled_scales = false)
{
    qii::Source src;
    int64_t R, C;
    qii_status st = nvfp4_source(in, transpose, rht_group, &src, &R, &C);
    if (st != QII_OK) return st;
    return quantize_source(src, R, C, mode, rht_group, seed_rht, seed_sr, nullptr, out, slot, tbuf, s, slot_zeroed, tiled_scales);
}

// quantizer workspace of a backward pass: four abs-max areas plus, for the post hoc scheme, the
// per-group f32 buffers (two of T x d_out / 16, or one of d_in x max(d_out, T) / 16 if that is larger)
size_t posthoc_region_bytes(int64_t T, int64_t d_in, int64_t d_out, qii_mode mode)
{
    if (mode != QII_MS_EDEN_PH) return 4 * kSlot;
    // Q(E) and Q(E^T) are produced together and need a buffer each; the two re-quantizations reuse the first
    const size_t e_bytes = 2 * align_up((size_t)(T * (d_out / 16)) * 4);
    int64_t groups = d_in * d_out / 16;
    if (d_in * T / 16 > groups) groups = d_in * T / 16;
    const size_t r_bytes = align_up((size_t)groups * 4);
    return 4 * kRegion + (e_bytes > r_bytes ? e_bytes : r_bytes);
}

// an NVFP4 tensor inside a workspace; its scale area has room for the row count rounded up to 256
// (the tiled scale layout of the main GEMM kernel)
size_t nvfp4_bytes(int64_t rows, int64_t cols)
{
    return align_up((size_t)(rows * cols / 2)) + align_up((size_t)((rows + 255) / 256 * 256 * cols / 16)) + kSlot;
}

qii_nvfp4 carve_nvfp4(uint8_t *&p, int64_t rows, int64_t cols)
{
    qii_nvfp4 t;
    t.codes = p; p += align_up((size_t)(rows * cols / 2));
    t.scales = p; p += align_up((size_t)((rows + 255) / 256 * 256 * cols / 16));
    t.tensor_scale = reinterpret_cast<float *>(p); p += kSlot;
    t.rows = rows; t.cols = cols;
    return t;
}

// ---- library-owned scratch for qii_quantize_nvfp4_noalloc ---------------------------------
// One abs-max slot plus one f32 per scale group of the post hoc scheme, for tensors of up to
// kScratchGroups groups.  Every GPU the library runs on holds its own copy of the array at its
// own address for the life of the process; in host code the array's name is only a handle for
// hipGetSymbolAddress, never a device address.
constexpr int64_t kScratchGroups = (int64_t)1 << 22;                       // 8192 x 8192 elements
constexpr size_t kScratchBytes = kRegion + (size_t)kScratchGroups * 4;     // 16 MiB + 16 KiB
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// device address of the current device's copy of `scratch` (looked up once per device)
qii_status scratch_address(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(QII_UNSUPPORTED, "device index %d beyond %d", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!p) return fail(QII_HIP_ERROR, "hipGetSymbolAddress(scratch) returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return QII_OK;
}

// Q(x) and Q(x^T) of one dense matrix (MS-EDEN or its post hoc form, rotation over 128).  slots:
// two abs-max areas (256 bytes each, or two 16 KiB regions for the post hoc scheme), tbufs: two
// per-group buffers (post hoc scheme).  Uses the single-read kernel where it applies, else the two
// quantizers one after the other.  All arguments have been validated by the caller.
qii_status quantize_pair(const qii::Source &src, int64_t rows, int64_t cols, qii_mode mode, uint64_t seed_rht_r,
                         uint64_t seed_sr_r, uint64_t seed_rht_c, uint64_t seed_sr_c, const qii_nvfp4 *out_r,
                         const qii_nvfp4 *out_c, float *slot_r, float *slot_c, float *tbuf_r, float *tbuf_c,
                         hipStream_t s, bool slots_zeroed, bool tiled_r = false, bool tiled_c = false)
{
    qii::Source srct = src;
    srct.transpose = 1;
    if (rows * cols == 0 || !qii::pair_kernel_applies(src, rows, cols)) {
        qii_status st = quantize_source(src, rows, cols, mode, 128, seed_rht_r, seed_sr_r, nullptr, out_r, slot_r, tbuf_r, s, slots_zeroed, tiled_r);
        if (st != QII_OK) return st;
        return quantize_source(srct, cols, rows, mode, 128, seed_rht_c, seed_sr_c, nullptr, out_c, slot_c, tbuf_c, s, slots_zeroed, tiled_c);
    }
    const bool ph = mode == QII_MS_EDEN_PH;
    if ((tiled_r || tiled_c) && !ph) return fail(QII_INVALID_ARG, "tiled scales are written by the post hoc scheme only");
    hipError_t e = hipSuccess;
    if (!slots_zeroed) {
        e = ph ? qii::launch_fill_u32(reinterpret_cast<uint32_t *>(slot_r), 0u, (int)qii::kAmaxSpread, (int)qii::kAmaxStrideWords, s)
               : qii::launch_fill_u32(reinterpret_cast<uint32_t *>(slot_r), 0u, 1, 1, s);
        if (e != hipSuccess) return hip_fail(e, "fill");
        e = ph ? qii::launch_fill_u32(reinterpret_cast<uint32_t *>(slot_c), 0u, (int)qii::kAmaxSpread, (int)qii::kAmaxStrideWords, s)
               : qii::launch_fill_u32(reinterpret_cast<uint32_t *>(slot_c), 0u, 1, 1, s);
        if (e != hipSuccess) return hip_fail(e, "fill");
    }
    if (!ph) {   // Algorithm 1 needs both rotated maxima before any scale: two abs-max passes, then one read for both outputs
        e = qii::launch_absmax(src, rows, cols, 1, seed_rht_r, slot_r, s);
        if (e != hipSuccess) return hip_fail(e, "absmax");
        e = qii::launch_absmax(srct, cols, rows, 1, seed_rht_c, slot_c, s);
        if (e != hipSuccess) return hip_fail(e, "absmax");
    }
    qii::PairQuantizeArgs p;
    p.src = src; p.rows = rows; p.cols = cols; p.mode = (int)mode;
    p.r = {seed_rht_r, seed_sr_r, ph ? nullptr : slot_r, out_r->codes, out_r->scales, out_r->tensor_scale, tbuf_r,
           ph ? reinterpret_cast<uint32_t *>(slot_r) : nullptr};
    p.c = {seed_rht_c, seed_sr_c, ph ? nullptr : slot_c, out_c->codes, out_c->scales, out_c->tensor_scale, tbuf_c,
           ph ? reinterpret_cast<uint32_t *>(slot_c) : nullptr};
    e = qii::launch_quantize_pair(p, s);
    if (e != hipSuccess) return hip_fail(e, "quantize (both orientations)");
    if (ph) {
        e = qii::launch_posthoc_scales(tbuf_r, slot_r, (int)qii::kAmaxSpread, rows, cols, seed_sr_r, out_r->scales, out_r->tensor_scale, s, tiled_r);
        if (e != hipSuccess) return hip_fail(e, "quantize (scales pass)");
        e = qii::launch_posthoc_scales(tbuf_c, slot_c, (int)qii::kAmaxSpread, cols, rows, seed_sr_c, out_c->scales, out_c->tensor_scale, s, tiled_c);
        if (e != hipSuccess) return hip_fail(e, "quantize (scales pass)");
    }
    return QII_OK;
}

size_t pair_ws_bytes(int64_t rows, int64_t cols, qii_mode mode)
{
    if (mode != QII_MS_EDEN_PH) return 2 * kSlot;
    return 2 * kRegion + 2 * align_up((size_t)(rows * (cols / 16)) * 4);
}

// every argument rule of the GEMM, checked before anything is launched
qii_status check_gemm_args(const qii_nvfp4 *A, const qii_nvfp4 *B, const void *C, qii_dtype c_dt, int64_t ldc)
{
    qii_status st = check_nvfp4(A, "A");
    if (st != QII_OK) return st;
    st = check_nvfp4(B, "B");
    if (st != QII_OK) return st;
    if (A->cols != B->cols) return fail(QII_BAD_SHAPE, "inner dimensions differ: %lld vs %lld", (long long)A->cols, (long long)B->cols);
    if (c_dt != QII_F32 && c_dt != QII_BF16) return fail(QII_INVALID_ARG, "bad output dtype");
    if (ldc < B->rows) return fail(QII_BAD_SHAPE, "ldc %lld < N %lld", (long long)ldc, (long long)B->rows);
    if (A->rows * B->rows == 0) return QII_OK;
    if (!C) return fail(QII_INVALID_ARG, "null C");
    if (!aligned(C, c_dt == QII_BF16 ? 2 : 4)) return fail(QII_INVALID_ARG, "misaligned C");
    if (A->cols == 0) return fail(QII_BAD_SHAPE, "K = 0");
    return QII_OK;
}

}  // namespace

extern "C" {

int qii_version(void) { return 1; }

const char *qii_last_error(void) { return g_err; }

const char *qii_status_string(qii_status s)
{
    switch (s) {
        case QII_OK: return "QII_OK";
        case QII_INVALID_ARG: return "QII_INVALID_ARG";
        case QII_BAD_SHAPE: return "QII_BAD_SHAPE";
        case QII_UNSUPPORTED: return "QII_UNSUPPORTED";
        case QII_WORKSPACE_TOO_SMALL: return "QII_WORKSPACE_TOO_SMALL";
        case QII_HIP_ERROR: return "QII_HIP_ERROR";
    }
    return "QII_UNKNOWN";
}

uint64_t qii_derive_seed(uint64_t seed, uint32_t i)
{
    const qii::U4 w = qii::philox_seeded(seed, i, 0, 0, qii::kStreamDerive);
    return ((uint64_t)w.y << 32) | w.x;
}

size_t qii_quantize_workspace_bytes(void) { return kSlot; }

size_t qii_quantize_posthoc_workspace_bytes(int64_t rows, int64_t cols)
{
    return kRegion + align_up((size_t)(rows * (cols / 16)) * 4);
}

size_t qii_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K) { return align_up(qii::gemm_workspace_bytes(M, N, K)); }

size_t qii_linear_fwd_workspace_bytes(int64_t T, int64_t d_in, int64_t d_out)
{
    return 2 * kSlot + qii_gemm_workspace_bytes(T, d_out, d_in);
}

size_t qii_linear_bwd_mode_workspace_bytes(int64_t T, int64_t d_in, int64_t d_out, qii_mode mode)
{
    const size_t g1 = qii_gemm_workspace_bytes(T, d_in, d_out), g2 = qii_gemm_workspace_bytes(d_out, d_in, T);
    return posthoc_region_bytes(T, d_in, d_out, mode) + nvfp4_bytes(T, d_out) + nvfp4_bytes(d_in, d_out) +
           nvfp4_bytes(d_out, T) + nvfp4_bytes(d_in, T) + (g1 > g2 ? g1 : g2);
}

size_t qii_linear_bwd_workspace_bytes(int64_t T, int64_t d_in, int64_t d_out)
{
    return qii_linear_bwd_mode_workspace_bytes(T, d_in, d_out, QII_MS_EDEN);
}

qii_status qii_rht(const void *x, qii_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                   int transpose, uint64_t seed_rht, float *y, float *amax, void *stream)
{
    qii::Source src;
    int64_t R, C;
    qii_status st = dense_source(x, dt, rows, cols, ld, transpose, 128, &src, &R, &C);
    if (st != QII_OK) return st;
    if (R * C == 0) return QII_OK;
    if (!y || !aligned(y, 16)) return fail(QII_INVALID_ARG, "y must be non-null and 16-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    if (amax) {
        hipError_t e = qii::launch_fill_u32(reinterpret_cast<uint32_t *>(amax), 0u, 1, 1, s);
        if (e != hipSuccess) return hip_fail(e, "fill");
    }
    hipError_t e = qii::launch_rht(src, R, C, seed_rht, y, amax, s);
    if (e != hipSuccess) return hip_fail(e, "rht");
    return QII_OK;
}

qii_status qii_absmax(const void *x, qii_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                      int transpose, int rht_group, uint64_t seed_rht, float *amax, void *stream)
{
    qii::Source src;
    int64_t R, C;
    qii_status st = dense_source(x, dt, rows, cols, ld, transpose, rht_group, &src, &R, &C);
    if (st != QII_OK) return st;
    if (!amax) return fail(QII_INVALID_ARG, "null amax");
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = qii::launch_fill_u32(reinterpret_cast<uint32_t *>(amax), 0u, 1, 1, s);
    if (e != hipSuccess) return hip_fail(e, "fill");
    e = qii::launch_absmax(src, R, C, rht_group == 128, seed_rht, amax, s);
    if (e != hipSuccess) return hip_fail(e, "absmax");
    return QII_OK;
}

qii_status qii_quantize_nvfp4(const void *x, qii_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                              int transpose, qii_mode mode, int rht_group, uint64_t seed_rht,
                              uint64_t seed_sr, const float *amax_in, const qii_nvfp4 *out,
                              void *ws, size_t ws_bytes, void *stream)
{
    qii::Source src;
    int64_t R, C;
    qii_status st = dense_source(x, dt, rows, cols, ld, transpose, rht_group, &src, &R, &C);
    if (st != QII_OK) return st;
    float *slot, *tbuf;
    st = carve_quantize_ws(mode, amax_in, R, C, ws, ws_bytes, &slot, &tbuf);
    if (st != QII_OK) return st;
    return quantize_source(src, R, C, mode, rht_group, seed_rht, seed_sr, amax_in, out, slot, tbuf,
                           (hipStream_t)stream);
}

qii_status qii_quantize_nvfp4_noalloc(const void *x, qii_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                                      int transpose, qii_mode mode, int rht_group, uint64_t seed_rht,
                                      uint64_t seed_sr, const qii_nvfp4 *out, void *stream)
{
    qii::Source src;
    int64_t R, C;
    qii_status st = dense_source(x, dt, rows, cols, ld, transpose, rht_group, &src, &R, &C);
    if (st != QII_OK) return st;
    if (mode == QII_MS_EDEN_PH && R * (C / 16) > kScratchGroups)
        return fail(QII_UNSUPPORTED, "qii_quantize_nvfp4_noalloc: the post hoc scheme needs one f32 per scale group and "
                    "the library's scratch holds %lld; this tensor has %lld (use qii_quantize_nvfp4 with a workspace)",
                    (long long)kScratchGroups, (long long)(R * (C / 16)));
    void *base = nullptr;
    st = scratch_address(&base);
    if (st != QII_OK) return st;
    // the slot is cleared by quantize_source (a fill kernel); the per-group buffer is written in
    // full by the heavy pass before the scales pass reads it
    float *slot = reinterpret_cast<float *>(base);
    float *tbuf = mode == QII_MS_EDEN_PH ? reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(base) + kRegion) : nullptr;
    return quantize_source(src, R, C, mode, rht_group, seed_rht, seed_sr, nullptr, out, slot, tbuf,
                           (hipStream_t)stream);
}

size_t qii_quantize_pair_workspace_bytes(int64_t rows, int64_t cols, qii_mode mode) { return pair_ws_bytes(rows, cols, mode); }

qii_status qii_quantize_pair_nvfp4(const void *x, qii_dtype dt, int64_t rows, int64_t cols, int64_t ld, qii_mode mode,
                                   uint64_t seed_rht_rows, uint64_t seed_sr_rows, uint64_t seed_rht_cols,
                                   uint64_t seed_sr_cols, const qii_nvfp4 *out_rows, const qii_nvfp4 *out_cols,
                                   void *ws, size_t ws_bytes, void *stream)
{
    if (mode != QII_MS_EDEN && mode != QII_MS_EDEN_PH)
        return fail(QII_INVALID_ARG, "qii_quantize_pair_nvfp4 takes QII_MS_EDEN or QII_MS_EDEN_PH, not mode %d", (int)mode);
    qii::Source src, srct;
    int64_t R, C;
    qii_status st = dense_source(x, dt, rows, cols, ld, 0, 128, &src, &R, &C);
    if (st != QII_OK) return st;
    st = dense_source(x, dt, rows, cols, ld, 1, 128, &srct, &R, &C);
    if (st != QII_OK) return st;
    st = check_nvfp4(out_rows, "out_rows");
    if (st != QII_OK) return st;
    st = check_nvfp4(out_cols, "out_cols");
    if (st != QII_OK) return st;
    if (out_rows->rows != rows || out_rows->cols != cols || out_cols->rows != cols || out_cols->cols != rows)
        return fail(QII_BAD_SHAPE, "out_rows must be %lld x %lld and out_cols %lld x %lld", (long long)rows,
                    (long long)cols, (long long)cols, (long long)rows);
    const size_t need = pair_ws_bytes(rows, cols, mode);
    if (!ws || ws_bytes < need || !aligned(ws, kSlot))
        return fail(QII_WORKSPACE_TOO_SMALL, "qii_quantize_pair_nvfp4 needs %zu bytes of 256-byte aligned workspace", need);
    if (rows * cols == 0) return QII_OK;
    uint8_t *p = reinterpret_cast<uint8_t *>(ws);
    const bool ph = mode == QII_MS_EDEN_PH;
    const size_t area = ph ? kRegion : kSlot, tb = align_up((size_t)(rows * (cols / 16)) * 4);
    float *slot_r = reinterpret_cast<float *>(p), *slot_c = reinterpret_cast<float *>(p + area);
    float *tbuf_r = ph ? reinterpret_cast<float *>(p + 2 * area) : nullptr;
    float *tbuf_c = ph ? reinterpret_cast<float *>(p + 2 * area + tb) : nullptr;
    return quantize_pair(src, rows, cols, mode, seed_rht_rows, seed_sr_rows, seed_rht_cols, seed_sr_cols, out_rows,
                         out_cols, slot_r, slot_c, tbuf_r, tbuf_c, (hipStream_t)stream, false);
}

qii_status qii_requantize_nvfp4(const qii_nvfp4 *in, int transpose, qii_mode mode, int rht_group,
                                uint64_t seed_rht, uint64_t seed_sr, const float *amax_in,
                                const qii_nvfp4 *out, void *ws, size_t ws_bytes, void *stream)
{
    qii::Source src;
    int64_t R, C;
    qii_status st = nvfp4_source(in, transpose, rht_group, &src, &R, &C);
    if (st != QII_OK) return st;
    float *slot, *tbuf;
    st = carve_quantize_ws(mode, amax_in, R, C, ws, ws_bytes, &slot, &tbuf);
    if (st != QII_OK) return st;
    return quantize_source(src, R, C, mode, rht_group, seed_rht, seed_sr, amax_in, out, slot, tbuf,
                           (hipStream_t)stream);
}

qii_status qii_dequantize_nvfp4(const qii_nvfp4 *in, float *y, void *stream)
{
    qii_status st = check_nvfp4(in, "in");
    if (st != QII_OK) return st;
    if (in->rows * in->cols == 0) return QII_OK;
    if (!y || !aligned(y, 16)) return fail(QII_INVALID_ARG, "y must be non-null and 16-byte aligned");
    hipError_t e = qii::launch_dequantize(in->codes, in->scales, in->tensor_scale, in->rows, in->cols,
                                          y, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "dequantize");
    return QII_OK;
}

qii_status qii_gemm_nvfp4_amax(const qii_nvfp4 *A, const qii_nvfp4 *B, void *C, qii_dtype c_dt,
                               int64_t ldc, float *amax_c, void *ws, size_t ws_bytes, void *stream)
{
    const qii_status st = check_gemm_args(A, B, C, c_dt, ldc);
    if (st != QII_OK) return st;
    if (amax_c && !aligned(amax_c, 4)) return fail(QII_INVALID_ARG, "misaligned amax_c");
    hipError_t e = qii::launch_gemm(*A, *B, C, c_dt == QII_BF16, ldc, amax_c, ws, ws_bytes, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "gemm");
    return QII_OK;
}

}  // extern "C"

namespace {
// the GEMM of a layer pass on operands quantized into the pass's workspace, whose scales may
// already be in the tiled layout (pretiled: bit 0 for A, bit 1 for B)
qii_status gemm_internal(const qii_nvfp4 *A, const qii_nvfp4 *B, void *C, qii_dtype c_dt, int64_t ldc, void *ws,
                         size_t ws_bytes, void *stream, int pretiled)
{
    const qii_status st = check_gemm_args(A, B, C, c_dt, ldc);
    if (st != QII_OK) return st;
    hipError_t e = qii::launch_gemm(*A, *B, C, c_dt == QII_BF16, ldc, nullptr, ws, ws_bytes, (hipStream_t)stream, pretiled);
    if (e != hipSuccess) return hip_fail(e, "gemm");
    return QII_OK;
}
}  // namespace

extern "C" {

qii_status qii_gemm_nvfp4(const qii_nvfp4 *A, const qii_nvfp4 *B, void *C, qii_dtype c_dt,
                          int64_t ldc, void *ws, size_t ws_bytes, void *stream)
{
    return qii_gemm_nvfp4_amax(A, B, C, c_dt, ldc, nullptr, ws, ws_bytes, stream);
}

qii_status qii_linear_fwd_amax(const void *X, const void *W, qii_dtype dt, int64_t T, int64_t d_in,
                               int64_t d_out, qii_mode mode, const float *amax_x, const float *amax_w,
                               void *Y, qii_dtype y_dt, float *amax_y, const qii_nvfp4 *Xq,
                               const qii_nvfp4 *Wq, void *ws, size_t ws_bytes, void *stream);

qii_status qii_linear_fwd_mode(const void *X, const void *W, qii_dtype dt, int64_t T, int64_t d_in,
                               int64_t d_out, qii_mode mode, const float *amax_x, const float *amax_w,
                               void *Y, qii_dtype y_dt, const qii_nvfp4 *Xq,
                               const qii_nvfp4 *Wq, void *ws, size_t ws_bytes, void *stream)
{
    return qii_linear_fwd_amax(X, W, dt, T, d_in, d_out, mode, amax_x, amax_w, Y, y_dt, nullptr, Xq, Wq, ws, ws_bytes, stream);
}

qii_status qii_linear_fwd_amax(const void *X, const void *W, qii_dtype dt, int64_t T, int64_t d_in,
                               int64_t d_out, qii_mode mode, const float *amax_x, const float *amax_w,
                               void *Y, qii_dtype y_dt, float *amax_y, const qii_nvfp4 *Xq,
                               const qii_nvfp4 *Wq, void *ws, size_t ws_bytes, void *stream)
{
    // every argument of the whole pass is checked before the first launch
    if (amax_y && !aligned(amax_y, 4)) return fail(QII_INVALID_ARG, "misaligned amax_y");
    if (mode != QII_RTN && mode != QII_RTN_46)
        return fail(QII_INVALID_ARG, "the forward pass takes QII_RTN or QII_RTN_46, not mode %d", (int)mode);
    if (T < 0 || d_in < 0 || d_out < 0) return fail(QII_BAD_SHAPE, "negative dimension");
    qii::Source sx, sw;
    int64_t R, C;
    qii_status st = dense_source(X, dt, T, d_in, d_in, 0, 0, &sx, &R, &C);
    if (st != QII_OK) return st;
    st = dense_source(W, dt, d_out, d_in, d_in, 0, 0, &sw, &R, &C);
    if (st != QII_OK) return st;
    st = check_nvfp4(Xq, "Xq_saved");
    if (st != QII_OK) return st;
    st = check_nvfp4(Wq, "Wq_saved");
    if (st != QII_OK) return st;
    if (Xq->rows != T || Xq->cols != d_in || Wq->rows != d_out || Wq->cols != d_in)
        return fail(QII_BAD_SHAPE, "Xq_saved must be %lld x %lld and Wq_saved %lld x %lld", (long long)T,
                    (long long)d_in, (long long)d_out, (long long)d_in);
    st = check_gemm_args(Xq, Wq, Y, y_dt, d_out);
    if (st != QII_OK) return st;
    if (!ws || ws_bytes < qii_linear_fwd_workspace_bytes(T, d_in, d_out) || !aligned(ws, kSlot))
        return fail(QII_WORKSPACE_TOO_SMALL, "linear_fwd needs %zu bytes of 256-byte aligned workspace",
                    qii_linear_fwd_workspace_bytes(T, d_in, d_out));
    uint8_t *p = reinterpret_cast<uint8_t *>(ws);
    hipStream_t s = (hipStream_t)stream;
    float *slots = reinterpret_cast<float *>(p);
    const int slot_words = (int)(kSlot / 4);
    if ((!amax_x || !amax_w) && (T * d_in > 0 || d_out * d_in > 0)) {
        hipError_t e = qii::launch_fill_u32(reinterpret_cast<uint32_t *>(slots), 0u, 2, slot_words, s);
        if (e != hipSuccess) return hip_fail(e, "fill");
    }
    // When the GEMM will take its main kernel (d_in a multiple of 256) the two quantizers also write
    // their scale bytes straight into the GEMM workspace in that kernel's tiled layout: no re-tiling launch.
    uint8_t *gws = p + 2 * kSlot;
    const bool tile = d_in % 256 == 0 && T * d_out > 0 && qii::rows_kernels_apply(sx, T, d_in) && qii::rows_kernels_apply(sw, d_out, d_in);
    uint8_t *x_tiled = tile ? gws : nullptr, *w_tiled = tile ? gws + (T + 255) / 256 * 256 * (d_in / 16) : nullptr;
    st = quantize_source(sx, T, d_in, mode, 0, 0, 0, amax_x, Xq, slots, nullptr, s, true, false, x_tiled);
    if (st != QII_OK) return st;
    st = quantize_source(sw, d_out, d_in, mode, 0, 0, 0, amax_w, Wq, slots + slot_words, nullptr, s, true, false, w_tiled);
    if (st != QII_OK) return st;
    // (the GEMM's arguments were checked above, before the first launch)
    hipError_t e = qii::launch_gemm(*Xq, *Wq, Y, y_dt == QII_BF16, d_out, amax_y, gws, ws_bytes - 2 * kSlot, s, tile ? 12 : 0);
    if (e != hipSuccess) return hip_fail(e, "gemm");
    return QII_OK;
}

qii_status qii_linear_fwd(const void *X, const void *W, qii_dtype dt, int64_t T, int64_t d_in,
                          int64_t d_out, void *Y, qii_dtype y_dt, const qii_nvfp4 *Xq,
                          const qii_nvfp4 *Wq, void *ws, size_t ws_bytes, void *stream)
{
    return qii_linear_fwd_mode(X, W, dt, T, d_in, d_out, QII_RTN, nullptr, nullptr, Y, y_dt, Xq, Wq, ws, ws_bytes, stream);
}

qii_status qii_linear_bwd_mode(const void *dY, qii_dtype dt, const qii_nvfp4 *Xq, const qii_nvfp4 *Wq,
                               uint64_t seed, qii_mode mode, void *dX, void *dW, qii_dtype g_dt, void *ws,
                               size_t ws_bytes, void *stream)
{
    if (mode != QII_MS_EDEN && mode != QII_MS_EDEN_PH)
        return fail(QII_INVALID_ARG, "the backward pass takes QII_MS_EDEN or QII_MS_EDEN_PH, not mode %d", (int)mode);
    qii_status st = check_nvfp4(Xq, "Xq_saved");
    if (st != QII_OK) return st;
    st = check_nvfp4(Wq, "Wq_saved");
    if (st != QII_OK) return st;
    const int64_t T = Xq->rows, d_in = Xq->cols, d_out = Wq->rows;
    if (Wq->cols != d_in) return fail(QII_BAD_SHAPE, "Xq is %lld x %lld but Wq is %lld x %lld", (long long)T, (long long)d_in, (long long)d_out, (long long)Wq->cols);
    if (T % 128 != 0 || d_out % 128 != 0) return fail(QII_BAD_SHAPE, "T and d_out must be multiples of 128");
    // every argument of the whole pass is checked before the first launch
    qii::Source se, set;
    int64_t R, C;
    st = dense_source(dY, dt, T, d_out, d_out, 0, 128, &se, &R, &C);
    if (st != QII_OK) return st;
    st = dense_source(dY, dt, T, d_out, d_out, 1, 128, &set, &R, &C);
    if (st != QII_OK) return st;
    if (g_dt != QII_F32 && g_dt != QII_BF16) return fail(QII_INVALID_ARG, "bad gradient dtype");
    if (T * d_in > 0 && (!dX || !aligned(dX, g_dt == QII_BF16 ? 2 : 4))) return fail(QII_INVALID_ARG, "dX is null or misaligned");
    if (d_out * d_in > 0 && (!dW || !aligned(dW, g_dt == QII_BF16 ? 2 : 4))) return fail(QII_INVALID_ARG, "dW is null or misaligned");
    if (T * d_out == 0) return fail(QII_BAD_SHAPE, "the backward pass needs a non-empty inner dimension (T and d_out)");
    const size_t need = qii_linear_bwd_mode_workspace_bytes(T, d_in, d_out, mode);
    if (!ws || ws_bytes < need || !aligned(ws, kSlot))
        return fail(QII_WORKSPACE_TOO_SMALL, "linear_bwd needs %zu bytes of 256-byte aligned workspace", need);
    uint8_t *p = reinterpret_cast<uint8_t *>(ws);
    // quantizer workspace: four abs-max slots, cleared by one launch, and, for the post hoc
    // scheme, one per-group f32 buffer sized for the largest tensor and used by the four
    // quantizers one after the other on the stream
    hipStream_t s = (hipStream_t)stream;
    float *slots = reinterpret_cast<float *>(p);
    const bool ph = mode == QII_MS_EDEN_PH;
    const int slot_words = (int)((ph ? kRegion : kSlot) / 4);   // distance between the four tensors' abs-max areas
    float *tbuf = ph ? reinterpret_cast<float *>(p + 4 * kRegion) : nullptr;
    float *tbuf2 = ph ? tbuf + align_up((size_t)(T * (d_out / 16)) * 4) / 4 : nullptr;   // second buffer for Q(E^T)
    p += posthoc_region_bytes(T, d_in, d_out, mode);
    qii_nvfp4 Eq = carve_nvfp4(p, T, d_out);
    qii_nvfp4 WTq = carve_nvfp4(p, d_in, d_out);
    qii_nvfp4 ETq = carve_nvfp4(p, d_out, T);
    qii_nvfp4 XTq = carve_nvfp4(p, d_in, T);
    void *gws = p;   // the two GEMMs run one after the other on the stream and share this region
    const size_t gws_bytes = reinterpret_cast<uint8_t *>(ws) + ws_bytes - p;
    uint64_t sd[6];
    for (uint32_t i = 0; i < 6; ++i) sd[i] = qii_derive_seed(seed, i);
    // (the post hoc scheme spreads each running maximum over 64 words, 256 bytes apart: the four
    // regions are contiguous, so one launch clears all 256 words)
    hipError_t e = ph ? qii::launch_fill_u32(reinterpret_cast<uint32_t *>(slots), 0u, 4 * (int)qii::kAmaxSpread, (int)qii::kAmaxStrideWords, s)
                      : qii::launch_fill_u32(reinterpret_cast<uint32_t *>(slots), 0u, 4, slot_words, s);
    if (e != hipSuccess) return hip_fail(e, "fill");
    // Q(E) and Q(E^T) from one read of dY: rotation sd[0] along d_out for the dX GEMM, sd[1] along
    // the tokens for the dW GEMM (their abs-max areas are the first and third of the four)
    // The four quantized operands live only in this workspace.  In the post hoc scheme their scale
    // bytes come from the scales pass, which writes them straight into the layout the main GEMM
    // kernel reads when the GEMM's inner dimension allows that kernel: no re-tiling launch.
    const bool tile_dx = ph && d_out % 256 == 0, tile_dw = ph && T % 256 == 0;
    st = quantize_pair(se, T, d_out, mode, sd[0], sd[2], sd[1], sd[4], &Eq, &ETq, slots, slots + 2 * slot_words, tbuf,
                       tbuf2, s, true, tile_dx, tile_dw);
    if (st != QII_OK) return st;
    // dX = Q(E) Q(W^T)^T : inner dimension d_out
    st = requantize_saved(Wq, 1, mode, 128, sd[0], sd[3], &WTq, slots + slot_words, tbuf, s, true, tile_dx);
    if (st != QII_OK) return st;
    st = gemm_internal(&Eq, &WTq, dX, g_dt, d_in, gws, gws_bytes, stream, tile_dx ? 3 : 0);
    if (st != QII_OK) return st;
    // dW = Q(E^T) Q(X^T)^T : inner dimension T
    st = requantize_saved(Xq, 1, mode, 128, sd[1], sd[5], &XTq, slots + 3 * slot_words, tbuf, s, true, tile_dw);
    if (st != QII_OK) return st;
    return gemm_internal(&ETq, &XTq, dW, g_dt, d_in, gws, gws_bytes, stream, tile_dw ? 3 : 0);
}

void qii_gemm_sharing_plan(int64_t M, int64_t N, int64_t K, int32_t plan[3])
{
    plan[0] = plan[1] = plan[2] = 0;
    if (M <= 0 || N <= 0 || K <= 0) return;
    qii::gemm_sharing_plan(M, N, K, plan);
}

int qii_gemm_sharing_segments(int rem, int ktotal, int grid, int block_id, int32_t *out)
{
    if (rem <= 0 || ktotal < 8 || grid <= 0 || block_id < 0 || block_id >= grid || !out) return -1;
    return qii::gemm_sharing_segments(rem, ktotal, grid, block_id, out);
}

void qii_gemm_sharing_tile_slots(int rem, int ktotal, int grid, int lt, int32_t out[2])
{
    out[0] = out[1] = -1;
    if (rem <= 0 || ktotal < 8 || grid <= 0 || lt < 0 || lt >= rem) return;
    qii::gemm_sharing_tile_slots(rem, ktotal, grid, lt, out);
}

qii_status qii_selftest_conversions(uint64_t *counts, void *stream)
{
    if (!counts || !aligned(counts, 8)) return fail(QII_INVALID_ARG, "counts must be 8 device uint64, 8-byte aligned");
    hipError_t e = qii::launch_selftest_conversions(reinterpret_cast<unsigned long long *>(counts), (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "selftest");
    return QII_OK;
}

size_t qii_gemm_inexact_workspace_bytes(int64_t M, int64_t N, int64_t K, qii_inexact_variant variant)
{
    if (variant != QII_INEXACT_FP8 && variant != QII_INEXACT_FP4_POW2) return 0;
    return align_up(qii::gemm_inexact_workspace_bytes(M, N, K, (int)variant));
}

qii_status qii_gemm_nvfp4_inexact(const qii_nvfp4 *A, const qii_nvfp4 *B, void *C, qii_dtype c_dt, int64_t ldc,
                                  qii_inexact_variant variant, void *ws, size_t ws_bytes, void *stream)
{
    if (variant != QII_INEXACT_FP8 && variant != QII_INEXACT_FP4_POW2) return fail(QII_INVALID_ARG, "bad variant %d", (int)variant);
    qii_status st = check_gemm_args(A, B, C, c_dt, ldc);
    if (st != QII_OK) return st;
    const int64_t slice = 64;
    if (A->cols % slice != 0) return fail(QII_BAD_SHAPE, "this variant needs K to be a multiple of %lld", (long long)slice);
    if (!aligned(A->scales, 8) || !aligned(B->scales, 8) || !aligned(A->codes, 16) || !aligned(B->codes, 16))
        return fail(QII_INVALID_ARG, "misaligned operand");
    const size_t need = qii_gemm_inexact_workspace_bytes(A->rows, B->rows, A->cols, variant);
    if (A->rows * B->rows != 0 && (!ws || ws_bytes < need || !aligned(ws, kSlot)))
        return fail(QII_WORKSPACE_TOO_SMALL, "qii_gemm_nvfp4_inexact needs %zu bytes of 256-byte aligned workspace", need);
    hipError_t e = qii::launch_gemm_inexact(*A, *B, C, c_dt == QII_BF16, ldc, (int)variant, ws, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "gemm (non-exact variant)");
    return QII_OK;
}

qii_status qii_microbench(int kind, void *a, void *b, uint64_t n, int blocks, int iters, void *stream)
{
    if (kind < QII_MB_EMPTY || kind > QII_MB_VALU_CVT_PK32_F16_FP6) return fail(QII_INVALID_ARG, "microbench: unknown kind");
    if (blocks < 1 || blocks > (1 << 20) || iters < 0) return fail(QII_INVALID_ARG, "microbench: blocks in 1..2^20, iters >= 0");
    const bool quant = kind == QII_MB_QUANT_TRAFFIC || kind == QII_MB_QUANT_TRAFFIC_COLS;
    const bool atomic = kind == QII_MB_ATOMIC_ONE_WORD || kind == QII_MB_ATOMIC_SPREAD;
    const bool needs_a = kind == QII_MB_COPY || kind == QII_MB_READ || quant || atomic;
    const bool needs_b = kind == QII_MB_COPY || kind == QII_MB_WRITE || quant;
    if ((needs_a && (!a || !aligned(a, 16))) || (needs_b && (!b || !aligned(b, 16))))
        return fail(QII_INVALID_ARG, "microbench: a buffer this kind uses is NULL or not 16-byte aligned");
    if ((needs_a || needs_b) && !atomic && (n == 0 || n % 16)) return fail(QII_BAD_SHAPE, "microbench: n must be a positive multiple of 16");
    if (kind == QII_MB_QUANT_TRAFFIC && (n % 262144 || n / 262144 > (1u << 20))) return fail(QII_BAD_SHAPE, "microbench: n must be a multiple of 262144 (16 rows of 8192 bf16)");
    if (kind == QII_MB_MFMA_DEQUANT && (n > 4 || (iters & 1))) return fail(QII_INVALID_ARG, "microbench: n must be 0..4 and iters even");
    if (kind == QII_MB_QUANT_TRAFFIC_COLS && n != 134217728u) return fail(QII_BAD_SHAPE, "microbench: n must be 134217728 (8192 x 8192 bf16)");
    hipError_t e = qii::launch_microbench(kind, a, b, n, blocks, iters, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "microbench");
    return QII_OK;
}

qii_status qii_linear_bwd(const void *dY, qii_dtype dt, const qii_nvfp4 *Xq, const qii_nvfp4 *Wq,
                          uint64_t seed, void *dX, void *dW, qii_dtype g_dt, void *ws,
                          size_t ws_bytes, void *stream)
{
    return qii_linear_bwd_mode(dY, dt, Xq, Wq, seed, QII_MS_EDEN, dX, dW, g_dt, ws, ws_bytes, stream);
}

}  // extern "C"
