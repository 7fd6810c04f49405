/* Sanitizer driver of the library's host code (argument checks, workspace arithmetic, helpers):
 * linked against a build of libqii whose host half is compiled with AddressSanitizer and
 * UndefinedBehaviorSanitizer (paper_2601_22813_amd/build.py: build_sanitized), it makes the calls
 * that return before anything is enqueued, so it needs no GPU.  Pointers such as 0x1000 are never
 * dereferenced by the host code; a sanitizer report would show that one was.
 * Built and run by tests/test_sanitizers.py.  Prints "abi sanitize: ok" and returns 0. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../include/qii.h"

static int fails = 0;
#define EXPECT(call, want)                                                                      \
    do {                                                                                        \
        const int got_ = (int)(call);                                                           \
        if (got_ != (int)(want)) {                                                              \
            fprintf(stderr, "line %d: %s returned %d (%s), expected %d\n", __LINE__, #call, got_, qii_last_error(), (int)(want)); \
            ++fails;                                                                            \
        }                                                                                       \
    } while (0)

#define P(x) ((void *)(uintptr_t)(x))

int main(void)
{
    /* helpers */
    if (qii_version() < 1) ++fails;
    for (int s = 0; s < 8; ++s)
        if (!qii_status_string((qii_status)s)) ++fails;
    volatile uint64_t sink = 0;
    for (uint32_t i = 0; i < 6; ++i) sink ^= qii_derive_seed(0xFFFFFFFFFFFFFFFFull, i) ^ qii_derive_seed(0, i);
    /* workspace sizes over small, ragged, large and degenerate shapes (size arithmetic must not overflow or shift out of range) */
    const int64_t dims[] = {0, 1, 16, 100, 128, 256, 384, 2048, 8192, 28672, 1 << 20};
    const int nd = (int)(sizeof dims / sizeof dims[0]);
    sink ^= qii_quantize_workspace_bytes();
    for (int a = 0; a < nd; ++a)
        for (int b = 0; b < nd; ++b) {
            sink ^= qii_quantize_posthoc_workspace_bytes(dims[a], dims[b]);
            for (int m = 0; m <= 5; ++m) sink ^= qii_quantize_pair_workspace_bytes(dims[a], dims[b], (qii_mode)m);
            for (int c = 0; c < nd; c += 2) {
                sink ^= qii_gemm_workspace_bytes(dims[a], dims[b], dims[c]);
                sink ^= qii_linear_fwd_workspace_bytes(dims[a], dims[b], dims[c]);
                sink ^= qii_linear_bwd_workspace_bytes(dims[a], dims[b], dims[c]);
                for (int m = 0; m <= 5; ++m) sink ^= qii_linear_bwd_mode_workspace_bytes(dims[a], dims[b], dims[c], (qii_mode)m);
            }
        }
    /* the GEMM's sharing plan and its index arithmetic (host-side test aids): every planned shape's segments stay in range */
    for (int a = 0; a < nd; ++a)
        for (int b = 0; b < nd; ++b)
            for (int c = 0; c < nd; ++c) {
                int32_t plan[3], seg[20], sl[2];
                qii_gemm_sharing_plan(dims[a], dims[b], dims[c], plan);
                if (plan[1] <= 0) continue;
                const int ktotal = (int)(dims[c] / 256);
                for (int id = 0; id < plan[2]; id += 1 + plan[2] / 7) {
                    const int n = qii_gemm_sharing_segments(plan[1], ktotal, plan[2], id, seg);
                    if (n < 1 || n > 2) ++fails;
                    for (int i = 0; i < n; ++i)
                        if (seg[5 * i + 1] < 0 || seg[5 * i + 1] >= plan[1] || seg[5 * i + 4] < 0 || seg[5 * i + 4] >= plan[1] + plan[2]) ++fails;
                }
                for (int lt = 0; lt < plan[1]; lt += 1 + plan[1] / 5) {
                    qii_gemm_sharing_tile_slots(plan[1], ktotal, plan[2], lt, sl);
                    if (sl[0] < 0 || sl[1] < sl[0] || sl[1] >= plan[1] + plan[2]) ++fails;
                }
            }
    {
        int32_t seg[20], sl[2];
        if (qii_gemm_sharing_segments(0, 8, 8, 0, seg) != -1 || qii_gemm_sharing_segments(4, 8, 8, 8, seg) != -1 ||
            qii_gemm_sharing_segments(4, 7, 8, 0, seg) != -1 || qii_gemm_sharing_segments(4, 8, 8, 0, NULL) != -1) ++fails;
        qii_gemm_sharing_tile_slots(4, 8, 8, 4, sl);
        if (sl[0] != -1) ++fails;
    }
    /* quantizer argument checks */
    qii_nvfp4 out = {P(0x1000), P(0x1000), P(0x1000), 4, 120};
    EXPECT(qii_quantize_nvfp4(P(0x1000), QII_BF16, 4, 120, 120, 0, QII_RTN, 0, 0, 0, NULL, &out, NULL, 0, NULL), QII_BAD_SHAPE);
    out.cols = 64;
    EXPECT(qii_quantize_nvfp4(P(0x1000), QII_BF16, 4, 64, 64, 0, QII_MS_EDEN, 128, 0, 0, NULL, &out, NULL, 0, NULL), QII_BAD_SHAPE);
    out.cols = 128;
    EXPECT(qii_quantize_nvfp4(P(0x1000), QII_BF16, 4, 128, 128, 0, (qii_mode)9, 128, 0, 0, P(0x2000), &out, NULL, 0, NULL), QII_INVALID_ARG);
    EXPECT(qii_quantize_nvfp4(P(0x1000), (qii_dtype)5, 4, 128, 128, 0, QII_MS_EDEN, 128, 0, 0, P(0x2000), &out, NULL, 0, NULL), QII_INVALID_ARG);
    EXPECT(qii_quantize_nvfp4(NULL, QII_BF16, 4, 128, 128, 0, QII_MS_EDEN, 128, 0, 0, P(0x2000), &out, NULL, 0, NULL), QII_INVALID_ARG);
    EXPECT(qii_quantize_nvfp4(P(0x1001), QII_BF16, 4, 128, 128, 0, QII_MS_EDEN, 128, 0, 0, P(0x2000), &out, NULL, 0, NULL), QII_INVALID_ARG);
    EXPECT(qii_quantize_nvfp4(P(0x1000), QII_BF16, 4, 128, 128, 1, QII_RTN, 0, 0, 0, P(0x2000), &out, NULL, 0, NULL), QII_BAD_SHAPE);
    EXPECT(qii_quantize_nvfp4(P(0x1000), QII_BF16, 4, 128, 128, 0, QII_MS_EDEN, 128, 0, 0, NULL, &out, NULL, 0, NULL), QII_WORKSPACE_TOO_SMALL);
    EXPECT(qii_quantize_nvfp4(P(0x1000), QII_BF16, 4, 128, 128, 0, QII_MS_EDEN_PH, 128, 0, 0, P(0x2000), &out, P(0x4000), 256, NULL), QII_WORKSPACE_TOO_SMALL);
    EXPECT(qii_quantize_nvfp4(P(0x1000), QII_BF16, 4, 128, 100, 0, QII_RTN, 0, 0, 0, P(0x2000), &out, NULL, 0, NULL), QII_BAD_SHAPE);
    EXPECT(qii_quantize_nvfp4(P(0x1000), QII_BF16, 4, 128, 128, 0, QII_RTN, 0, 0, 0, P(0x2000), NULL, NULL, 0, NULL), QII_INVALID_ARG);
    EXPECT(qii_quantize_nvfp4_noalloc(NULL, QII_BF16, 4, 128, 128, 0, QII_MS_EDEN, 128, 0, 0, &out, NULL), QII_INVALID_ARG);
    EXPECT(qii_quantize_nvfp4_noalloc(P(0x1000), QII_BF16, 4, 120, 120, 0, QII_MS_EDEN, 0, 0, 0, &out, NULL), QII_BAD_SHAPE);
    qii_nvfp4 empty = {NULL, NULL, NULL, 0, 128};
    EXPECT(qii_quantize_nvfp4(NULL, QII_BF16, 0, 128, 128, 0, QII_MS_EDEN, 128, 0, 0, P(0x2000), &empty, NULL, 0, NULL), QII_OK);
    qii_nvfp4 o2 = {P(0x1000), P(0x1000), P(0x1000), 128, 4};
    EXPECT(qii_quantize_pair_nvfp4(P(0x1000), QII_BF16, 4, 128, 128, QII_RTN, 0, 0, 0, 0, &out, &o2, P(0x4000), 1 << 20, NULL), QII_INVALID_ARG);
    EXPECT(qii_quantize_pair_nvfp4(P(0x1000), QII_BF16, 4, 128, 128, QII_MS_EDEN, 0, 0, 0, 0, &out, &o2, P(0x4000), 1 << 20, NULL), QII_BAD_SHAPE);
    EXPECT(qii_quantize_pair_nvfp4(P(0x1000), QII_BF16, 128, 128, 128, QII_MS_EDEN, 0, 0, 0, 0, &out, &o2, P(0x4000), 1 << 20, NULL), QII_BAD_SHAPE);
    EXPECT(qii_absmax(NULL, QII_BF16, 4, 128, 128, 0, 128, 0, P(0x2000), NULL), QII_INVALID_ARG);
    EXPECT(qii_absmax(P(0x1000), QII_BF16, 4, 100, 100, 0, 128, 0, P(0x2000), NULL), QII_BAD_SHAPE);
    EXPECT(qii_rht(P(0x1000), QII_F32, 4, 100, 100, 0, 0, P(0x3000), NULL, NULL), QII_BAD_SHAPE);
    EXPECT(qii_rht(P(0x1000), QII_F32, 4, 128, 128, 0, 0, NULL, NULL, NULL), QII_INVALID_ARG);
    EXPECT(qii_requantize_nvfp4(NULL, 1, QII_MS_EDEN, 128, 0, 0, NULL, &out, P(0x4000), 256, NULL), QII_INVALID_ARG);
    EXPECT(qii_requantize_nvfp4(&out, 1, QII_MS_EDEN, 128, 0, 0, NULL, &out, P(0x4000), 256, NULL), QII_BAD_SHAPE);
    EXPECT(qii_dequantize_nvfp4(&out, NULL, NULL), QII_INVALID_ARG);
    EXPECT(qii_dequantize_nvfp4(NULL, P(0x1000), NULL), QII_INVALID_ARG);
    /* GEMM argument checks */
    qii_nvfp4 a = {P(0x1000), P(0x1000), P(0x1000), 8, 64}, b = {P(0x1000), P(0x1000), P(0x1000), 8, 128};
    EXPECT(qii_gemm_nvfp4(&a, &b, P(0x3000), QII_F32, 8, NULL, 0, NULL), QII_BAD_SHAPE);
    a.cols = b.cols = 40;
    EXPECT(qii_gemm_nvfp4(&a, &b, P(0x3000), QII_F32, 8, NULL, 0, NULL), QII_BAD_SHAPE);
    a.cols = b.cols = 48;
    EXPECT(qii_gemm_nvfp4(&a, &b, P(0x3000), QII_F32, 7, NULL, 0, NULL), QII_BAD_SHAPE);
    EXPECT(qii_gemm_nvfp4(&a, &b, P(0x3000), (qii_dtype)7, 8, NULL, 0, NULL), QII_INVALID_ARG);
    EXPECT(qii_gemm_nvfp4(&a, &b, NULL, QII_F32, 8, NULL, 0, NULL), QII_INVALID_ARG);
    EXPECT(qii_gemm_nvfp4(&a, &b, P(0x3002), QII_F32, 8, NULL, 0, NULL), QII_INVALID_ARG);
    EXPECT(qii_gemm_nvfp4(NULL, &b, P(0x3000), QII_F32, 8, NULL, 0, NULL), QII_INVALID_ARG);
    EXPECT(qii_gemm_nvfp4_amax(&a, &b, P(0x3000), QII_F32, 8, P(0x5002), NULL, 0, NULL), QII_INVALID_ARG);
    EXPECT(qii_gemm_nvfp4_inexact(&a, &b, P(0x3000), QII_F32, 8, (qii_inexact_variant)5, P(0x4000), (size_t)1 << 30, NULL), QII_INVALID_ARG);
    EXPECT(qii_gemm_nvfp4_inexact(&a, &b, P(0x3000), QII_F32, 8, QII_INEXACT_FP8, P(0x4000), (size_t)1 << 30, NULL), QII_BAD_SHAPE);   /* K = 48 */
    a.cols = b.cols = 64;
    EXPECT(qii_gemm_nvfp4_inexact(&a, &b, P(0x3000), QII_F32, 8, QII_INEXACT_FP4_POW2, NULL, 0, NULL), QII_WORKSPACE_TOO_SMALL);
    EXPECT(qii_gemm_nvfp4_inexact(&a, &b, NULL, QII_F32, 8, QII_INEXACT_FP8, P(0x4000), (size_t)1 << 30, NULL), QII_INVALID_ARG);
    for (int a_ = 0; a_ < nd; ++a_)
        for (int c_ = 0; c_ < nd; c_ += 3)
            for (int v = 0; v <= 2; ++v) sink ^= qii_gemm_inexact_workspace_bytes(dims[a_], dims[nd - 1 - a_], dims[c_], (qii_inexact_variant)v);
    /* layer passes: everything is checked before the first launch */
    const int64_t T = 256, d_in = 128, d_out = 384;
    qii_nvfp4 xq = {P(0x10000), P(0x20000), P(0x30000), T, d_in}, wq = {P(0x40000), P(0x50000), P(0x60000), d_out, d_in};
    const size_t big = (size_t)1 << 30;
    EXPECT(qii_linear_fwd_mode(P(0x1000), P(0x2000), QII_BF16, T, d_in, d_out, QII_RTN, NULL, NULL, NULL, QII_BF16, &xq, &wq, P(0x100000), big, NULL), QII_INVALID_ARG);
    EXPECT(qii_linear_fwd_mode(P(0x1000), P(0x2000), QII_BF16, T, d_in, d_out, QII_MS_EDEN, NULL, NULL, P(0x3000), QII_BF16, &xq, &wq, P(0x100000), big, NULL), QII_INVALID_ARG);
    EXPECT(qii_linear_fwd_mode(NULL, P(0x2000), QII_BF16, T, d_in, d_out, QII_RTN, NULL, NULL, P(0x3000), QII_BF16, &xq, &wq, P(0x100000), big, NULL), QII_INVALID_ARG);
    EXPECT(qii_linear_fwd_mode(P(0x1000), P(0x2000), QII_BF16, T, d_in, d_out, QII_RTN, NULL, NULL, P(0x3000), QII_BF16, &xq, &wq, P(0x100000), 16, NULL), QII_WORKSPACE_TOO_SMALL);
    EXPECT(qii_linear_fwd_mode(P(0x1000), P(0x2000), QII_BF16, T, d_in, d_out, QII_RTN, NULL, NULL, P(0x3000), QII_BF16, &xq, &wq, P(0x100010), big, NULL), QII_WORKSPACE_TOO_SMALL);
    EXPECT(qii_linear_fwd(P(0x1000), P(0x2000), QII_BF16, T, d_in + 8, d_out, P(0x3000), QII_BF16, &xq, &wq, P(0x100000), big, NULL), QII_BAD_SHAPE);
    EXPECT(qii_linear_fwd_amax(P(0x1000), P(0x2000), QII_BF16, T, d_in, d_out, QII_RTN, NULL, NULL, P(0x3000), QII_BF16, P(0x7002), &xq, &wq, P(0x100000), big, NULL), QII_INVALID_ARG);
    EXPECT(qii_linear_bwd_mode(NULL, QII_BF16, &xq, &wq, 0, QII_MS_EDEN, P(0x3000), P(0x5000), QII_BF16, P(0x100000), big, NULL), QII_INVALID_ARG);
    EXPECT(qii_linear_bwd_mode(P(0x1000), QII_BF16, &xq, &wq, 0, QII_SR, P(0x3000), P(0x5000), QII_BF16, P(0x100000), big, NULL), QII_INVALID_ARG);
    EXPECT(qii_linear_bwd_mode(P(0x1000), QII_BF16, &xq, &wq, 0, QII_MS_EDEN, P(0x3000), NULL, QII_BF16, P(0x100000), big, NULL), QII_INVALID_ARG);
    EXPECT(qii_linear_bwd_mode(P(0x1000), QII_BF16, &xq, &wq, 0, QII_MS_EDEN_PH, P(0x3000), P(0x5000), QII_BF16, P(0x100000), 16, NULL), QII_WORKSPACE_TOO_SMALL);
    EXPECT(qii_linear_bwd(P(0x1000), QII_BF16, &xq, &wq, 0, P(0x3000), P(0x5000), QII_BF16, P(0x100000), 16, NULL), QII_WORKSPACE_TOO_SMALL);
    xq.rows = T + 64;
    EXPECT(qii_linear_bwd_mode(P(0x1000), QII_BF16, &xq, &wq, 0, QII_MS_EDEN, P(0x3000), P(0x5000), QII_BF16, P(0x100000), big, NULL), QII_BAD_SHAPE);
    /* maintenance entry points */
    EXPECT(qii_selftest_conversions(NULL, NULL), QII_INVALID_ARG);
    EXPECT(qii_selftest_conversions(P(0x1004), NULL), QII_INVALID_ARG);
    EXPECT(qii_microbench(99, NULL, NULL, 0, 1, 0, NULL), QII_INVALID_ARG);
    EXPECT(qii_microbench(QII_MB_COPY, NULL, P(0x1000), 1024, 1, 0, NULL), QII_INVALID_ARG);
    EXPECT(qii_microbench(QII_MB_COPY, P(0x1000), P(0x2000), 1000, 1, 0, NULL), QII_BAD_SHAPE);
    EXPECT(qii_microbench(QII_MB_EMPTY, NULL, NULL, 0, 0, 0, NULL), QII_INVALID_ARG);
    if (strlen(qii_last_error()) == 0) ++fails;
    if (fails) return 1;
    printf("abi sanitize: ok (%u)\n", (unsigned)(sink & 1u));
    return 0;
}
