/*
 * qii_oracle.c -- CPU oracle for the NVFP4 linear-layer path of Quartet II.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, scalar statement of
 * what the path computes, written from the paper.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.  It shares no code
 * with the HIP library and the HIP library never calls it.
 *
 * Arithmetic contract.  The quantizers decide integers (4-bit codes, scale
 * bytes) from floating point, so every step below is one IEEE binary32
 * operation (round to nearest even, denormals kept, no contraction) unless a
 * comment says "exact" or "double".  Compile with -ffp-contract=off and
 * without fast-math.  The GEMM has a plain definition and is done in double.
 *
 * Paper passages followed (section / equation / algorithm names only):
 *   Sec. 3.1  "NVFP4 and Stochastic Rounding": the format triple
 *             {FP4 elements, one FP8 E4M3 scale per 16, one FP32 scale} and
 *             the three equations of Q_SR (constants 6, 16/17, 448).
 *   Sec. 3.3  "Our Solution: Microscaling EDEN": Algorithm 1 (MS-EDEN) and
 *             the three equations of the clipping quantizer Q_RTN(x, s) with
 *             cap 256 and s = 6*(16/17)/0.93.
 *   Table 1   row "RTN 1x16": plain round-to-nearest NVFP4 (s = 6, cap 448).
 *   Sec. 4.1  "Forward Pass Using 4/6" and Table 1 row "+4/6": per block, the
 *             round-to-nearest quantization is done twice, with the block
 *             maximum mapped to 6 and to 4, and the one with the lower squared
 *             error is kept (mode RTN_46).
 *   Sec. 5    forward pass (RTN on X and W, save the quantized tensors) and
 *             backward pass (dequantize, transpose, re-quantize with MS-EDEN,
 *             MS-EDEN of E and E^T, two GEMMs; rotations cancel on the inner
 *             dimension).
 *   Sec. 7    "Post Hoc Range Alignment": MS-EDEN without knowing the tensor
 *             maximum in the heavy pass (mode MS_EDEN_PH): group scales are
 *             rounded to E8M3 (three mantissa bits, binary32 exponent range)
 *             instead of being aligned to the E4M3 range first, codes and EDEN
 *             factors follow from those pseudo-scales, and a second pass over
 *             the scales alone shifts them by the tensor scale and rounds them
 *             stochastically to E4M3.
 *   App. A    one rotation per tensor, shared by all its 128-chunks.
 *
 * Every function is pinned by tests/test_oracle_*.py against format
 * definitions, closed forms, brute force, library routines and Table 1.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define QO_RTN 0
#define QO_SR 1
#define QO_MS_EDEN 2
#define QO_RTN_46 3
#define QO_MS_EDEN_PH 4

#define QO_F32 0
#define QO_BF16 1

#define QO_OK 0
#define QO_BAD 1

/* Philox counter word 3 separates the uses of one seed. */
#define QO_STREAM_RHT 0x52485400u    /* the 128 rotation signs             */
#define QO_STREAM_SCALE 0x53434c00u  /* one draw per 16-group (MS-EDEN)    */
#define QO_STREAM_ELEM 0x454c4d00u   /* one draw per element (SR)          */
#define QO_STREAM_DERIVE 0x44525600u /* sub-seeds of the backward pass     */

/* ------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as  */
/* easy as 1, 2, 3", SC'11): the counter-based generator behind omega_RHT   */
/* and omega_SR of Algorithm 1.  key = the 64-bit seed.                     */
/* ------------------------------------------------------------------------ */
void qo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static void philox_seeded(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t out[4])
{
    uint32_t ctr[4] = {c0, c1, c2, c3};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    qo_philox4x32_10(ctr, key, out);
}

/* omega_RHT -> 128 signs: bit (j mod 32) of word (j div 32); 1 means -1.    */
void qo_rht_signs(uint64_t seed_rht, uint32_t signbits[4])
{
    philox_seeded(seed_rht, 0, 0, 0, QO_STREAM_RHT, signbits);
}

/* omega_SR -> the 20 random bits of scale group (row, cg): rows r..r+3 of   */
/* one column group share one generator call.                               */
uint32_t qo_scale_draw(uint64_t seed_sr, int64_t row, int64_t cg)
{
    uint32_t w[4];
    philox_seeded(seed_sr, (uint32_t)cg, (uint32_t)(row >> 2), 0, QO_STREAM_SCALE, w);
    return w[row & 3] >> 12;
}

/* omega_SR -> the 16 random bits of element (row, col): eight consecutive   */
/* columns share one generator call, low half-word first.                   */
uint32_t qo_elem_draw(uint64_t seed_sr, int64_t row, int64_t col)
{
    uint32_t w[4];
    philox_seeded(seed_sr, (uint32_t)(col >> 3), (uint32_t)row, 0, QO_STREAM_ELEM, w);
    uint32_t word = w[(col & 7) >> 1];
    return (col & 1) ? (word >> 16) : (word & 0xFFFFu);
}

/* Backward-pass sub-seed i (0..5) of one layer seed.                        */
uint64_t qo_derive_seed(uint64_t seed, uint32_t i)
{
    uint32_t w[4];
    philox_seeded(seed, i, 0, 0, QO_STREAM_DERIVE, w);
    return ((uint64_t)w[1] << 32) | w[0];
}

/* ------------------------------------------------------------------------ */
/* Number formats (Sec. 3.1).                                               */
/* ------------------------------------------------------------------------ */

/* E2M1: 1 sign, 2 exponent, 1 mantissa bit: magnitudes 0 .5 1 1.5 2 3 4 6. */
static const float E2M1_MAG[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};

float qo_e2m1_decode(uint8_t code)
{
    float m = E2M1_MAG[code & 7];
    return (code & 8) ? -m : m;
}

/* Index of the largest grid magnitude <= a (a >= 0, grid ascending).       */
static int floor_index(const float *grid, int n, float a)
{
    int i = 0;
    while (i + 1 < n && grid[i + 1] <= a) ++i;
    return i;
}

/* Round to nearest E2M1, ties to the even code, saturating at 6; the sign  */
/* bit of q is kept (so a small negative q gives the code of -0).           */
uint8_t qo_e2m1_rtn(float q)
{
    float a = fabsf(q);
    int lo = floor_index(E2M1_MAG, 8, a);
    int idx = lo;
    if (lo < 7) {
        double dlo = (double)a - (double)E2M1_MAG[lo];       /* exact */
        double dhi = (double)E2M1_MAG[lo + 1] - (double)a;   /* exact */
        if (dhi < dlo) idx = lo + 1;
        else if (dhi == dlo) idx = (lo & 1) ? lo + 1 : lo;
    }
    return (uint8_t)((signbit(q) ? 8 : 0) | idx);
}

/* Stochastic rounding to E2M1 (SR_FP4 of Sec. 3.1) with 16 random bits R:  */
/* with lo <= |q| < hi the grid neighbours and d = (|q|-lo)/(hi-lo) * 2^16, */
/* round up iff R + d >= 2^16, i.e. with probability floor(d)/2^16.         */
uint8_t qo_e2m1_sr(float q, uint32_t r16)
{
    float a = fabsf(q);
    int lo = floor_index(E2M1_MAG, 8, a);
    int idx = lo;
    if (lo < 7) {
        double d = ((double)a - (double)E2M1_MAG[lo]) /
                   ((double)E2M1_MAG[lo + 1] - (double)E2M1_MAG[lo]) * 65536.0;
        if ((double)(r16 & 0xFFFFu) + d >= 65536.0) idx = lo + 1;
    }
    return (uint8_t)((signbit(q) ? 8 : 0) | idx);
}

/* E4M3 (OCP "e4m3fn"): bias 7, 3 mantissa bits, subnormals m/8 * 2^-6,     */
/* largest finite value 448 = 0x7E; 0x7F is NaN and is never produced.      */
/* Scales are non-negative, so only bytes 0x00..0x7E occur.                 */
float qo_e4m3_decode(uint8_t b)
{
    int e = (b >> 3) & 15, m = b & 7;
    float v = (e == 0) ? ldexpf((float)m / 8.0f, -6) : ldexpf(1.0f + (float)m / 8.0f, e - 7);
    return (b & 0x80) ? -v : v;
}

static float E4M3_GRID[127];
static int e4m3_grid_ready = 0;
static void e4m3_grid_init(void)
{
    if (!e4m3_grid_ready) {
        for (int b = 0; b < 127; ++b) E4M3_GRID[b] = qo_e4m3_decode((uint8_t)b);
        e4m3_grid_ready = 1;
    }
}

/* RTN_FP8 of the scale equations: nearest E4M3 value of r >= 0, ties to    */
/* the even byte, saturating at 448.                                        */
uint8_t qo_e4m3_rtn(float r)
{
    e4m3_grid_init();
    if (!(r > 0.0f)) return 0;
    int lo = floor_index(E4M3_GRID, 127, r);
    if (lo == 126) return 0x7E;
    double dlo = (double)r - (double)E4M3_GRID[lo];       /* exact */
    double dhi = (double)E4M3_GRID[lo + 1] - (double)r;   /* exact */
    if (dhi < dlo) return (uint8_t)(lo + 1);
    if (dhi == dlo) return (uint8_t)((lo & 1) ? lo + 1 : lo);
    return (uint8_t)lo;
}

/* SR_FP8 of Algorithm 1 with 20 random bits R: with lo <= t < hi the E4M3  */
/* neighbours (0 and subnormals included) and d = (t-lo)/(hi-lo) * 2^20,    */
/* round up iff R + d >= 2^20.  t >= 448 saturates to 448.                  */
uint8_t qo_e4m3_sr(float t, uint32_t r20)
{
    e4m3_grid_init();
    if (!(t > 0.0f)) return 0;
    int lo = floor_index(E4M3_GRID, 127, t);
    if (lo == 126) return 0x7E;
    double d = ((double)t - (double)E4M3_GRID[lo]) /
               ((double)E4M3_GRID[lo + 1] - (double)E4M3_GRID[lo]) * 1048576.0;
    if ((double)(r20 & 0xFFFFFu) + d >= 1048576.0) return (uint8_t)(lo + 1);
    return (uint8_t)lo;
}

static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* ------------------------------------------------------------------------ */
/* Randomized Hadamard transform over one chunk of 128 (Algorithm 1, first  */
/* loop): y = H (d .* v) / sqrt(128), H the Sylvester matrix                */
/* H[i][j] = (-1)^popcount(i & j), d the sign vector of omega_RHT.          */
/* Butterfly stages run over index bits 0,1,..,6 in that order; every       */
/* add/sub and the final scaling is one rounded binary32 operation.  The    */
/* scaling is written as fma(v, 2^-3.5, +0): same value, but a result that  */
/* is exactly zero comes out as +0 whatever signs of zero met on the way    */
/* (the paper leaves the sign of a zero open; both FP4 zeros decode to 0).  */
/* ------------------------------------------------------------------------ */
static void rht128(float *v, const uint32_t signbits[4])
{
    for (int j = 0; j < 128; ++j)
        if ((signbits[j >> 5] >> (j & 31)) & 1u) v[j] = -v[j];
    for (int len = 1; len < 128; len <<= 1)
        for (int i = 0; i < 128; ++i)
            if ((i & len) == 0) {
                float a = v[i], b = v[i + len];
                v[i] = a + b;
                v[i + len] = a - b;
            }
    const float inv_sqrt_128 = 0x1.6a09e6p-4f; /* binary32 nearest to 2^-3.5 */
    for (int j = 0; j < 128; ++j) v[j] = fmaf(v[j], inv_sqrt_128, 0.0f);
}

/* The logical matrix the quantizer works on: x (rows x cols, leading       */
/* dimension ld, f32 or bf16) or its transpose, widened to f32 (exact),     */
/* then rotated chunk by chunk along its rows when rht_group == 128.        */
/* out is R x C with (R, C) = (rows, cols) or (cols, rows).                 */
static int build_rotated(const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld,
                         int transpose, int rht_group, uint64_t seed_rht, float *out)
{
    int64_t R = transpose ? cols : rows, C = transpose ? rows : cols;
    if (rows < 0 || cols < 0 || ld < cols) return QO_BAD;
    if (rht_group != 0 && rht_group != 128) return QO_BAD;
    if (C % 16 != 0 || (rht_group == 128 && C % 128 != 0)) return QO_BAD;
    if (dtype != QO_F32 && dtype != QO_BF16) return QO_BAD;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r)
        for (int64_t c = 0; c < C; ++c) {
            int64_t src = transpose ? c * ld + r : r * ld + c;
            out[r * C + c] = (dtype == QO_F32) ? ((const float *)x)[src]
                                               : bf16_to_f32(((const uint16_t *)x)[src]);
        }
    if (rht_group == 128) {
        uint32_t signbits[4];
        qo_rht_signs(seed_rht, signbits);
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < R; ++r)
            for (int64_t h = 0; h < C; h += 128) rht128(out + r * C + h, signbits);
    }
    return QO_OK;
}

static float tensor_absmax(const float *y, int64_t n)
{
    float amax = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        float a = fabsf(y[i]);
        if (a > amax) amax = a;
    }
    return amax;
}

/* y = rotated (and possibly transposed) x as f32; amax (nullable) = max|y|. */
int qo_rht(const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld, int transpose,
           int rht_group, uint64_t seed_rht, float *y, float *amax)
{
    int rc = build_rotated(x, dtype, rows, cols, ld, transpose, rht_group, seed_rht, y);
    if (rc != QO_OK) return rc;
    if (amax) *amax = tensor_absmax(y, rows * cols);
    return QO_OK;
}

/* Grid max s and scale cap of each mode:                                   */
/*   RTN     (Table 1, "RTN 1x16")        s = 6,             cap 448        */
/*   SR      (Sec. 3.1, Q_SR)             s = 6*16/17,       cap 448        */
/*   MS-EDEN (Sec. 3.3, Q_RTN(x, s))      s = 6*16/17/0.93,  cap 256        */
/*   RTN+4/6 (Sec. 4.1)                   s = 6 (and 4),     cap 256: the   */
/*           scale of a block mapped to 4 is 1.5 times that of the same     */
/*           block mapped to 6, and 1.5 * 256 = 384 still is an E4M3 value  */
/* s_override > 0 replaces s (Algorithm 1 takes s as an input).             */
static void mode_constants(int mode, float s_override, float *s, float *cap)
{
    if (mode == QO_RTN) { *s = 6.0f; *cap = 448.0f; }
    else if (mode == QO_RTN_46) { *s = 6.0f; *cap = 256.0f; }
    else if (mode == QO_MS_EDEN_PH) { *s = (float)(96.0 / 17.0 / 0.93); *cap = 256.0f; }
    else if (mode == QO_SR) { *s = (float)(96.0 / 17.0); *cap = 448.0f; }
    else { *s = (float)(96.0 / 17.0 / 0.93); *cap = 256.0f; }
    if (s_override > 0.0f) *s = s_override;
}

/* One candidate of the 4/6 choice (Sec. 4.1): round the 16 values of a      */
/* group to nearest with the group maximum mapped to `level` (6 or 4).      */
/* Returns the scale byte, the codes (8 bytes) and the squared error of the */
/* de-quantized group: d_i = x_i - c_i * (x^FP8 * x^FP32) as one fused      */
/* multiply-add, summed as a fused multiply-add chain in index order.       */
static uint8_t rtn_candidate(const float *yg, float gmax, float x32, float level, uint8_t *cg,
                             float *err_out)
{
    uint8_t b = qo_e4m3_rtn(gmax / (x32 * level));
    float err = 0.0f;
    memset(cg, 0, 8);
    if (b == 0) { /* scale under-flowed: all codes zero, error = <x, x> */
        for (int k = 0; k < 16; ++k) err = fmaf(yg[k], yg[k], err);
        *err_out = err;
        return 0;
    }
    const float p = qo_e4m3_decode(b) * x32;
    const float inv = 1.0f / p;
    for (int k = 0; k < 16; ++k) {
        uint8_t code = qo_e2m1_rtn(yg[k] * inv);
        float d = fmaf(-qo_e2m1_decode(code), p, yg[k]);
        err = fmaf(d, d, err);
        if (k & 1) cg[k >> 1] |= (uint8_t)(code << 4);
        else cg[k >> 1] = code;
    }
    *err_out = err;
    return b;
}

/* E8M3 (Sec. 7): a non-negative binary32 rounded to three mantissa bits,     */
/* nearest even, exponent range unchanged ("extended-range" stand-in for E4M3).*/
float qo_e8m3_rtn(float u)
{
    uint32_t b;
    memcpy(&b, &u, 4);
    b = (b + 0x7FFFFu + ((b >> 20) & 1u)) & 0xFFF00000u;
    memcpy(&u, &b, 4);
    return u;
}

/* MS-EDEN with post hoc range alignment (Sec. 7), in the paper's two passes. */
/* Pass 1 needs no tensor maximum: pseudo-scale p_g = RTN_E8M3(max_g|x| / s),  */
/* codes RTN_FP4(x_i / p_g), and the corrected pseudo-scale                   */
/*   t_g = S_g * p_g = <x,x> / <x, x^FP4>   (p_g cancels; t_g = p_g if the     */
/*   denominator is not positive), kept in binary32.                          */
/* Pass 2 reads only t_g and the tensor maximum: x^FP32 = max|x| / (s * 256), */
/* scale byte = SR_E4M3(t_g / x^FP32) with the same draw as Algorithm 1.      */
static void quantize_rotated_posthoc(const float *y, int64_t R, int64_t C, float s, float cap,
                                     float amax, uint64_t seed_sr, uint8_t *codes, uint8_t *scales,
                                     float *tensor_scale)
{
    int64_t G = C / 16;
    float *t = (float *)malloc(sizeof(float) * (size_t)(R * G > 0 ? R * G : 1));
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r)
        for (int64_t g = 0; g < G; ++g) {
            const float *yg = y + r * C + g * 16;
            uint8_t *cg = codes + (r * C + g * 16) / 2;
            float gmax = 0.0f;
            for (int k = 0; k < 16; ++k) {
                float a = fabsf(yg[k]);
                if (a > gmax) gmax = a;
            }
            const float p = qo_e8m3_rtn(gmax / s);
            memset(cg, 0, 8);
            if (!(p > 0.0f)) { /* all-zero group (or a maximum that rounds to nothing) */
                t[r * G + g] = 0.0f;
                continue;
            }
            const float inv = 1.0f / p;
            float num = 0.0f, den = 0.0f;
            for (int k = 0; k < 16; ++k) {
                uint8_t code = qo_e2m1_rtn(yg[k] * inv);
                if (k & 1) cg[k >> 1] |= (uint8_t)(code << 4);
                else cg[k >> 1] = code;
                num = fmaf(yg[k], yg[k], num);
                den = fmaf(yg[k], qo_e2m1_decode(code), den);
            }
            t[r * G + g] = den > 0.0f ? num / den : p;
        }
    if (!(amax > 0.0f)) {
        *tensor_scale = 1.0f;
        memset(scales, 0, (size_t)(R * G));
    } else {
        const float x32 = amax / (s * cap);
        *tensor_scale = x32;
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < R; ++r)
            for (int64_t g = 0; g < G; ++g) {
                scales[r * G + g] = qo_e4m3_sr(t[r * G + g] / x32, qo_scale_draw(seed_sr, r, g));
            }
    }
    free(t);
}

/* Quantize an already rotated R x C f32 matrix y, groups of 16 along rows. */
static void quantize_rotated(const float *y, int64_t R, int64_t C, int mode, float s_override,
                             float amax, uint64_t seed_sr, uint8_t *codes, uint8_t *scales,
                             float *tensor_scale)
{
    int64_t G = C / 16;
    if (!(amax > 0.0f)) { /* all-zero tensor: nothing to scale */
        *tensor_scale = 1.0f;
        memset(codes, 0, (size_t)(R * C / 2));
        memset(scales, 0, (size_t)(R * G));
        return;
    }
    float s, cap;
    mode_constants(mode, s_override, &s, &cap);
    if (mode == QO_MS_EDEN_PH) {
        quantize_rotated_posthoc(y, R, C, s, cap, amax, seed_sr, codes, scales, tensor_scale);
        return;
    }
    /* x^FP32 = max|x| / (s * cap)                                          */
    const float x32 = amax / (s * cap);
    *tensor_scale = x32;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r)
        for (int64_t g = 0; g < G; ++g) {
            const float *yg = y + r * C + g * 16;
            uint8_t *cg = codes + (r * C + g * 16) / 2;
            /* x^FP8_g = RTN_FP8( max_g |x| / (x^FP32 * s) )                 */
            float gmax = 0.0f;
            for (int k = 0; k < 16; ++k) {
                float a = fabsf(yg[k]);
                if (a > gmax) gmax = a;
            }
            if (mode == QO_RTN_46) {
                /* Sec. 4.1: keep the candidate with the lower squared error; */
                /* the usual mapping to 6 wins ties                          */
                uint8_t c6[8], c4[8];
                float e6, e4;
                uint8_t b6 = rtn_candidate(yg, gmax, x32, 6.0f, c6, &e6);
                uint8_t b4 = rtn_candidate(yg, gmax, x32, 4.0f, c4, &e4);
                int use4 = e4 < e6;
                memcpy(cg, use4 ? c4 : c6, 8);
                scales[r * G + g] = use4 ? b4 : b6;
                continue;
            }
            uint8_t b = qo_e4m3_rtn(gmax / (x32 * s));
            if (b == 0) { /* scale under-flowed to 0: the group is all zeros */
                memset(cg, 0, 8);
                scales[r * G + g] = 0;
                continue;
            }
            const float x8 = qo_e4m3_decode(b);
            /* x^FP4_i = round( x_i / (x^FP8_g * x^FP32) ), the divisor      */
            /* inverted once per group                                       */
            const float inv = 1.0f / (x8 * x32);
            float cval[16];
            for (int k = 0; k < 16; ++k) {
                float q = yg[k] * inv;
                uint8_t code = (mode == QO_SR)
                                   ? qo_e2m1_sr(q, qo_elem_draw(seed_sr, r, g * 16 + k))
                                   : qo_e2m1_rtn(q);
                cval[k] = qo_e2m1_decode(code);
                if (k & 1) cg[k >> 1] |= (uint8_t)(code << 4);
                else cg[k >> 1] = code;
            }
            if (mode == QO_MS_EDEN) {
                /* S_g = <x_g, x_g> / <x_g, x^RTN_g> with                    */
                /* x^RTN = x^FP4 * x^FP8 * x^FP32, so the new scale          */
                /* S_g * x^FP8_g = <x_g,x_g> / (<x_g,x^FP4_g> * x^FP32):     */
                /* x^FP8_g cancels.  Dot products: fused multiply-add chain  */
                /* in index order starting from 0.                           */
                float num = 0.0f, den = 0.0f;
                for (int k = 0; k < 16; ++k) {
                    num = fmaf(yg[k], yg[k], num);
                    den = fmaf(yg[k], cval[k], den);
                }
                if (den > 0.0f) {
                    float t = num / (den * x32);
                    b = qo_e4m3_sr(t, qo_scale_draw(seed_sr, r, g));
                }
            }
            scales[r * G + g] = b;
        }
}

/* Q(x) or Q(x^T): mode RTN | SR | MS_EDEN | RTN_46 | MS_EDEN_PH.  Output is */
/* in rotated space:                                                        */
/* codes R*C/2 bytes (element 2j in the low nibble), scales R*C/16 bytes    */
/* row-major, one f32 tensor scale.  amax_in (nullable) replaces the        */
/* measured max of the rotated tensor.                                      */
int qo_quantize(const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld, int transpose,
                int mode, int rht_group, uint64_t seed_rht, uint64_t seed_sr,
                const float *amax_in, float s_override, uint8_t *codes, uint8_t *scales,
                float *tensor_scale)
{
    if (mode != QO_RTN && mode != QO_SR && mode != QO_MS_EDEN && mode != QO_RTN_46 && mode != QO_MS_EDEN_PH) return QO_BAD;
    int64_t R = transpose ? cols : rows, C = transpose ? rows : cols;
    float *y = (float *)malloc(sizeof(float) * (size_t)(R * C > 0 ? R * C : 1));
    if (!y) return QO_BAD;
    int rc = build_rotated(x, dtype, rows, cols, ld, transpose, rht_group, seed_rht, y);
    if (rc == QO_OK) {
        float amax = amax_in ? *amax_in : tensor_absmax(y, R * C);
        quantize_rotated(y, R, C, mode, s_override, amax, seed_sr, codes, scales, tensor_scale);
    }
    free(y);
    return rc;
}

/* x_hat = (x^FP4 * x^FP8) * x^FP32: the first product is exact, the second */
/* is one binary32 rounding.                                                */
int qo_dequantize(const uint8_t *codes, const uint8_t *scales, const float *tensor_scale,
                  int64_t rows, int64_t cols, float *y)
{
    if (cols % 16 != 0) return QO_BAD;
    const float x32 = *tensor_scale;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            uint8_t byte = codes[(r * cols + c) / 2];
            uint8_t code = (c & 1) ? (byte >> 4) : (byte & 15);
            float x8 = qo_e4m3_decode(scales[r * (cols / 16) + c / 16]);
            y[r * cols + c] = (qo_e2m1_decode(code) * x8) * x32;
        }
    return QO_OK;
}

/* Backward-pass re-quantization (Sec. 5): dequantize a saved NVFP4 tensor, */
/* optionally transpose, then quantize as above.                            */
int qo_requantize(const uint8_t *in_codes, const uint8_t *in_scales, const float *in_tensor_scale,
                  int64_t rows, int64_t cols, int transpose, int mode, int rht_group,
                  uint64_t seed_rht, uint64_t seed_sr, const float *amax_in, uint8_t *codes,
                  uint8_t *scales, float *tensor_scale)
{
    float *xd = (float *)malloc(sizeof(float) * (size_t)(rows * cols > 0 ? rows * cols : 1));
    if (!xd) return QO_BAD;
    int rc = qo_dequantize(in_codes, in_scales, in_tensor_scale, rows, cols, xd);
    if (rc == QO_OK)
        rc = qo_quantize(xd, QO_F32, rows, cols, cols, transpose, mode, rht_group, seed_rht,
                         seed_sr, amax_in, 0.0f, codes, scales, tensor_scale);
    free(xd);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Block-scaled GEMM, by definition:                                        */
/*   C[m][n] = sum_k A_hat[m][k] * B_hat[n][k],                             */
/*   A_hat = x^FP4 * x^FP8 * x^FP32 formed in double (exact).               */
/* Both operands are K-contiguous.  abs_sum (nullable) = sum_k |A_hat*B_hat|*/
/* is the scale of the rounding-error bound used by the parity tests.       */
/* ------------------------------------------------------------------------ */
static double dq_double(const uint8_t *codes, const uint8_t *scales, double ts, int64_t K,
                        int64_t row, int64_t k)
{
    uint8_t byte = codes[(row * K + k) / 2];
    uint8_t code = (k & 1) ? (byte >> 4) : (byte & 15);
    return (double)qo_e2m1_decode(code) * (double)qo_e4m3_decode(scales[row * (K / 16) + k / 16]) * ts;
}

int qo_gemm(const uint8_t *a_codes, const uint8_t *a_scales, const float *a_ts, int64_t M,
            const uint8_t *b_codes, const uint8_t *b_scales, const float *b_ts, int64_t N,
            int64_t K, double *C, double *abs_sum)
{
    if (K % 16 != 0) return QO_BAD;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0, aacc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double p = dq_double(a_codes, a_scales, (double)*a_ts, K, m, k) *
                           dq_double(b_codes, b_scales, (double)*b_ts, K, n, k);
                acc += p;
                aacc += fabs(p);
            }
            C[m * N + n] = acc;
            if (abs_sum) abs_sum[m * N + n] = aacc;
        }
    return QO_OK;
}

/* The same definition evaluated only at the listed (m, n) pairs.           */
int qo_gemm_sampled(const uint8_t *a_codes, const uint8_t *a_scales, const float *a_ts,
                    const uint8_t *b_codes, const uint8_t *b_scales, const float *b_ts, int64_t K,
                    const int64_t *ms, const int64_t *ns, int64_t count, double *out,
                    double *abs_sum)
{
    if (K % 16 != 0) return QO_BAD;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        double acc = 0.0, aacc = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double p = dq_double(a_codes, a_scales, (double)*a_ts, K, ms[i], k) *
                       dq_double(b_codes, b_scales, (double)*b_ts, K, ns[i], k);
            acc += p;
            aacc += fabs(p);
        }
        out[i] = acc;
        if (abs_sum) abs_sum[i] = aacc;
    }
    return QO_OK;
}

int qo_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
