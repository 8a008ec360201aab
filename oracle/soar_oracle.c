/*
 * soar_oracle.c -- plain, slow CPU statement of the SOAR hot path (one CJSO step
 * followed by one DSS search) for NVFP4 weight quantization.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the reference against which the HIP
 * library is compared; it is never part of the product path.  Only the tests,
 * the smoke check and the benchmark's CPU-baseline leg may load it.  It shares
 * no code, header, table or constant generator with the HIP sources.
 *
 * Every function cites the passage of the paper (arXiv 2605.12245, "SOAR:
 * Scale Optimization for Accurate Reconstruction in NVFP4 Quantization") that
 * it follows.  Where the paper leaves the arithmetic open (rounding ties,
 * order of sums, precision of intermediate results) the choice made here is
 * stated next to the code; those choices are part of the contract the HIP path
 * must reproduce bit for bit.
 *
 * Arithmetic conventions
 *   - every float operation below is one IEEE-754 binary32 operation, rounded
 *     to nearest even; build with -ffp-contract=off so that the compiler never
 *     fuses a multiply and an add by itself;
 *   - fmaf(a,b,c) is the single-rounding fused multiply-add of C99;
 *   - binary32 subnormals are kept (no flush to zero);
 *   - sums over the 16 elements of a block run in ascending element order in
 *     one binary32 accumulator that starts at 0;
 *   - sums over blocks (the two tensor-wide statistics of Eq. 5) are taken in
 *     binary64 over an adjacent-pair binary tree on the flat block index
 *     (row-major: i = row * (cols/16) + block-in-row); an odd element at the
 *     end of a level is carried up unchanged, which equals padding with zeros
 *     to a power of two.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py against
 * something other than itself (brute force over the value grids, a library
 * float8 cast, least-squares routines, closed-form tensors, exhaustive search
 * over all E4M3 scales, exact equivariances).  No function is "parity
 * unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define BLOCK 16                /* Sec. 3.1: one block scale every 16 elements */
#define M_FP4 6.0f              /* Sec. 3.1: largest E2M1 magnitude           */
#define M_FP8 448.0f            /* Sec. 3.1: largest E4M3 magnitude           */
#define E4M3_CODE_MIN 0x01      /* smallest positive E4M3 value, 2^-9         */
#define E4M3_CODE_MAX 0x7E      /* 448; 0x7F is NaN in the OCP "fn" variant   */

enum { ORACLE_BF16 = 0, ORACLE_FP32 = 1 };
enum { ORACLE_METHOD_RTN = 0, ORACLE_METHOD_SOAR = 1 };
enum { ORACLE_STATUS_NONFINITE = 1, ORACLE_STATUS_ALLZERO = 2, ORACLE_STATUS_BAD_AMAX = 4 };

/* ------------------------------------------------------------------------- */
/* Number formats (Sec. 3.1)                                                  */
/* ------------------------------------------------------------------------- */

/* bf16 is the upper half of a binary32: widening is exact. */
float soar_oracle_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* binary32 -> bf16, round to nearest even (used only by dequantize output). */
uint16_t soar_oracle_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)          /* NaN stays NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/*
 * Q_FP4: Eq. 2 of Sec. 3.1, the three-piece rounding onto the E2M1 grid
 * {0, 0.5, 1, 1.5, 2, 3, 4, 6}.  The bracket "round to nearest" is taken as
 * round-half-to-even (rintf in the default rounding mode), which is the same
 * as IEEE round-to-nearest-even on the E2M1 code.  Magnitudes above 6, which
 * Eq. 2 does not list, saturate to 6.  The sign of x is kept, also on a zero
 * result.
 */
float soar_oracle_e2m1_round(float x)
{
    float a = fabsf(x);
    float r;
    if (a < 2.0f)
        r = 0.5f * rintf(2.0f * a);
    else if (a < 4.0f)
        r = rintf(a);
    else if (a <= M_FP4)
        r = 2.0f * rintf(a / 2.0f);
    else
        r = M_FP4;
    return copysignf(r, x);
}

/* Stored form of an E2M1 value: bit 3 = sign, bits 0..2 = index into the
 * magnitude grid (which is also the E2M1 bit pattern: 2 exponent bits, 1
 * mantissa bit, bias 1). */
static const float E2M1_GRID[8] = { 0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f };

uint8_t soar_oracle_e2m1_nibble_of_value(float q)
{
    float a = fabsf(q);
    uint8_t m = 0;
    for (int k = 0; k < 8; ++k)
        if (E2M1_GRID[k] == a) m = (uint8_t)k;
    return (uint8_t)((signbit(q) ? 8 : 0) | m);
}

float soar_oracle_e2m1_value(uint8_t nibble)
{
    float a = E2M1_GRID[nibble & 7];
    return (nibble & 8) ? -a : a;
}

uint8_t soar_oracle_e2m1_nibble(float x)
{
    return soar_oracle_e2m1_nibble_of_value(soar_oracle_e2m1_round(x));
}

/* Value of a positive E4M3 code (OCP "fn" variant: bias 7, 3 mantissa bits,
 * subnormals m * 2^-9, largest finite 448 = 0x7E; Sec. 3.1 fixes M_FP8=448). */
float soar_oracle_e4m3_value(uint8_t code)
{
    int e = (code >> 3) & 0xF;
    int m = code & 7;
    if (e == 0)
        return ldexpf((float)m, -9);
    return ldexpf(1.0f + (float)m / 8.0f, e - 7);
}

/*
 * Projection of a real scale onto E4M3 (Appendix D, last equation:
 * clip(round_E4M3(.), min_E4M3, max_E4M3)).  Rounding is to the nearest
 * representable value, ties to the even mantissa; the result is then clipped
 * to [2^-9, 448], min_E4M3 being read as the smallest POSITIVE value because a
 * zero block scale would make W/(alpha*Delta) undefined.  Returns the code.
 * +inf maps to 448; NaN and non-positive inputs map to 2^-9.
 */
uint8_t soar_oracle_e4m3_project(float y)
{
    if (!(y > 0.0f))
        return E4M3_CODE_MIN;
    if (isinf(y))
        return E4M3_CODE_MAX;
    double v = (double)y;
    int ex;
    (void)frexp(v, &ex);             /* v = m * 2^ex with m in [0.5, 1)        */
    int E = ex - 1;                  /* floor(log2 v)                          */
    if (E < -6) E = -6;              /* below 2^-6 the spacing stays 2^-9      */
    double quantum = ldexp(1.0, E - 3);
    double r = rint(v / quantum) * quantum;   /* both scalings are exact       */
    if (r > (double)M_FP8) r = (double)M_FP8;
    if (r < ldexp(1.0, -9)) r = ldexp(1.0, -9);
    /* encode r, which is now exactly representable */
    (void)frexp(r, &ex);
    E = ex - 1;
    if (E < -6)
        return (uint8_t)lrint(ldexp(r, 9));
    int m = (int)lrint((ldexp(r, -E) - 1.0) * 8.0);
    return (uint8_t)(((E + 7) << 3) | m);
}

/* Array forms of the two projections, for exhaustive comparisons. */
void soar_oracle_e2m1_nibble_many(const float *x, int64_t n, uint8_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = soar_oracle_e2m1_nibble(x[i]);
}

void soar_oracle_e4m3_project_many(const float *y, int64_t n, uint8_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = soar_oracle_e4m3_project(y[i]);
}

/* ------------------------------------------------------------------------- */
/* Per-block steps                                                            */
/* ------------------------------------------------------------------------- */

static inline float load_w(const void *w, int dtype, int64_t idx)
{
    if (dtype == ORACLE_BF16)
        return soar_oracle_bf16_to_f32(((const uint16_t *)w)[idx]);
    return ((const float *)w)[idx];
}

/* Q_i = Q_FP4(W_i / (alpha * Delta)) (Eq. 2, and the first line of the loop
 * body of Algorithm 1).  The quotient is evaluated as a product with the
 * reciprocal of the combined scale, the reciprocal being one IEEE division
 * per block:  r = 1 / (alpha * Delta),  x_j = w_j * r. */
static void assign_codes(const float wv[BLOCK], float alpha, float delta, float q[BLOCK])
{
    float scale = alpha * delta;
    float r = 1.0f / scale;
    for (int j = 0; j < BLOCK; ++j)
        q[j] = soar_oracle_e2m1_round(wv[j] * r);
}

/* Block reconstruction error of Eq. 8 (= one block of Eq. 4) for signed codes
 * q and combined dequantization scale s = alpha * Delta^d:
 *     e_j = w_j - q_j * s   (one fused operation),   err = sum_j e_j^2
 * accumulated in ascending j with fused multiply-adds, starting from 0. */
static float block_error(const float wv[BLOCK], const float q[BLOCK], float s)
{
    float err = 0.0f;
    for (int j = 0; j < BLOCK; ++j) {
        float e = fmaf(-q[j], s, wv[j]);
        err = fmaf(e, e, err);
    }
    return err;
}

/* The two block sums that both closed forms (Eq. 5 and Eq. 6) are built from:
 *     a = sum_j w_j q_j,    b = sum_j q_j^2
 * (ascending j, fused multiply-add accumulation from 0). */
static void block_sums(const float wv[BLOCK], const float q[BLOCK], float *a, float *b)
{
    float sa = 0.0f, sb = 0.0f;
    for (int j = 0; j < BLOCK; ++j) {
        sa = fmaf(wv[j], q[j], sa);
        sb = fmaf(q[j], q[j], sb);
    }
    *a = sa;
    *b = sb;
}

static void pack_block(const float wv[BLOCK], const float q[BLOCK], uint8_t out[BLOCK / 2])
{
    /* element 2k in the low nibble, element 2k+1 in the high nibble; the sign
     * bit is the sign of the weight, also when the magnitude rounds to 0. */
    for (int k = 0; k < BLOCK / 2; ++k) {
        uint8_t lo = soar_oracle_e2m1_nibble_of_value(copysignf(fabsf(q[2 * k]), wv[2 * k]));
        uint8_t hi = soar_oracle_e2m1_nibble_of_value(copysignf(fabsf(q[2 * k + 1]), wv[2 * k + 1]));
        out[k] = (uint8_t)(lo | (hi << 4));
    }
}

/* Adjacent-pair binary tree sum in binary64, in place; t is destroyed. */
static double tree_sum(double *t, int64_t n)
{
    if (n <= 0) return 0.0;
    while (n > 1) {
        int64_t half = n / 2;
        for (int64_t k = 0; k < half; ++k)
            t[k] = t[2 * k] + t[2 * k + 1];
        if (n & 1) {
            t[half] = t[n - 1];
            n = half + 1;
        } else {
            n = half;
        }
    }
    return t[0];
}

/* ------------------------------------------------------------------------- */
/* Optional trace of intermediate results, for the pin tests                  */
/* ------------------------------------------------------------------------- */
typedef struct {
    float   alpha0;        /* Eq. 1 global scale                                */
    float   alpha1;        /* Eq. 5 global scale after the closed-form step     */
    double  N, M;          /* numerator / denominator of Eq. 5                  */
    uint8_t *code0;        /* [blocks]  E4M3 code of the Eq. 1 block scale      */
    uint8_t *nib0;         /* [elems/2] packed codes of the Eq. 1 assignment    */
    float   *a;            /* [blocks]  sum_j w q  under the Eq. 1 assignment   */
    float   *b;            /* [blocks]  sum_j q^2  under the Eq. 1 assignment   */
    float   *delta_star;   /* [blocks]  Eq. 6 block scale, unrounded (= Delta^q)*/
    uint8_t *centre;       /* [blocks]  E4M3 code of the projected Eq. 6 scale  */
    float   *err_best;     /* [blocks]  Eq. 8 value of the chosen candidate     */
} soar_oracle_trace;

/* ------------------------------------------------------------------------- */
/* Whole path                                                                 */
/* ------------------------------------------------------------------------- */

/*
 * soar_oracle_quantize
 *
 * method = RTN : max-based NVFP4 of Sec. 3.1 (Eq. 1-2).
 * method = SOAR: Algorithm 1 with T = 1:
 *     initialisation by Eq. 1 with Delta^q = Delta^d,
 *     FP4 assignment Q0 (Eq. 2),
 *     global scale by Eq. 5,
 *     block scale by Eq. 6 (kept unrounded as the quantization scale Delta^q),
 *     projection of that scale onto E4M3 (Appendix D),
 *     new assignment Q1 under (alpha1, Delta^q),
 *     search of the stored scale Delta^d over the E4M3 codes centre-K..centre+K
 *     by the block error of Eq. 8,
 *     emission of Q1, the chosen code and alpha1.
 * The quantization-scale side of the search uses the single value beta = 1.
 *
 * w: rows x cols, row-major with leading dimension ld (elements); blocks are
 * 16 consecutive elements of a row.  codes: rows*cols/2 bytes; scales:
 * rows*cols/16 bytes, row-major.  Returns 0, or -1 on a bad argument.
 */
int soar_oracle_quantize(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld,
                         int method, int dss_radius,
                         uint8_t *codes, uint8_t *scales, float *global_scale,
                         double *sse, int32_t *status, soar_oracle_trace *trace)
{
    if (!w || !codes || !scales || !global_scale) return -1;
    if (rows <= 0 || cols <= 0 || cols % BLOCK != 0 || ld < cols) return -1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_FP32) return -1;
    if (method != ORACLE_METHOD_RTN && method != ORACLE_METHOD_SOAR) return -1;
    if (dss_radius < 0 || dss_radius > 125) return -1;

    const int64_t bpr = cols / BLOCK;          /* blocks per row */
    const int64_t nblk = rows * bpr;
    int32_t st = 0;

    /* ---- Eq. 1, first half: alpha0 = max|W| / (M_FP4 * M_FP8) ---- */
    float amax = 0.0f;
    int nonfinite = 0;
#pragma omp parallel for schedule(static) reduction(max : amax) reduction(| : nonfinite)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            float v = load_w(w, dtype, r * ld + c);
            if (!isfinite(v)) nonfinite = 1;
            else if (fabsf(v) > amax) amax = fabsf(v);
        }
    if (nonfinite) {
        st |= ORACLE_STATUS_NONFINITE;      /* outputs are unspecified */
        if (status) *status = st;
        if (sse) *sse = NAN;
        *global_scale = NAN;
        return 0;
    }
    if (amax == 0.0f) {
        /* all-zero tensor: unit global scale, smallest block scale, zero codes
         * that keep the sign of the weight, zero error */
        st |= ORACLE_STATUS_ALLZERO;
        for (int64_t i = 0; i < nblk; ++i) {
            int64_t r = i / bpr, cb = i % bpr;
            scales[i] = E4M3_CODE_MIN;
            for (int k = 0; k < BLOCK / 2; ++k) {
                float w0 = load_w(w, dtype, r * ld + cb * BLOCK + 2 * k);
                float w1 = load_w(w, dtype, r * ld + cb * BLOCK + 2 * k + 1);
                codes[i * (BLOCK / 2) + k] = (uint8_t)((signbit(w0) ? 0x08 : 0) | (signbit(w1) ? 0x80 : 0));
            }
        }
        *global_scale = 1.0f;
        if (sse) *sse = 0.0;
        if (status) *status = st;
        return 0;
    }
    const float alpha0 = amax / (M_FP4 * M_FP8);
    const float alpha0_m = alpha0 * M_FP4;

    double *termN = (double *)malloc(sizeof(double) * (size_t)nblk);
    double *termM = (double *)malloc(sizeof(double) * (size_t)nblk);
    float *a_all = (float *)malloc(sizeof(float) * (size_t)nblk);
    float *b_all = (float *)malloc(sizeof(float) * (size_t)nblk);
    uint8_t *c0_all = (uint8_t *)malloc((size_t)nblk);
    double *errs = (double *)malloc(sizeof(double) * (size_t)nblk);
    if (!termN || !termM || !a_all || !b_all || !c0_all || !errs) {
        free(termN); free(termM); free(a_all); free(b_all); free(c0_all); free(errs);
        return -1;
    }

    /* ---- Eq. 1, second half, and the Eq. 2 assignment under it ---- */
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nblk; ++i) {
        int64_t r = i / bpr, cb = i % bpr;
        float wv[BLOCK], q0[BLOCK];
        float bmax = 0.0f;
        for (int j = 0; j < BLOCK; ++j) {
            wv[j] = load_w(w, dtype, r * ld + cb * BLOCK + j);
            if (fabsf(wv[j]) > bmax) bmax = fabsf(wv[j]);
        }
        /* Delta0_i = Q_E4M3( max|W_i| / (alpha0 * M_FP4) ) */
        uint8_t c0 = soar_oracle_e4m3_project(bmax / alpha0_m);
        float delta0 = soar_oracle_e4m3_value(c0);
        assign_codes(wv, alpha0, delta0, q0);
        float a, b;
        block_sums(wv, q0, &a, &b);
        a_all[i] = a;
        b_all[i] = b;
        c0_all[i] = c0;
        /* terms of Eq. 5; each product is exact in binary64 */
        termN[i] = (double)a * (double)delta0;
        termM[i] = ((double)b * (double)delta0) * (double)delta0;
        if (trace) {
            if (trace->code0) trace->code0[i] = c0;
            if (trace->a) trace->a[i] = a;
            if (trace->b) trace->b[i] = b;
            if (trace->nib0) pack_block(wv, q0, trace->nib0 + i * (BLOCK / 2));
        }
        if (method == ORACLE_METHOD_RTN) {
            scales[i] = c0;
            pack_block(wv, q0, codes + i * (BLOCK / 2));
            errs[i] = (double)block_error(wv, q0, alpha0 * delta0);
        }
    }

    if (method == ORACLE_METHOD_RTN) {
        *global_scale = alpha0;
        if (trace) { trace->alpha0 = alpha0; trace->alpha1 = alpha0; trace->N = 0; trace->M = 0; }
        if (sse) *sse = tree_sum(errs, nblk);
        if (status) *status = st;
        free(termN); free(termM); free(a_all); free(b_all); free(c0_all); free(errs);
        return 0;
    }

    /* ---- Eq. 5: alpha1 = sum_i a_i Delta0_i / sum_i b_i Delta0_i^2 ---- */
    const double N = tree_sum(termN, nblk);
    const double M = tree_sum(termM, nblk);
    /* M == 0 (no non-zero code in the whole tensor) leaves 0/0: keep alpha0 */
    const float alpha1 = (M > 0.0) ? (float)(N / M) : alpha0;
    if (trace) { trace->alpha0 = alpha0; trace->alpha1 = alpha1; trace->N = N; trace->M = M; }

    /* ---- Eq. 6, projection, re-assignment, Eq. 8 search ---- */
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nblk; ++i) {
        int64_t r = i / bpr, cb = i % bpr;
        float wv[BLOCK], q1[BLOCK];
        for (int j = 0; j < BLOCK; ++j)
            wv[j] = load_w(w, dtype, r * ld + cb * BLOCK + j);
        /* Delta*_i = (sum w q alpha) / (sum q^2 alpha^2) = (a_i / b_i) / alpha1:
         * two binary32 divisions; a block whose codes are all zero leaves 0/0
         * and keeps its Eq. 1 scale */
        float delta_star;
        if (b_all[i] == 0.0f)
            delta_star = soar_oracle_e4m3_value(c0_all[i]);
        else
            delta_star = (a_all[i] / b_all[i]) / alpha1;
        const uint8_t centre = soar_oracle_e4m3_project(delta_star);
        /* quantization scale Delta^q = Delta* (not rounded): new assignment */
        assign_codes(wv, alpha1, delta_star, q1);
        /* candidates for the stored scale: offsets 0,-1,+1,-2,+2,...,-K,+K in
         * code space; the first strictly smaller error wins */
        int best_code = centre;
        float best_err = block_error(wv, q1, alpha1 * soar_oracle_e4m3_value(centre));
        for (int k = 1; k <= dss_radius; ++k) {
            for (int sgn = -1; sgn <= 1; sgn += 2) {
                int c = (int)centre + sgn * k;
                if (c < E4M3_CODE_MIN || c > E4M3_CODE_MAX) continue;
                float err = block_error(wv, q1, alpha1 * soar_oracle_e4m3_value((uint8_t)c));
                if (err < best_err) { best_err = err; best_code = c; }
            }
        }
        scales[i] = (uint8_t)best_code;
        pack_block(wv, q1, codes + i * (BLOCK / 2));
        errs[i] = (double)best_err;
        if (trace) {
            if (trace->delta_star) trace->delta_star[i] = delta_star;
            if (trace->centre) trace->centre[i] = centre;
            if (trace->err_best) trace->err_best[i] = best_err;
        }
    }
    *global_scale = alpha1;
    if (sse) *sse = tree_sum(errs, nblk);
    if (status) *status = st;
    free(termN); free(termM); free(a_all); free(b_all); free(c0_all); free(errs);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1 in full: T iterations, beta grid, early stop                     */
/* ------------------------------------------------------------------------- */

typedef struct {
    int32_t iters;           /* T of Algorithm 1 (the paper uses 15)                       */
    int32_t n_beta;          /* size of the quantization-scale grid (paper: 101)           */
    float   beta_lo;         /* paper: 0.5                                                 */
    float   beta_hi;         /* paper: 1.5                                                 */
    int32_t dd_mode;         /* 0: E4M3 codes centre-K..centre+K around the rounded Eq. 6
                                scale; 1: the two representable values that surround it
                                (Appendix B.3)                                             */
    int32_t dss_radius;      /* K of dd_mode 0                                             */
    float   early_stop_rel;  /* stop when the relative drop of the error is below this
                                (paper: 1e-3); <= 0 never stops                            */
    int32_t arm;             /* 0: SOAR (CJSO + DSS);
                                1: "+CJSO" alone (Sec. 3.2, refinement scheme): Eq. 5, Eq. 6,
                                   projection onto E4M3, ONE scale for assignment and storage;
                                   needs n_beta 1, beta 1, dd_mode 0, dss_radius 0;
                                2: "+DSS" alone (Sec. 3.3 (i)-(ii)): the global scale stays
                                   at its Eq. 1 value and the search is centred on the block's
                                   current stored scale instead of Eq. 6                     */
} soar_oracle_iter_params;
enum { ORACLE_ARM_SOAR = 0, ORACLE_ARM_CJSO_ONLY = 1, ORACLE_ARM_DSS_ONLY = 2 };

/* largest E4M3 code in [0x01, 0x7E] whose value does not exceed y (0x01 if none) */
static int e4m3_floor_code(float y)
{
    int best = E4M3_CODE_MIN;
    for (int c = E4M3_CODE_MIN; c <= E4M3_CODE_MAX; ++c)
        if (soar_oracle_e4m3_value((uint8_t)c) <= y) best = c;
    return best;
}

/* beta_k of the grid: lo and hi are hit exactly, and so is 1 on the paper's grid */
static float beta_of(const soar_oracle_iter_params *p, int k)
{
    if (p->n_beta <= 1) return p->beta_lo;
    return (p->beta_lo * (float)(p->n_beta - 1 - k) + p->beta_hi * (float)k) / (float)(p->n_beta - 1);
}

/*
 * soar_oracle_quantize_iter -- Algorithm 1 as printed: initialisation by Eq. 1
 * with Delta^q = Delta^d; then T times
 *     Q      = Q_FP4(W / (alpha Delta^q))                         (Eq. 2)
 *     alpha <- sum W Q Delta^d / sum Q^2 (Delta^d)^2              (Eq. 5)
 *     Delta* = (sum W Q / sum Q^2) / alpha                        (Eq. 6)
 *     D^d    = E4M3 candidates near Delta*,  D^q = {Delta* beta}  (Sec. 3.3 (ii), App. B.3)
 *     (Delta^q, Delta^d) <- argmin over D^q x D^d of Eq. 8
 * with early stopping on the relative drop of the total error, and the final
 * reconstruction Q_FP4(W/(alpha Delta^q)) * (alpha Delta^d).
 *
 * Candidate pairs are tried with beta ascending and, for each beta, the stored
 * scales in the order "centre, -1, +1, -2, ..." (dd_mode 0) or "lower, upper"
 * (dd_mode 1); a later pair wins only if strictly better in binary32.  All
 * per-block and tensor-wide arithmetic is that of soar_oracle_quantize; with
 * iters = 1, n_beta = 1, beta = 1, dd_mode = 0 the two functions agree bit
 * for bit.
 *
 * The ablation arms of the paper's component study (p->arm): "+CJSO" alone runs
 * Eq. 5, Eq. 6 and the E4M3 projection with ONE block scale for assignment and
 * storage (Sec. 3.2, refinement scheme; alpha and Delta are both updated from
 * the same assignment, as in the listing's closed-form stage); "+DSS" alone
 * keeps the Eq. 1 global scale and centres the joint search of Sec. 3.3 (ii)
 * on the block's current stored scale.
 *
 * sse_trace (may be NULL): iters+1 doubles; [0] is the error of the Eq. 1-2
 * state, [t+1] the error after iteration t; entries after an early stop are
 * left untouched.  iters_run (may be NULL): iterations carried out.
 */
int soar_oracle_quantize_iter(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld,
                              const soar_oracle_iter_params *p,
                              uint8_t *codes, uint8_t *scales, float *global_scale,
                              double *sse, int32_t *status, int32_t *iters_run, double *sse_trace)
{
    if (!w || !codes || !scales || !global_scale || !p) return -1;
    if (rows <= 0 || cols <= 0 || cols % BLOCK != 0 || ld < cols) return -1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_FP32) return -1;
    if (p->iters < 1 || p->n_beta < 1 || p->n_beta > 4096) return -1;
    if (!(p->beta_lo > 0.0f) || !(p->beta_hi >= p->beta_lo)) return -1;
    if (p->dd_mode != 0 && p->dd_mode != 1) return -1;
    if (p->dss_radius < 0 || p->dss_radius > 125) return -1;
    if (p->arm < ORACLE_ARM_SOAR || p->arm > ORACLE_ARM_DSS_ONLY) return -1;
    if (p->arm == ORACLE_ARM_CJSO_ONLY &&
        (p->n_beta != 1 || p->beta_lo != 1.0f || p->dd_mode != 0 || p->dss_radius != 0))
        return -1;

    const int64_t bpr = cols / BLOCK;
    const int64_t nblk = rows * bpr;

    float amax = 0.0f;
    int nonfinite = 0;
#pragma omp parallel for schedule(static) reduction(max : amax) reduction(| : nonfinite)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            float v = load_w(w, dtype, r * ld + c);
            if (!isfinite(v)) nonfinite = 1;
            else if (fabsf(v) > amax) amax = fabsf(v);
        }
    if (nonfinite || amax == 0.0f) {
        /* degenerate tensors behave as in the single-step function */
        if (iters_run) *iters_run = 0;
        return soar_oracle_quantize(w, dtype, rows, cols, ld, ORACLE_METHOD_SOAR, 0, codes, scales,
                                    global_scale, sse, status, NULL);
    }

    float *dq = (float *)malloc(sizeof(float) * (size_t)nblk);       /* Delta^q */
    uint8_t *dd = (uint8_t *)malloc((size_t)nblk);                   /* code of Delta^d */
    float *a_all = (float *)malloc(sizeof(float) * (size_t)nblk);
    float *b_all = (float *)malloc(sizeof(float) * (size_t)nblk);
    double *termN = (double *)malloc(sizeof(double) * (size_t)nblk);
    double *termM = (double *)malloc(sizeof(double) * (size_t)nblk);
    double *errs = (double *)malloc(sizeof(double) * (size_t)nblk);
    if (!dq || !dd || !a_all || !b_all || !termN || !termM || !errs) {
        free(dq); free(dd); free(a_all); free(b_all); free(termN); free(termM); free(errs);
        return -1;
    }

    /* ---- initialisation: Eq. 1, Delta^q = Delta^d; error of the Eq. 1-2 state ---- */
    float alpha = amax / (M_FP4 * M_FP8);
    const float alpha0_m = alpha * M_FP4;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nblk; ++i) {
        int64_t r = i / bpr, cb = i % bpr;
        float wv[BLOCK], q0[BLOCK];
        float bmax = 0.0f;
        for (int j = 0; j < BLOCK; ++j) {
            wv[j] = load_w(w, dtype, r * ld + cb * BLOCK + j);
            if (fabsf(wv[j]) > bmax) bmax = fabsf(wv[j]);
        }
        dd[i] = soar_oracle_e4m3_project(bmax / alpha0_m);
        dq[i] = soar_oracle_e4m3_value(dd[i]);
        assign_codes(wv, alpha, dq[i], q0);
        errs[i] = (double)block_error(wv, q0, alpha * dq[i]);
    }
    double prev = tree_sum(errs, nblk);
    if (sse_trace) sse_trace[0] = prev;

    int done = 0;
    double cur = prev;
    for (int t = 0; t < p->iters; ++t) {
        /* ---- Q under the current scales, block sums, Eq. 5 ---- */
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < nblk; ++i) {
            int64_t r = i / bpr, cb = i % bpr;
            float wv[BLOCK], q[BLOCK];
            for (int j = 0; j < BLOCK; ++j) wv[j] = load_w(w, dtype, r * ld + cb * BLOCK + j);
            assign_codes(wv, alpha, dq[i], q);
            block_sums(wv, q, &a_all[i], &b_all[i]);
            float d = soar_oracle_e4m3_value(dd[i]);
            termN[i] = (double)a_all[i] * (double)d;
            termM[i] = ((double)b_all[i] * (double)d) * (double)d;
        }
        const double N = tree_sum(termN, nblk);
        const double M = tree_sum(termM, nblk);
        float alpha_new = (M > 0.0) ? (float)(N / M) : alpha;
        if (p->arm == ORACLE_ARM_DSS_ONLY) alpha_new = alpha;       /* no closed-form step */

        /* ---- Eq. 6 and the joint search of Sec. 3.3 ---- */
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < nblk; ++i) {
            int64_t r = i / bpr, cb = i % bpr;
            float wv[BLOCK], q[BLOCK], qbest[BLOCK];
            for (int j = 0; j < BLOCK; ++j) wv[j] = load_w(w, dtype, r * ld + cb * BLOCK + j);
            float delta_star;
            if (b_all[i] == 0.0f || p->arm == ORACLE_ARM_DSS_ONLY)
                delta_star = soar_oracle_e4m3_value(dd[i]);         /* centre: the current stored scale */
            else
                delta_star = (a_all[i] / b_all[i]) / alpha_new;
            /* stored-scale candidates */
            int cand[256], ncand = 0;
            if (p->dd_mode == 0) {
                int centre = soar_oracle_e4m3_project(delta_star);
                cand[ncand++] = centre;
                for (int k = 1; k <= p->dss_radius; ++k)
                    for (int sgn = -1; sgn <= 1; sgn += 2) {
                        int c = centre + sgn * k;
                        if (c >= E4M3_CODE_MIN && c <= E4M3_CODE_MAX) cand[ncand++] = c;
                    }
            } else {
                int lo = e4m3_floor_code(delta_star);
                cand[ncand++] = lo;
                if (lo < E4M3_CODE_MAX) cand[ncand++] = lo + 1;
            }
            int have = 0, best_code = cand[0];
            float best_err = 0.0f, best_dq = delta_star;
            for (int k = 0; k < p->n_beta; ++k) {
                float dq_k = delta_star * beta_of(p, k);
                if (p->arm == ORACLE_ARM_CJSO_ONLY)                 /* one scale: assign with the projected one */
                    dq_k = soar_oracle_e4m3_value((uint8_t)cand[0]);
                assign_codes(wv, alpha_new, dq_k, q);
                for (int c = 0; c < ncand; ++c) {
                    float err = block_error(wv, q, alpha_new * soar_oracle_e4m3_value((uint8_t)cand[c]));
                    if (!have || err < best_err) {
                        have = 1;
                        best_err = err;
                        best_code = cand[c];
                        best_dq = dq_k;
                        memcpy(qbest, q, sizeof qbest);
                    }
                }
            }
            dq[i] = best_dq;
            dd[i] = (uint8_t)best_code;
            errs[i] = (double)best_err;
            pack_block(wv, qbest, codes + i * (BLOCK / 2));
        }
        alpha = alpha_new;
        cur = tree_sum(errs, nblk);
        if (sse_trace) sse_trace[t + 1] = cur;
        done = t + 1;
        /* early stop: relative drop of the error below the threshold */
        if (p->early_stop_rel > 0.0f && (prev - cur) < (double)p->early_stop_rel * prev) break;
        prev = cur;
    }
    memcpy(scales, dd, (size_t)nblk);
    *global_scale = alpha;
    if (sse) *sse = cur;
    if (status) *status = 0;
    if (iters_run) *iters_run = done;
    free(dq); free(dd); free(a_all); free(b_all); free(termN); free(termM); free(errs);
    return 0;
}

/*
 * soar_oracle_quantize_rtn_amax -- the max-based NVFP4 of Sec. 3.1 (Eq. 1-2) with
 * the tensor's maximum magnitude SUPPLIED instead of measured: the form in which
 * the standard format is applied to activations (Appendix B.2), where the
 * maximum comes from calibration or from an earlier pass.
 *     alpha   = amax / (M_FP4 * M_FP8)
 *     Delta_i = Q_E4M3( max|W_i| / (alpha * M_FP4) )      (clipped to 448)
 *     codes   = Q_FP4( W_i / (alpha Delta_i) )              (saturating at +-6)
 * so values above amax saturate.  amax must be finite and > 0; otherwise
 * *status = ORACLE_STATUS_BAD_AMAX and nothing else is written.  The weights
 * are not scanned for non-finite values in this mode (status stays 0).
 */
int soar_oracle_quantize_rtn_amax(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld,
                                  float amax, uint8_t *codes, uint8_t *scales, float *global_scale,
                                  double *sse, int32_t *status)
{
    if (!w || !codes || !scales || !global_scale) return -1;
    if (rows <= 0 || cols <= 0 || cols % BLOCK != 0 || ld < cols) return -1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_FP32) return -1;
    if (!isfinite(amax) || !(amax > 0.0f)) {
        if (status) *status = ORACLE_STATUS_BAD_AMAX;
        return 0;
    }
    const int64_t bpr = cols / BLOCK;
    const int64_t nblk = rows * bpr;
    const float alpha = amax / (M_FP4 * M_FP8);
    const float alpha_m = alpha * M_FP4;
    double *errs = (double *)malloc(sizeof(double) * (size_t)nblk);
    if (!errs) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nblk; ++i) {
        int64_t r = i / bpr, cb = i % bpr;
        float wv[BLOCK], q[BLOCK];
        float bmax = 0.0f;
        for (int j = 0; j < BLOCK; ++j) {
            wv[j] = load_w(w, dtype, r * ld + cb * BLOCK + j);
            if (fabsf(wv[j]) > bmax) bmax = fabsf(wv[j]);
        }
        uint8_t c = soar_oracle_e4m3_project(bmax / alpha_m);
        float delta = soar_oracle_e4m3_value(c);
        assign_codes(wv, alpha, delta, q);
        scales[i] = c;
        pack_block(wv, q, codes + i * (BLOCK / 2));
        errs[i] = (double)block_error(wv, q, alpha * delta);
    }
    *global_scale = alpha;
    if (sse) *sse = tree_sum(errs, nblk);
    if (status) *status = 0;
    free(errs);
    return 0;
}

/*
 * Dequantization, Eq. 3:  w^_ij = q_ij * (alpha * d_i), the combined scale
 * being rounded to binary32 first.  out_dtype BF16 rounds the result to
 * nearest even.
 */
int soar_oracle_dequantize(const uint8_t *codes, const uint8_t *scales, float global_scale,
                           int64_t rows, int64_t cols, int out_dtype, void *out, int64_t ld)
{
    if (!codes || !scales || !out) return -1;
    if (rows <= 0 || cols <= 0 || cols % BLOCK != 0 || ld < cols) return -1;
    if (out_dtype != ORACLE_BF16 && out_dtype != ORACLE_FP32) return -1;
    const int64_t bpr = cols / BLOCK;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows * bpr; ++i) {
        int64_t r = i / bpr, cb = i % bpr;
        float s = global_scale * soar_oracle_e4m3_value(scales[i]);
        for (int j = 0; j < BLOCK; ++j) {
            uint8_t byte = codes[i * (BLOCK / 2) + j / 2];
            uint8_t nib = (j & 1) ? (byte >> 4) : (byte & 0xF);
            float v = soar_oracle_e2m1_value(nib) * s;
            int64_t idx = r * ld + cb * BLOCK + j;
            if (out_dtype == ORACLE_BF16)
                ((uint16_t *)out)[idx] = soar_oracle_f32_to_bf16(v);
            else
                ((float *)out)[idx] = v;
        }
    }
    return 0;
}

/*
 * Reconstruction error, Eq. 4, of stored codes / block scales / global scale
 * against the original weights: the block error of Eq. 8 with the stored
 * scale, summed over blocks in binary64.
 */
int soar_oracle_recon_error(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld,
                            const uint8_t *codes, const uint8_t *scales, float global_scale,
                            double *sse)
{
    if (!w || !codes || !scales || !sse) return -1;
    if (rows <= 0 || cols <= 0 || cols % BLOCK != 0 || ld < cols) return -1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_FP32) return -1;
    const int64_t bpr = cols / BLOCK;
    const int64_t nblk = rows * bpr;
    double *errs = (double *)malloc(sizeof(double) * (size_t)nblk);
    if (!errs) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nblk; ++i) {
        int64_t r = i / bpr, cb = i % bpr;
        float wv[BLOCK], q[BLOCK];
        for (int j = 0; j < BLOCK; ++j) {
            wv[j] = load_w(w, dtype, r * ld + cb * BLOCK + j);
            uint8_t byte = codes[i * (BLOCK / 2) + j / 2];
            q[j] = soar_oracle_e2m1_value((j & 1) ? (byte >> 4) : (byte & 0xF));
        }
        errs[i] = (double)block_error(wv, q, global_scale * soar_oracle_e4m3_value(scales[i]));
    }
    *sse = tree_sum(errs, nblk);
    free(errs);
    return 0;
}

/* Thread control for the timed CPU baseline. */
int soar_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void soar_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------------- */
/* Decoupled Scale Search on MXFP4 (Sec. 4.3, "DSS on MXFP4")                  */
/* ------------------------------------------------------------------------- */
/*
 * The paper applies DSS to MXFP4 without restating the format; it is taken
 * from the public OCP Microscaling Formats specification (v1.0): blocks of 32
 * E2M1 elements along a row share one E8M0 scale X = 2^(e-127), e in [0, 254]
 * (255 encodes NaN and is never produced); there is no tensor-wide scale.
 *
 * Baseline conversion (that specification, Sec. 6.3):
 *     shared exponent = floor(log2 max|W_i|) - 2     (2 = exponent of the largest
 *     E2M1 value 6 = 1.5 * 2^2), clamped to [-127, 127];
 *     codes = Q_FP4(W_i / X), round to nearest even, saturating at +-6
 * (a block maximum in (6X, 8X) saturates: that is the format's own behaviour).
 * A block of zeros takes X = 1 (e = 127).
 *
 * DSS (Sec. 3.3 carried over; no closed-form step exists without a global
 * scale, so this is the "+DSS" arm): the stored scale Delta^d is searched over
 * the E8M0 codes e0-K .. e0+K around the baseline code e0 (order 0,-1,+1,...,
 * codes outside [0, 254] skipped), the assignment scale over Delta^q = X0 beta_k,
 * beta_k as in soar_oracle_quantize_iter, beta ascending (outer loop); a later
 * pair wins only if strictly better in binary32.  Error of a pair: Eq. 8 with
 * alpha = 1 over the 32 elements, one ascending chain of fused operations.
 *
 * codes: rows*cols/2 bytes (nibble layout as for NVFP4); scales: rows*cols/32
 * E8M0 bytes.  status: ORACLE_STATUS_NONFINITE if any value is NaN or Inf
 * (outputs then unspecified).  Returns 0, or -1 on a bad argument.
 */
#define MX_BLOCK 32
#define MX_EMAX_ELEM 2

static float e8m0_value(int e) { return ldexpf(1.0f, e - 127); }

static float mx_block_error(const float *wv, const float *q, float s)
{
    float err = 0.0f;
    for (int j = 0; j < MX_BLOCK; ++j) {
        float e = fmaf(-q[j], s, wv[j]);
        err = fmaf(e, e, err);
    }
    return err;
}

static void mx_assign(const float *wv, float scale, float *q)
{
    float r = 1.0f / scale;
    for (int j = 0; j < MX_BLOCK; ++j)
        q[j] = soar_oracle_e2m1_round(wv[j] * r);
}

int soar_oracle_mxfp4_quantize(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld,
                               int dss, int32_t n_beta, float beta_lo, float beta_hi, int32_t radius,
                               uint8_t *codes, uint8_t *scales, double *sse, int32_t *status)
{
    if (!w || !codes || !scales) return -1;
    if (rows <= 0 || cols <= 0 || cols % MX_BLOCK != 0 || ld < cols) return -1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_FP32) return -1;
    if (dss != 0 && dss != 1) return -1;
    if (dss && (n_beta < 1 || n_beta > 4096 || !(beta_lo > 0.0f) || !(beta_hi >= beta_lo) || radius < 0 || radius > 127))
        return -1;
    const int64_t bpr = cols / MX_BLOCK;
    const int64_t nblk = rows * bpr;
    double *errs = (double *)malloc(sizeof(double) * (size_t)nblk);
    if (!errs) return -1;
    soar_oracle_iter_params grid;
    memset(&grid, 0, sizeof grid);
    grid.n_beta = n_beta;
    grid.beta_lo = beta_lo;
    grid.beta_hi = beta_hi;
    int nonfinite = 0;
#pragma omp parallel for schedule(static) reduction(| : nonfinite)
    for (int64_t i = 0; i < nblk; ++i) {
        int64_t r = i / bpr, cb = i % bpr;
        float wv[MX_BLOCK], q[MX_BLOCK], qbest[MX_BLOCK];
        float bmax = 0.0f;
        for (int j = 0; j < MX_BLOCK; ++j) {
            wv[j] = load_w(w, dtype, r * ld + cb * MX_BLOCK + j);
            if (!isfinite(wv[j])) nonfinite = 1;
            else if (fabsf(wv[j]) > bmax) bmax = fabsf(wv[j]);
        }
        int e0 = 127;
        if (bmax > 0.0f) {
            int ex;
            (void)frexpf(bmax, &ex);                 /* bmax = m * 2^ex, m in [0.5, 1): floor(log2) = ex - 1 */
            int shared = (ex - 1) - MX_EMAX_ELEM;
            if (shared < -127) shared = -127;
            if (shared > 127) shared = 127;
            e0 = shared + 127;
        }
        const float x0 = e8m0_value(e0);
        int best_code = e0;
        float best_err;
        if (!dss) {
            mx_assign(wv, x0, qbest);
            best_err = mx_block_error(wv, qbest, x0);
        } else {
            int have = 0;
            best_err = 0.0f;
            for (int k = 0; k < n_beta; ++k) {
                mx_assign(wv, x0 * beta_of(&grid, k), q);
                for (int c = 0; c <= 2 * radius; ++c) {
                    int o = (c + 1) / 2;
                    int code = (c & 1) ? e0 - o : e0 + o;
                    if (code < 0 || code > 254) continue;
                    float err = mx_block_error(wv, q, e8m0_value(code));
                    if (!have || err < best_err) {
                        have = 1;
                        best_err = err;
                        best_code = code;
                        memcpy(qbest, q, sizeof qbest);
                    }
                }
            }
        }
        scales[i] = (uint8_t)best_code;
        errs[i] = (double)best_err;
        for (int k = 0; k < MX_BLOCK / 2; ++k) {
            uint8_t lo = soar_oracle_e2m1_nibble_of_value(copysignf(fabsf(qbest[2 * k]), wv[2 * k]));
            uint8_t hi = soar_oracle_e2m1_nibble_of_value(copysignf(fabsf(qbest[2 * k + 1]), wv[2 * k + 1]));
            codes[i * (MX_BLOCK / 2) + k] = (uint8_t)(lo | (hi << 4));
        }
    }
    if (sse) *sse = tree_sum(errs, nblk);
    if (status) *status = nonfinite ? ORACLE_STATUS_NONFINITE : 0;
    free(errs);
    return 0;
}

/* w^_ij = q_ij * X_i (exact in binary32 unless it underflows); out_dtype BF16 rounds to nearest even. */
int soar_oracle_mxfp4_dequantize(const uint8_t *codes, const uint8_t *scales, int64_t rows, int64_t cols,
                                 int out_dtype, void *out, int64_t ld)
{
    if (!codes || !scales || !out) return -1;
    if (rows <= 0 || cols <= 0 || cols % MX_BLOCK != 0 || ld < cols) return -1;
    if (out_dtype != ORACLE_BF16 && out_dtype != ORACLE_FP32) return -1;
    const int64_t bpr = cols / MX_BLOCK;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows * bpr; ++i) {
        int64_t r = i / bpr, cb = i % bpr;
        if (scales[i] == 255) continue;
        float s = e8m0_value(scales[i]);
        for (int j = 0; j < MX_BLOCK; ++j) {
            uint8_t byte = codes[i * (MX_BLOCK / 2) + j / 2];
            uint8_t nib = (j & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 0xF);
            float v = soar_oracle_e2m1_value(nib) * s;
            int64_t o = r * ld + cb * MX_BLOCK + j;
            if (out_dtype == ORACLE_BF16) ((uint16_t *)out)[o] = soar_oracle_f32_to_bf16(v);
            else ((float *)out)[o] = v;
        }
    }
    return 0;
}
