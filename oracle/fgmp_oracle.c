/*
 * FGMP oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, step-by-step CPU statement of what the FGMP inference hot
 * path computes (arxiv 2504.14152): Fisher-weighted block scoring, the
 * FP8-E4M3 / NVFP4 precision decision, the two encodings, and the matrix
 * product over the encoded operands.  Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may use it.  It shares no code, header, table
 * or helper with the HIP library and never calls it.
 *
 * Arithmetic rules (all fp32 steps are single, separately rounded IEEE
 * operations; build with -ffp-contract=off and without fast-math):
 *
 *   formats   E2M1 (4 bit: s e1 e0 m; magnitudes 0,.5,1,1.5,2,3,4,6) and
 *             OCP E4M3 "FN" (bias 7, subnormal step 2^-9, max 448, 0x7F/0xFF
 *             are NaN and never produced)                        [Sec. 4]
 *   rounding  nearest representable magnitude, ties to the even code,
 *             saturating at the format maximum, sign bit copied from the input
 *   block     16 consecutive elements along the dot-product dimension
 *                                                             [Sec. 1, Sec. 4]
 *   NVFP4     block scale from the block maximum ("dynamic max") [Sec. 3.3],
 *             stored as E4M3; values as E2M1                     [Sec. 4]
 *   FP8       E4M3 values, no block scale                        [Sec. 5.1]
 *   score     sum_i F_i * (x_i - Q_NVFP4(x_i))^2                 [Eq. 6, Eq. 2]
 *   decision  block kept in FP8 iff score > threshold (strict)   [Sec. 4.2]
 *   product   FP32-or-better accumulation of block dot products; the block
 *             scale multiplies only where an FP4 operand is involved
 *                                                                [Sec. 4.1]
 *   threshold order statistic of the scores of one tensor        [Eq. 9]
 *   gate      h = SiLU(g) * u in front of the output quantizer; not in the
 *             paper, defined further down as a fixed fp32 sequence
 *
 * Readings the paper leaves open (one FP32 scale S per tensor, RNE for the
 * block scale, one reciprocal per block, balanced summation tree, zero block
 * scale, strict compare, percentile direction) are fixed here and listed in
 * the design notes of the repository.
 *
 * Pins: the codecs are pinned by the format definitions (tables, tie points,
 * an independent library cast), the quantizer by exact-representability and
 * scaling invariants and an fp64 recomputation, the threshold by its counting
 * property, the product by numpy fp64 brute force and its two single-format
 * special cases, the byte accounting by the memory savings the paper prints
 * (Sec. 5.4.1), the gated activation and its exponential by the fp64
 * functions (units in the last place) and their closed forms.  End-to-end model quality (perplexity etc.) is "parity
 * unpinned": the paper prints no worked example of a quantized block.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define FGMP_ORACLE_BLOCK 16

/* ------------------------------------------------------------------ */
/* Formats                                                             */
/* ------------------------------------------------------------------ */

/* Magnitude of an E2M1 code's low three bits: exponent bias 1, one mantissa
 * bit, subnormal 0.5 [Sec. 4]. */
static double e2m1_magnitude(unsigned code3)
{
    unsigned e = (code3 >> 1) & 3u, m = code3 & 1u;
    if (e == 0) return 0.5 * (double)m;
    return (1.0 + 0.5 * (double)m) * ldexp(1.0, (int)e - 1);
}

/* Magnitude of an E4M3 code's low seven bits (0..0x7E): bias 7, three
 * mantissa bits, subnormals m * 2^-9 [Sec. 4]. */
static double e4m3_magnitude(unsigned code7)
{
    unsigned e = (code7 >> 3) & 15u, m = code7 & 7u;
    if (e == 0) return ldexp((double)m, -9);
    return (1.0 + (double)m / 8.0) * ldexp(1.0, (int)e - 7);
}

float fgmp_oracle_e2m1_decode(uint8_t code)
{
    double v = e2m1_magnitude(code & 7u);
    return (float)((code & 8u) ? -v : v);
}

float fgmp_oracle_e4m3_decode(uint8_t code)
{
    if ((code & 0x7Fu) == 0x7Fu) return NAN;
    double v = e4m3_magnitude(code & 0x7Fu);
    return (float)((code & 0x80u) ? -v : v);
}

/* The magnitudes of every code, tabulated once at load time from the two
 * formulas above (code order = magnitude order). */
static double E2M1_MAG[8];
static double E4M3_MAG[127];

__attribute__((constructor)) static void fill_magnitude_tables(void)
{
    for (unsigned c = 0; c < 8; ++c) E2M1_MAG[c] = e2m1_magnitude(c);
    for (unsigned c = 0; c < 127; ++c) E4M3_MAG[c] = e4m3_magnitude(c);
}

/* Round |r| to the nearest of the n_codes magnitudes mag[0] < mag[1] < ...;
 * a tie goes to the even code; anything beyond the last magnitude saturates
 * to it (clamped first, so that the differences below stay exact).
 * Differences are taken in fp64, where fp32 inputs up to the format maximum
 * and the format's magnitudes are exact, so an exact tie is seen as one. */
static unsigned nearest_code(double a, const double *mag, unsigned n_codes)
{
    if (a > mag[n_codes - 1]) a = mag[n_codes - 1];
    unsigned best = 0;
    double best_err = fabs(a - mag[0]);
    for (unsigned c = 1; c < n_codes; ++c) {
        double err = fabs(a - mag[c]);
        if (err < best_err || (err == best_err && (c & 1u) == 0u)) {
            best = c;
            best_err = err;
        }
    }
    return best;
}

static unsigned sign_of(float r)
{
    uint32_t bits;
    memcpy(&bits, &r, sizeof bits);
    return bits >> 31;
}

uint8_t fgmp_oracle_e2m1_encode(float r)
{
    unsigned c = nearest_code(fabs((double)r), E2M1_MAG, 8);
    return (uint8_t)((sign_of(r) << 3) | c);
}

uint8_t fgmp_oracle_e4m3_encode(float r)
{
    unsigned c = nearest_code(fabs((double)r), E4M3_MAG, 127);
    return (uint8_t)((sign_of(r) << 7) | c);
}

void fgmp_oracle_e2m1_encode_many(const float *r, int64_t n, uint8_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = fgmp_oracle_e2m1_encode(r[i]);
}

void fgmp_oracle_e4m3_encode_many(const float *r, int64_t n, uint8_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = fgmp_oracle_e4m3_encode(r[i]);
}

/* ------------------------------------------------------------------ */
/* One block                                                           */
/* ------------------------------------------------------------------ */

/* Quantize one block of 16 values x with sensitivities f (both fp32).
 * S is the tensor's FP32 scale, T the calibrated threshold.
 * Writes 16 code bytes (E2M1 nibble value 0..15, or E4M3 byte), the E4M3
 * block scale (0 for an FP8 block), the mask (1 = FP8) and the score. */
/* score_mode 0: the block's score is the sensitivity-weighted NVFP4 error
 * [Eq. 6 with the low-precision error of Eq. 2].  score_mode 1: the weighted
 * square of the error *increase* from keeping the block in NVFP4 rather than
 * FP8, Q_NVFP4(v) - Q_FP8(v) [Eq. 7, Eq. 8]; with the weights set to one, or
 * to the other operand's mean squared channel magnitude, the same sum is the
 * "quantization error" and "output error" baseline policy [Sec. 3.4, Eq. 12, Eq. 13]. */
/* Sensitivity-weighted NVFP4 error of one block under the block scale code sc
 * [the objective of Eq. 11]: the same arithmetic as the scoring below. */
static float nvfp4_error_with_scale(const float *x, const float *f, float S,
                                    uint8_t sc)
{
    const float d = fgmp_oracle_e4m3_decode(sc) * S;
    float inv_d = 0.0f;
    if (sc != 0) inv_d = 1.0f / d;
    float lvl[FGMP_ORACLE_BLOCK];
    for (int i = 0; i < FGMP_ORACLE_BLOCK; ++i) {
        float xhat = 0.0f;
        if (sc != 0)
            xhat = fgmp_oracle_e2m1_decode(fgmp_oracle_e2m1_encode(x[i] * inv_d)) * d;
        float e = x[i] - xhat;
        float e2 = e * e;
        lvl[i] = e2 * f[i];
    }
    for (int width = FGMP_ORACLE_BLOCK; width > 1; width /= 2)
        for (int i = 0; i < width / 2; ++i) lvl[i] = lvl[2 * i] + lvl[2 * i + 1];
    return lvl[0];
}

/* Sensitivity-weighted clipping [Sec. 3.3, Eq. 11]: brute force over every
 * non-negative E4M3 scale code (0 .. 0x7E); the code with the smallest weighted
 * error wins, the smallest code among equals. */
static uint8_t clipped_scale(const float *x, const float *f, float S)
{
    uint8_t best = 0;
    float best_err = nvfp4_error_with_scale(x, f, S, 0);
    for (int sc = 1; sc <= 0x7E; ++sc) {
        float err = nvfp4_error_with_scale(x, f, S, (uint8_t)sc);
        if (err < best_err) {
            best_err = err;
            best = (uint8_t)sc;
        }
    }
    return best;
}

static void quantize_block(const float *x, const float *f, float S, float T,
                           int score_mode, int clip, uint8_t *codes,
                           uint8_t *scale, uint8_t *mask, float *score)
{
    const float inv_S = 1.0f / S;
    const float S6 = 6.0f * S; /* largest E2M1 magnitude times the tensor scale */

    /* dynamic-max block scale [Sec. 3.3], stored as E4M3 [Sec. 4]; or the
     * clipped one [Eq. 11] */
    float amax = 0.0f;
    for (int i = 0; i < FGMP_ORACLE_BLOCK; ++i) {
        float a = fabsf(x[i]);
        if (a > amax) amax = a;
    }
    const float u = amax / S6;
    const uint8_t sc = clip ? clipped_scale(x, f, S) : fgmp_oracle_e4m3_encode(u);
    const float d = fgmp_oracle_e4m3_decode(sc) * S;

    /* NVFP4 values and their reconstruction */
    uint8_t q[FGMP_ORACLE_BLOCK];
    float t[FGMP_ORACLE_BLOCK];
    float inv_d = 0.0f;
    if (sc != 0) inv_d = 1.0f / d;
    for (int i = 0; i < FGMP_ORACLE_BLOCK; ++i) {
        float xhat;
        if (sc == 0) {
            q[i] = (uint8_t)(sign_of(x[i]) << 3);
            xhat = 0.0f;
        } else {
            float r = x[i] * inv_d;
            q[i] = fgmp_oracle_e2m1_encode(r);
            xhat = fgmp_oracle_e2m1_decode(q[i]) * d;
        }
        /* quantization error [Eq. 2] and its sensitivity-weighted square
         * [Eq. 6]; the sign convention of the error does not matter */
        float e;
        if (score_mode == 0) {
            e = x[i] - xhat;
        } else {
            /* the same element kept in FP8: (Q4 - v) - (Q8 - v) = Q4 - Q8 */
            float x8 = fgmp_oracle_e4m3_decode(fgmp_oracle_e4m3_encode(x[i] * inv_S)) * S;
            e = xhat - x8;
        }
        float e2 = e * e;
        t[i] = e2 * f[i];
    }

    /* balanced tree over adjacent pairs, fp32 */
    float lvl[FGMP_ORACLE_BLOCK];
    for (int i = 0; i < FGMP_ORACLE_BLOCK; ++i) lvl[i] = t[i];
    for (int width = FGMP_ORACLE_BLOCK; width > 1; width /= 2)
        for (int i = 0; i < width / 2; ++i) lvl[i] = lvl[2 * i] + lvl[2 * i + 1];
    *score = lvl[0];

    /* precision decision [Sec. 4.2] */
    if (lvl[0] > T) {
        *mask = 1;
        *scale = 0; /* FP8 carries no block scale [Sec. 5.1] */
        for (int i = 0; i < FGMP_ORACLE_BLOCK; ++i)
            codes[i] = fgmp_oracle_e4m3_encode(x[i] * inv_S);
    } else {
        *mask = 0;
        *scale = sc;
        for (int i = 0; i < FGMP_ORACLE_BLOCK; ++i) codes[i] = q[i];
    }
}

/* ------------------------------------------------------------------ */
/* Tensors                                                             */
/* ------------------------------------------------------------------ */

/* Quantize a rows x K tensor (K contiguous, leading dimension ldx) in blocks
 * of 16 along K.  fisher: ld_fisher == 0 -> one value per K channel shared by
 * all rows (activations, Sec. 3.1); otherwise one value per element with that
 * leading dimension (weights, Sec. 3.1).
 * Outputs (row-major, caller-allocated): codes rows*K bytes, scales / mask /
 * scores rows*K/16 entries.  Returns 0, or -1 on a bad argument (null pointer,
 * non-positive size, K not a multiple of 16, non-finite input or scale). */
static int quantize_tensor(const float *x, int64_t rows, int64_t K, int64_t ldx,
                           const float *fisher, int64_t ld_fisher, float T,
                           float S, int score_mode, int clip, uint8_t *codes,
                           uint8_t *scales, uint8_t *mask, float *scores)
{
    if (!x || !fisher || !codes || !scales || !mask || !scores) return -1;
    if (score_mode != 0 && score_mode != 1) return -1;
    if (rows <= 0 || K <= 0 || K % FGMP_ORACLE_BLOCK != 0 || ldx < K) return -1;
    if (!(S > 0.0f) || !isfinite(S) || isnan(T)) return -1;
    const int64_t nb = K / FGMP_ORACLE_BLOCK;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t b = 0; b < nb; ++b) {
            const float *xb = x + r * ldx + b * FGMP_ORACLE_BLOCK;
            const float *fb = fisher + (ld_fisher ? r * ld_fisher : 0) +
                              b * FGMP_ORACLE_BLOCK;
            for (int i = 0; i < FGMP_ORACLE_BLOCK; ++i)
                if (!isfinite(xb[i]) || !isfinite(fb[i])) bad = 1;
            quantize_block(xb, fb, S, T, score_mode, clip,
                           codes + r * K + b * FGMP_ORACLE_BLOCK,
                           scales + r * nb + b, mask + r * nb + b,
                           scores + r * nb + b);
        }
    }
    return bad ? -1 : 0;
}

/* Score selected by score_mode (0: Eq. 6, 1: Eq. 8); dynamic-max block scales. */
int fgmp_oracle_quantize_mode(const float *x, int64_t rows, int64_t K, int64_t ldx,
                              const float *fisher, int64_t ld_fisher, float T,
                              float S, int score_mode, uint8_t *codes,
                              uint8_t *scales, uint8_t *mask, float *scores)
{
    return quantize_tensor(x, rows, K, ldx, fisher, ld_fisher, T, S, score_mode, 0,
                           codes, scales, mask, scores);
}

/* Offline weight quantization with sensitivity-weighted clipping of the block
 * scales [Sec. 3.3, Eq. 11]; the score of a block is its weighted NVFP4 error
 * under the chosen scale [Eq. 6]. */
int fgmp_oracle_quantize_clip(const float *x, int64_t rows, int64_t K, int64_t ldx,
                              const float *fisher, int64_t ld_fisher, float T,
                              float S, uint8_t *codes, uint8_t *scales,
                              uint8_t *mask, float *scores)
{
    return quantize_tensor(x, rows, K, ldx, fisher, ld_fisher, T, S, 0, 1, codes,
                           scales, mask, scores);
}

/* The default scoring [Eq. 6]. */
int fgmp_oracle_quantize(const float *x, int64_t rows, int64_t K, int64_t ldx,
                         const float *fisher, int64_t ld_fisher, float T,
                         float S, uint8_t *codes, uint8_t *scales,
                         uint8_t *mask, float *scores)
{
    return fgmp_oracle_quantize_mode(x, rows, K, ldx, fisher, ld_fisher, T, S, 0,
                                     codes, scales, mask, scores);
}

/* Real value (without the tensor scale) of every stored element:
 * FP8 block -> e4m3(code); FP4 block -> e2m1(code) * e4m3(block scale). */
int fgmp_oracle_dequantize(const uint8_t *codes, const uint8_t *scales,
                           const uint8_t *mask, int64_t rows, int64_t K,
                           double *out)
{
    if (!codes || !scales || !mask || !out || rows <= 0 || K <= 0 ||
        K % FGMP_ORACLE_BLOCK != 0)
        return -1;
    const int64_t nb = K / FGMP_ORACLE_BLOCK;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t b = 0; b < nb; ++b)
            for (int i = 0; i < FGMP_ORACLE_BLOCK; ++i) {
                int64_t k = b * FGMP_ORACLE_BLOCK + i;
                uint8_t c = codes[r * K + k];
                double v;
                if (mask[r * nb + b])
                    v = (double)fgmp_oracle_e4m3_decode(c);
                else
                    v = (double)fgmp_oracle_e2m1_decode(c) *
                        (double)fgmp_oracle_e4m3_decode(scales[r * nb + b]);
                out[r * K + k] = v;
            }
    return 0;
}

/* Matrix product over the encoded operands, Y = X * W^T [Sec. 3], for the
 * n_rows x n_cols sub-matrix given by row_idx (into X) and col_idx (into W);
 * a null index list means 0..n-1.  ax is M x K, aw is N x K: the dequantized
 * operands of fgmp_oracle_dequantize.  fp64, k ascending.
 *   Y[i][j]   = Sx*Sw * sum_k ax[row_i][k]*aw[col_j][k]
 *   tol[i][j] = 1e-5 * Sx*Sw * sum_k |ax[row_i][k]*aw[col_j][k]|
 * Both outputs are n_rows x n_cols, row-major. */
int fgmp_oracle_gemm(const double *ax, double Sx, const double *aw, double Sw,
                     int64_t K, const int64_t *row_idx, int64_t n_rows,
                     const int64_t *col_idx, int64_t n_cols, double *Y,
                     double *tol)
{
    if (!ax || !aw || !Y || !tol || K <= 0 || n_rows <= 0 || n_cols <= 0)
        return -1;
    const double SS = Sx * Sw;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t i = 0; i < n_rows; ++i)
        for (int64_t j = 0; j < n_cols; ++j) {
            const double *a = ax + (row_idx ? row_idx[i] : i) * K;
            const double *b = aw + (col_idx ? col_idx[j] : j) * K;
            double acc = 0.0, mag = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double p = a[k] * b[k];
                acc += p;
                mag += fabs(p);
            }
            Y[i * n_cols + j] = SS * acc;
            tol[i * n_cols + j] = 1e-5 * SS * mag;
        }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Gated activation in front of the output quantizer                   */
/* ------------------------------------------------------------------ */

/* The paper's unit quantizes a layer's results before they are written out
 * [Sec. 4.2]; between the two MLP products of the Llama models it evaluates
 * sits h = SiLU(g) * u with SiLU(g) = g / (1 + e^-g), which the paper does
 * not discuss.  Because the quantized codes depend on h to the last bit, h is
 * defined here as a fixed sequence of separately rounded fp32 operations:
 *
 *   E(x), x clamped to [-87, 88]:
 *     n = nearest integer to fl(x * fl(log2 e)), ties to even
 *     r = fl(fl(x - n * C1) - fl(n * C2)),  C1 = 0.693359375 (n * C1 is exact),
 *                                           C2 = fl(ln 2 - C1)
 *     p = the degree-7 Taylor polynomial of e^r by Horner's rule, every
 *         multiply and every add rounded to fp32, coefficients fl(1/k!)
 *     E = p * 2^n (exact)
 *   h = fl(fl(g / fl(1 + E(-g))) * u)
 *
 * |r| <= 0.347, so the polynomial's truncation error is below 2^-27; the
 * pins compare E and h with the fp64 functions (a few units in the last
 * place) and check the closed forms at 0 and for large |g|. */
static float exp_fp32_steps(float x)
{
    if (x > 88.0f) x = 88.0f;
    if (x < -87.0f) x = -87.0f;
    const float y = x * 1.44269504f;
    const float n = rintf(y); /* round-to-nearest-even is the default mode */
    float r = x - n * 0.693359375f;
    r = r - n * -2.12194440e-4f;
    static const float inv_fact[8] = {1.0f, 1.0f, 0.5f, 1.0f / 6.0f, 1.0f / 24.0f,
                                      1.0f / 120.0f, 1.0f / 720.0f, 1.0f / 5040.0f};
    float p = inv_fact[7];
    for (int k = 6; k >= 0; --k) {
        const float pr = p * r;
        p = pr + inv_fact[k];
    }
    union { uint32_t u; float f; } two_n;
    two_n.u = (uint32_t)((int)n + 127) << 23;
    return p * two_n.f;
}

float fgmp_oracle_exp_steps(float x) { return exp_fp32_steps(x); }

/* h[i] = SiLU(g[i]) * u[i] as defined above. */
void fgmp_oracle_silu_mul(const float *g, const float *u, int64_t n, float *h)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const float e = exp_fp32_steps(-g[i]);
        const float d = 1.0f + e;
        const float s = g[i] / d;
        h[i] = s * u[i];
    }
}

/* The same two functions written a second, structurally different way, as
 * a cross-check of the sequence above (used by the pins only, never by a
 * parity test): no range reduction, no polynomial -- the C library's fp64
 * exponential and ONE rounding to fp32 at the very end.  E_ref(x) is the
 * correctly rounded fp32 value of e^x (x clamped like above); h_ref is the
 * fp32 nearest to g / (1 + e^-g) * u evaluated in fp64. */
float fgmp_oracle_exp_rounded_once(float x)
{
    double xd = (double)x;
    if (xd > 88.0) xd = 88.0;
    if (xd < -87.0) xd = -87.0;
    return (float)exp(xd);
}

void fgmp_oracle_silu_mul_rounded_once(const float *g, const float *u, int64_t n, float *h)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const double gd = (double)g[i];
        h[i] = (float)(gd / (1.0 + exp(-gd)) * (double)u[i]);
    }
}

/* ------------------------------------------------------------------ */
/* Threshold for a target fraction of high-precision blocks [Eq. 9]    */
/* ------------------------------------------------------------------ */

static int cmp_float(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return (x > y) - (x < y);
}

/* The threshold T for which round(p*J) of the J scores lie strictly above
 * it (when the boundary score is not tied): the score that sits just below
 * the round(p*J) largest ones.  p = 0 -> +inf, p = 1 -> -inf. */
float fgmp_oracle_threshold(const float *scores, int64_t J, double p)
{
    if (!scores || J <= 0 || !(p >= 0.0) || !(p <= 1.0)) return NAN;
    int64_t n_hi = (int64_t)floor(p * (double)J + 0.5);
    if (n_hi <= 0) return INFINITY;
    if (n_hi >= J) return -INFINITY;
    float *sorted = (float *)malloc((size_t)J * sizeof(float));
    if (!sorted) return NAN;
    memcpy(sorted, scores, (size_t)J * sizeof(float));
    qsort(sorted, (size_t)J, sizeof(float), cmp_float);
    float T = sorted[J - n_hi - 1];
    free(sorted);
    return T;
}

/* ------------------------------------------------------------------ */
/* Storage accounting [Sec. 5.4.1]                                     */
/* ------------------------------------------------------------------ */

/* Bits needed by n_lo NVFP4 blocks and n_hi FP8 blocks: 16 four-bit values
 * plus one 8-bit scale, or 16 eight-bit values and no scale, plus one
 * metadata bit per block [Sec. 4]. */
int64_t fgmp_oracle_storage_bits(int64_t n_lo, int64_t n_hi)
{
    return n_lo * (16 * 4 + 8) + n_hi * (16 * 8) + (n_lo + n_hi);
}

/* Threads the OpenMP loops above will use (reported beside timings). */
int fgmp_oracle_num_threads(void) { return omp_get_max_threads(); }

/* Number of threads for the loops above from now on (for timing the oracle on one core). */
void fgmp_oracle_set_num_threads(int n)
{
    if (n > 0) omp_set_num_threads(n);
}
