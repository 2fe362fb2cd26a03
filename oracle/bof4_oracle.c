/*
 * CPU oracle for block-wise (signed) absmax 4-bit quantisation with BOF4 / BOF4-S codebooks, OPQ
 * outlier extraction and the empirical (Monte-Carlo) Lloyd / EM step of arxiv 2505.06653.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a deliberately slow, scalar, one-block-at-a-time
 * transcription of the paper's definitions, used only to check the HIP library and to give a reported CPU
 * baseline.  It shares no code, header, table or helper with the HIP path and must never be called from it.
 *
 * Every function cites the passage of the paper it follows.  Where the paper leaves a rounding, a tie or
 * a storage format open, the choice made here is stated next to the code.
 *
 * Pins (see tests, all CPU-only):
 *   nearest-level assignment   : exact rational brute force over all 16 levels on tiny inputs, incl. exact ties
 *   signed absmax + scale      : block maximum reconstructs bit-exactly; other elements within half a level gap
 *   lloyd step / update        : weighted SSE non-increasing; fixed point on Gaussian samples equals the
 *                                numerically integrated closed form (appendix B.2) and the printed codebooks
 *   OPQ threshold / detection  : closed form F_M^{-1}; Monte-Carlo exceedance = 1-q; planted single outlier
 *   MAE step (weighted median): brute-force minimiser of sum a|x - c| on tiny inputs; the plain lower median
 *                                when all blocks weigh the same; fixed point on Gaussian samples equals the
 *                                printed MAE codebooks; one update from the MSE codebook equals the theoretical
 *                                update of section 3.2 eq. 7 (numerical integration, bisection); without weights
 *                                (appendix D) numpy's sorted lower median of every region on blocks of very
 *                                different maxima
 *   quantisation error         : zero on a tensor that is already decoded (Q is idempotent); one hand-made block;
 *                                within the decoder's rounding of the Lloyd step's sse (appendix B.3); the orderings
 *                                the paper reports (signed below absolute, MAE-/MSE-optimised best on their own
 *                                metric, OPQ lowers both)
 *   decoder inside a matrix-vector product: constant codes (level times sum of x), unit vectors (one column of
 *                                the decoded matrix), planted outliers, linearity, and the decoded bfloat16 matrix
 *                                times x within the decoder's rounding bound
 *   the product over the decoded bfloat16 matrix: equals a binary64 matrix product of oracle_dequantize's output
 *                                (library routine on an independently pinned function); unit vectors; within the
 *                                decoder's rounding of oracle_gemv
 *   tie rules (equal |w| of opposite sign, exact mid-point x, all-zero block, -0.0): parity unpinned by the
 *   paper - fixed only by the definitions written below.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp (OpenMP only splits independent blocks over cores;
 * per-block arithmetic and the order of every floating-point sum are the same for any thread count, see
 * oracle_lloyd_step).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_CAPACITY (-2)

#define NLEVELS 16

/* ---------------------------------------------------------------- 16-bit float formats ------------------ */

/* bfloat16 is the upper half of an IEEE binary32, so widening is a shift and exact. */
static float bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* binary32 -> bfloat16, round to nearest, ties to even. NaN stays NaN. */
static uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* binary32 -> binary16 (1-5-10), round to nearest, ties to even; overflow gives infinity, small values
 * become binary16 subnormals or zero.  Written from the format definition. */
static uint16_t f32_to_f16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);          /* NaN */
    if (a >= 0x47800000u) return (uint16_t)(sign | 0x7c00u);         /* |f| >= 65536 -> inf */
    int e = (int)(a >> 23) - 127;                                    /* unbiased exponent */
    uint32_t man = (a & 0x007fffffu);
    if (e >= -14) {
        /* normal binary16 candidate: keep 10 mantissa bits, drop 13 */
        uint32_t v = ((uint32_t)(e + 15) << 10) | (man >> 13);
        uint32_t rem = man & 0x1fffu;
        if (rem > 0x1000u || (rem == 0x1000u && (v & 1u))) v++;      /* may carry into exponent, incl. to inf */
        return (uint16_t)(sign | v);
    }
    if (e < -25) return sign;                                        /* below half the smallest subnormal */
    /* subnormal: value = man24 * 2^(e-23), unit 2^-24 */
    uint32_t man24 = man | 0x00800000u;
    int shift = (-14 - e) + 13;                                      /* 14..24 */
    uint32_t v = man24 >> shift;
    uint32_t rem = man24 & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (v & 1u))) v++;
    return (uint16_t)(sign | v);
}

/* binary16 -> binary32, exact. */
static float f16_to_f32(uint16_t h) {
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1fu;
    uint32_t man = h & 0x3ffu;
    float mag;
    if (e == 0) {
        mag = ldexpf((float)man, -24);
    } else if (e == 31) {
        mag = man ? NAN : INFINITY;
    } else {
        mag = ldexpf((float)(man | 0x400u), (int)e - 25);
    }
    uint32_t u;
    memcpy(&u, &mag, 4);
    u |= sign;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

uint16_t oracle_f32_to_f16(float f) { return f32_to_f16_rne(f); }
float oracle_f16_to_f32(uint16_t h) { return f16_to_f32(h); }
uint16_t oracle_f32_to_bf16(float f) { return f32_to_bf16_rne(f); }
float oracle_bf16_to_f32(uint16_t b) { return bf16_to_f32(b); }

/* ---------------------------------------------------------------- OPQ threshold ------------------------- */

/* Standard normal CDF through the complementary error function of libm. */
static double std_normal_cdf(double t) { return 0.5 * erfc(-t / sqrt(2.0)); }

/*
 * q-quantile of the absolute block maximum M of I i.i.d. standard normal weights (section 3.3, eq. 9, with
 * F_M = F_|W|^I and F_|W| = 2 F_W - 1 from appendix B.1):  F_M(t) = (2 G(t) - 1)^I = q.
 * Solved by plain bisection on F_M itself; t lies in (0, 40).
 */
double oracle_opq_threshold(double q, uint32_t I) {
    if (!(q > 0.0 && q < 1.0) || I < 2) return NAN;
    double lo = 0.0, hi = 40.0;
    for (int it = 0; it < 200; ++it) {
        double mid = 0.5 * (lo + hi);
        double FM = pow(2.0 * std_normal_cdf(mid) - 1.0, (double)I);
        if (FM < q) lo = mid; else hi = mid;
    }
    return 0.5 * (lo + hi);
}

/* ---------------------------------------------------------------- per-block front end -------------------- */

static int valid_block(uint32_t I) { return I == 32 || I == 64 || I == 128 || I == 256; }

static int valid_codebook(const double* cb) {
    for (int l = 0; l < NLEVELS; ++l)
        if (!isfinite(cb[l])) return 0;
    for (int l = 1; l < NLEVELS; ++l)
        if (!(cb[l] > cb[l - 1])) return 0;
    return 1;
}

/*
 * Decision thresholds xi(1..15) between neighbouring reconstruction levels: the nearest-neighbour rule of
 * Lloyd's algorithm (section 3.2, appendix B.2) puts them at the mid-points.
 */
static void midpoints(const double* cb, double* xi) {
    for (int k = 0; k < NLEVELS - 1; ++k) xi[k] = (cb[k] + cb[k + 1]) * 0.5;
}

/*
 * Index (0..15) of the reconstruction level nearest to x.  A value exactly on a mid-point goes to the lower
 * level (the paper's half-open regions would send it up; the difference has measure zero in its analysis and
 * the lower-index rule is what a first-minimum search over |x - level| returns).
 */
static int nearest_level(float x, const double* xi) {
    int code = 0;
    for (int k = 0; k < NLEVELS - 1; ++k)
        if ((double)x > xi[k]) code++;
    return code;
}

/*
 * Everything that happens to one block before the scalar quantiser is applied:
 *   1. OPQ (section 3.3, eq. 9; appendix E.1 eq. for sigma_b): element i is an outlier iff
 *        |w_i| > sigma_b * T,  sigma_b^2 = sum_i (w_i - mean)^2 / (I - 1)   over ALL I raw elements.
 *      Evaluated without square root or division as
 *        w_i^2 * I (I-1)  >  T^2 * V,   V = I * sum w^2 - (sum w)^2  = I (I-1) sigma_b^2,
 *      in binary64 with V = fma(-S, S, I*Q).  A constant block (V <= 0) has no outliers.  Outliers are
 *      replaced by +0 before the maximum search.
 *   2. block constant (section 2.1 eq. 1 / section 3.1 eq. 4): j* = lowest index of maximal |w|;
 *      m = |w_j*| (absolute) or w_j* (signed).  The constant is stored as binary16 and the quantiser
 *      normalises by the stored value, so encoder and decoder use the same number.
 *   3. normalisation (eq. 2): x_i = w_i / m in binary32, one correctly rounded division; a zero constant
 *      gives x_i = 0.
 * Outputs: wz[] weights after zeroing, is_out[] flags, x[] normalised weights, *scale16, *m_eff.
 */
static void block_front_end(const uint16_t* w, uint32_t I, int signed_norm, double T,
                            float* wz, uint8_t* is_out, float* x, uint16_t* scale16, float* m_eff) {
    for (uint32_t i = 0; i < I; ++i) {
        wz[i] = bf16_to_f32(w[i]);
        is_out[i] = 0;
    }
    if (T > 0.0) {
        double S = 0.0, Q = 0.0;
        for (uint32_t i = 0; i < I; ++i) {
            double d = (double)wz[i];
            S += d;
            Q += d * d;
        }
        double V = fma(-S, S, (double)I * Q);
        if (V > 0.0) {
            double rhs = (T * T) * V;
            double II1 = (double)I * (double)(I - 1);
            for (uint32_t i = 0; i < I; ++i) {
                double d = (double)wz[i];
                if ((d * d) * II1 > rhs) is_out[i] = 1;
            }
        }
        for (uint32_t i = 0; i < I; ++i)
            if (is_out[i]) wz[i] = 0.0f;
    }
    uint32_t jstar = 0;
    uint32_t best = 0;
    for (uint32_t i = 0; i < I; ++i) {
        uint32_t u;
        memcpy(&u, &wz[i], 4);
        uint32_t mag = u & 0x7fffffffu;
        if (i == 0 || mag > best) {
            best = mag;
            jstar = i;
        }
    }
    float m = signed_norm ? wz[jstar] : fabsf(wz[jstar]);
    *scale16 = f32_to_f16_rne(m);
    *m_eff = f16_to_f32(*scale16);
    for (uint32_t i = 0; i < I; ++i) x[i] = (*m_eff == 0.0f) ? 0.0f : wz[i] / *m_eff;
}

/* ---------------------------------------------------------------- quantise -------------------------------- */

/*
 * Block-wise (signed) absmax quantisation with optional OPQ (sections 2.1, 3.1, 3.3).
 *   w        n bfloat16 weights, flat; block b is w[b*I .. b*I+I-1]
 *   codes    n/2 bytes; element 2j in the low nibble of byte j, element 2j+1 in the high nibble;
 *            code = zero-based level index
 *   scales   n/I binary16 block constants
 *   out_idx / out_val  outliers in ascending flat index, value as binary16 (exact for every bfloat16 whose
 *            magnitude lies in binary16's normal range); at most `capacity` are written
 *   *n_outliers  number found (also when it exceeds capacity, then ORACLE_ERR_CAPACITY is returned)
 */
int oracle_quantize(const uint16_t* w, uint64_t n, uint32_t I, const double* cb, int signed_norm, double T,
                    uint8_t* codes, uint16_t* scales, int64_t* out_idx, uint16_t* out_val, uint64_t capacity,
                    uint64_t* n_outliers) {
    if (!w || !cb || !codes || !scales || !n_outliers) return ORACLE_ERR_ARG;
    if (!valid_block(I) || n == 0 || n % I != 0 || !valid_codebook(cb) || !(T >= 0.0)) return ORACLE_ERR_ARG;
    if (T > 0.0 && capacity > 0 && (!out_idx || !out_val)) return ORACLE_ERR_ARG;
    double xi[NLEVELS - 1];
    midpoints(cb, xi);
    uint64_t nout = 0;
    float wz[256], x[256];
    uint8_t is_out[256];
    for (uint64_t b = 0; b < n / I; ++b) {
        uint16_t s16;
        float m_eff;
        block_front_end(w + b * I, I, signed_norm, T, wz, is_out, x, &s16, &m_eff);
        scales[b] = s16;
        for (uint32_t i = 0; i < I; ++i) {
            uint64_t flat = b * I + i;
            if (is_out[i]) {
                if (nout < capacity) {
                    out_idx[nout] = (int64_t)flat;
                    out_val[nout] = f32_to_f16_rne(bf16_to_f32(w[flat]));
                }
                nout++;
            }
            int code = nearest_level(x[i], xi);
            if ((flat & 1u) == 0)
                codes[flat >> 1] = (uint8_t)code;
            else
                codes[flat >> 1] |= (uint8_t)(code << 4);
        }
    }
    *n_outliers = nout;
    return nout > capacity ? ORACLE_ERR_CAPACITY : ORACLE_OK;
}

/* ---------------------------------------------------------------- dequantise ------------------------------ */

/*
 * Decoder (section 2.1 eq. 3): w~ = m_b * level[code], evaluated as one binary32 multiply of the stored
 * constant with the level rounded to binary32, result rounded to bfloat16; outliers are written back last.
 */
int oracle_dequantize(const uint8_t* codes, const uint16_t* scales, uint64_t n, uint32_t I, const double* cb,
                      const int64_t* out_idx, const uint16_t* out_val, uint64_t n_outliers, uint16_t* w_out) {
    if (!codes || !scales || !cb || !w_out) return ORACLE_ERR_ARG;
    if (!valid_block(I) || n == 0 || n % I != 0 || !valid_codebook(cb)) return ORACLE_ERR_ARG;
    if (n_outliers > 0 && (!out_idx || !out_val)) return ORACLE_ERR_ARG;
    for (uint64_t k = 0; k < n_outliers; ++k)
        if (out_idx[k] < 0 || (uint64_t)out_idx[k] >= n) return ORACLE_ERR_ARG;
    for (uint64_t i = 0; i < n; ++i) {
        int code = (codes[i >> 1] >> ((i & 1u) * 4)) & 0xf;
        float s = f16_to_f32(scales[i / I]);
        float lv = (float)cb[code];
        w_out[i] = f32_to_bf16_rne(s * lv);
    }
    for (uint64_t k = 0; k < n_outliers; ++k) w_out[out_idx[k]] = f32_to_bf16_rne(f16_to_f32(out_val[k]));
    return ORACLE_OK;
}

/* ---------------------------------------------------------------- quantisation error --------------------- */

typedef struct {
    double sse;          /* sum over all n weights of (w - Q(w))^2                                             */
    double sae;          /* sum of |w - Q(w)|                                                                  */
    double max_abs;      /* largest |w - Q(w)|                                                                 */
    uint64_t n_outliers; /* weights stored as outliers                                                         */
    uint64_t n;          /* weights compared                                                                   */
} oracle_error_stats;

/*
 * The error of the quantiser on a tensor, as the paper reports it (MSE = sse / n, MAE = sae / n: section 5,
 * quantisation-error paragraphs and table; the decomposition of appendix B.3 is in terms of the same difference):
 * Q(w) is what oracle_dequantize returns for what oracle_quantize made of w - the decoded bfloat16 weight, or the
 * stored outlier.  Nothing else happens here: quantise, decode, subtract, add up in binary64 in index order.
 */
int oracle_quant_error(const uint16_t* w, uint64_t n, uint32_t I, const double* cb, int signed_norm, double T,
                       oracle_error_stats* out) {
    if (!w || !cb || !out) return ORACLE_ERR_ARG;
    if (!valid_block(I) || n == 0 || n % I != 0 || !valid_codebook(cb) || !(T >= 0.0)) return ORACLE_ERR_ARG;
    uint8_t* codes = (uint8_t*)malloc(n / 2);
    uint16_t* scales = (uint16_t*)malloc((n / I) * sizeof(uint16_t));
    uint16_t* deq = (uint16_t*)malloc(n * sizeof(uint16_t));
    const uint64_t cap = T > 0.0 ? n : 0;
    int64_t* oidx = (int64_t*)malloc((cap ? cap : 1) * sizeof(int64_t));
    uint16_t* oval = (uint16_t*)malloc((cap ? cap : 1) * sizeof(uint16_t));
    int st = ORACLE_ERR_ARG;
    if (codes && scales && deq && oidx && oval) {
        uint64_t k = 0;
        st = oracle_quantize(w, n, I, cb, signed_norm, T, codes, scales, oidx, oval, cap, &k);
        if (st == ORACLE_OK) st = oracle_dequantize(codes, scales, n, I, cb, oidx, oval, k, deq);
        if (st == ORACLE_OK) {
            double sse = 0.0, sae = 0.0, mx = 0.0;
            for (uint64_t i = 0; i < n; ++i) {
                const double d = (double)bf16_to_f32(w[i]) - (double)bf16_to_f32(deq[i]);
                sse += d * d;
                sae += fabs(d);
                if (fabs(d) > mx) mx = fabs(d);
            }
            out->sse = sse;
            out->sae = sae;
            out->max_abs = mx;
            out->n_outliers = k;
            out->n = n;
        }
    }
    free(codes);
    free(scales);
    free(deq);
    free(oidx);
    free(oval);
    return st;
}

/* ---------------------------------------------------------------- decoder inside a matrix-vector product --- */

/*
 * The decoder in use (section 2.1 eq. 3 inside a linear layer; section 3.3 for the outliers; the inference setting of
 * the appendix on OPQ runtime): the quantised tensor is a row-major [rows x cols] matrix, blocks run along the flat
 * layout, and for every token t
 *     y[t][r] = sum_c  w~[r][c] * x[t][c],      w~ = m_b * level[code]   (the exact product of eq. 3, not rounded),
 * except at listed outlier positions, where w~ is the stored binary16 value (of two entries with one index the later
 * wins).  The level is taken as the decoder stores it (rounded to binary32); everything else is binary64.  abs_out
 * receives sum_c |w~ x|, the scale of the rounding error of any finite-precision evaluation.
 */
int oracle_gemv(const uint8_t* codes, const uint16_t* scales, uint64_t rows, uint64_t cols, uint32_t I,
                const double* cb, const int64_t* out_idx, const uint16_t* out_val, uint64_t n_outliers,
                const uint16_t* x, uint32_t n_tokens, double* y, double* abs_out) {
    if (!codes || !scales || !cb || !x || !y) return ORACLE_ERR_ARG;
    if (!valid_block(I) || rows == 0 || cols == 0 || cols % I != 0 || n_tokens == 0 || !valid_codebook(cb))
        return ORACLE_ERR_ARG;
    if (n_outliers > 0 && (!out_idx || !out_val)) return ORACLE_ERR_ARG;
    const uint64_t n = rows * cols;
    for (uint64_t k = 0; k < n_outliers; ++k)
        if (out_idx[k] < 0 || (uint64_t)out_idx[k] >= n) return ORACLE_ERR_ARG;
    double* wt = (double*)malloc(n * sizeof(double));
    if (!wt) return ORACLE_ERR_ARG;
    for (uint64_t i = 0; i < n; ++i) {
        int code = (codes[i >> 1] >> ((i & 1u) * 4)) & 0xf;
        wt[i] = (double)f16_to_f32(scales[i / I]) * (double)(float)cb[code];
    }
    for (uint64_t k = 0; k < n_outliers; ++k) wt[out_idx[k]] = (double)f16_to_f32(out_val[k]);
    for (uint32_t t = 0; t < n_tokens; ++t)
        for (uint64_t r = 0; r < rows; ++r) {
            double acc = 0.0, aacc = 0.0;
            for (uint64_t c = 0; c < cols; ++c) {
                const double term = wt[r * cols + c] * (double)bf16_to_f32(x[(uint64_t)t * cols + c]);
                acc += term;
                aacc += fabs(term);
            }
            y[(uint64_t)t * rows + r] = acc;
            if (abs_out) abs_out[(uint64_t)t * rows + r] = aacc;
        }
    free(wt);
    return ORACLE_OK;
}

/*
 * The same product for many tokens as an inference engine runs it (the paper's decode path: decode the matrix to
 * bfloat16, then a bfloat16 matrix product): y[t][r] = sum_c W^[r][c] * x[t][c] with W^ exactly what oracle_dequantize
 * returns - every weight rounded to bfloat16 (section 2.1 eq. 3), outliers written back (section 3.3).  Binary64 sums.
 */
int oracle_gemm(const uint8_t* codes, const uint16_t* scales, uint64_t rows, uint64_t cols, uint32_t I,
                const double* cb, const int64_t* out_idx, const uint16_t* out_val, uint64_t n_outliers,
                const uint16_t* x, uint32_t n_tokens, double* y, double* abs_out) {
    if (!codes || !scales || !cb || !x || !y) return ORACLE_ERR_ARG;
    if (rows == 0 || cols == 0 || n_tokens == 0 || (valid_block(I) && cols % I != 0)) return ORACLE_ERR_ARG;
    const uint64_t n = rows * cols;
    uint16_t* deq = (uint16_t*)malloc(n * sizeof(uint16_t));
    if (!deq) return ORACLE_ERR_ARG;
    int st = oracle_dequantize(codes, scales, n, I, cb, out_idx, out_val, n_outliers, deq);
    if (st == ORACLE_OK) {
        for (uint32_t t = 0; t < n_tokens; ++t)
            for (uint64_t r = 0; r < rows; ++r) {
                double acc = 0.0, aacc = 0.0;
                for (uint64_t c = 0; c < cols; ++c) {
                    const double term = (double)bf16_to_f32(deq[r * cols + c]) *
                                        (double)bf16_to_f32(x[(uint64_t)t * cols + c]);
                    acc += term;
                    aacc += fabs(term);
                }
                y[(uint64_t)t * rows + r] = acc;
                if (abs_out) abs_out[(uint64_t)t * rows + r] = aacc;
            }
    }
    free(deq);
    return st;
}

/* ---------------------------------------------------------------- Lloyd / EM ------------------------------ */

typedef struct {
    double num[NLEVELS];   /* sum over region l of  g * x          (numerator of section 3.2 eq. 6)   */
    double den[NLEVELS];   /* sum over region l of  g              (denominator of eq. 6)             */
    uint64_t cnt[NLEVELS]; /* K_l, number of normalised weights in region l                           */
    double sse;            /* sum of g * (x - level[code])^2  (appendix B.3, MSE decomposition)       */
    uint64_t n_used;       /* weights that entered the statistics (n minus outliers)                  */
    uint64_t n_outliers;
} oracle_lloyd_stats;

/*
 * One expectation pass of the data-driven Lloyd algorithm (section 3.2 eq. 6; appendix B.3): normalise every
 * block, assign each normalised weight to its nearest level, and accumulate per region the sums of eq. 6 with
 * g = (block constant)^2 (weight_by_max2 != 0), or g = 1 for the plain normalised-error variant of appendix D.
 * Outliers (OPQ on) are stored exactly and therefore take no part.
 *
 * All sums are binary64.  Blocks are split into a fixed number of contiguous chunks (independent of the thread
 * count); each chunk is summed left to right and the chunk totals are added in chunk order, so the result does
 * not depend on how many threads ran.
 */
#define LLOYD_CHUNKS 64
int oracle_lloyd_step(const uint16_t* w, uint64_t n, uint32_t I, const double* cb, int signed_norm, double T,
                      int weight_by_max2, oracle_lloyd_stats* out) {
    if (!w || !cb || !out) return ORACLE_ERR_ARG;
    if (!valid_block(I) || n == 0 || n % I != 0 || !valid_codebook(cb) || !(T >= 0.0)) return ORACLE_ERR_ARG;
    double xi[NLEVELS - 1];
    midpoints(cb, xi);
    uint64_t B = n / I;
    oracle_lloyd_stats* part = (oracle_lloyd_stats*)calloc(LLOYD_CHUNKS, sizeof(oracle_lloyd_stats));
    if (!part) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < LLOYD_CHUNKS; ++c) {
        uint64_t b0 = B * (uint64_t)c / LLOYD_CHUNKS, b1 = B * (uint64_t)(c + 1) / LLOYD_CHUNKS;
        oracle_lloyd_stats* p = &part[c];
        float wz[256], x[256];
        uint8_t is_out[256];
        for (uint64_t b = b0; b < b1; ++b) {
            uint16_t s16;
            float m_eff;
            block_front_end(w + b * I, I, signed_norm, T, wz, is_out, x, &s16, &m_eff);
            double g = weight_by_max2 ? (double)m_eff * (double)m_eff : 1.0;
            for (uint32_t i = 0; i < I; ++i) {
                if (is_out[i]) {
                    p->n_outliers++;
                    continue;
                }
                int code = nearest_level(x[i], xi);
                double xd = (double)x[i];
                double d = xd - cb[code];
                p->cnt[code]++;
                p->den[code] += g;
                p->num[code] += g * xd;
                p->sse += g * d * d;
                p->n_used++;
            }
        }
    }
    memset(out, 0, sizeof(*out));
    for (int c = 0; c < LLOYD_CHUNKS; ++c) {
        for (int l = 0; l < NLEVELS; ++l) {
            out->num[l] += part[c].num[l];
            out->den[l] += part[c].den[l];
            out->cnt[l] += part[c].cnt[l];
        }
        out->sse += part[c].sse;
        out->n_used += part[c].n_used;
        out->n_outliers += part[c].n_outliers;
    }
    free(part);
    return ORACLE_OK;
}

/*
 * Maximisation step (section 3.2 eq. 6 and the last paragraph of 3.2): every level that is not pinned and whose
 * region is not empty moves to num/den; pinned levels (bit l of pinned_mask set) and empty regions keep their
 * value.
 */
int oracle_codebook_update(const oracle_lloyd_stats* st, uint16_t pinned_mask, double* cb) {
    if (!st || !cb) return ORACLE_ERR_ARG;
    for (int l = 0; l < NLEVELS; ++l) {
        if ((pinned_mask >> l) & 1u) continue;
        if (st->den[l] > 0.0) cb[l] = st->num[l] / st->den[l];
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------- Lloyd / EM, MAE criterion ---------------- */

typedef struct {
    double median[NLEVELS]; /* weighted median of the normalised weights of region l (NaN: no weight there)   */
    double den[NLEVELS];    /* sum over region l of |block constant|                                          */
    uint64_t cnt[NLEVELS];  /* K_l                                                                            */
    double sae;             /* sum of |block constant| * |x - level[code]|: n_used * MAE(W, Q(W))             */
    uint64_t n_used;
    uint64_t n_outliers;
} oracle_mae_stats;

typedef struct {
    float x;
    uint16_t a16; /* |block constant| as stored (binary16 bit pattern without the sign) */
} mae_sample;

static int cmp_mae_sample(const void* pa, const void* pb) {
    float a = ((const mae_sample*)pa)->x, b = ((const mae_sample*)pb)->x;
    return (a > b) - (a < b);
}

/* |block constant| * 2^24 as an integer: exact for every binary16 number (the smallest subnormal is 2^-24).  A
 * constant that overflowed binary16 (infinite; out of contract) carries no weight. */
static uint64_t weight_units(uint16_t a16) {
    if (a16 >= 0x7C00u) return 0;
    return (uint64_t)ldexp((double)f16_to_f32(a16), 24);
}

/* What a normalised weight counts with in its region's median: its block's constant (eq. 8), or one unit for the
 * plain median of appendix D. */
static uint64_t sample_weight(uint16_t a16, int weight_by_max) {
    if (a16 >= 0x7C00u) return 0;
    return weight_by_max ? weight_units(a16) : 1;
}

/*
 * One expectation pass of Lloyd's algorithm under the MAE criterion (section 3.2 eq. 7-8; appendix B.4): the
 * new level of region l minimises f(c) = sum_k a_k |x_k - c| over the normalised weights x_k of the region, a_k
 * being the absolute block maximum of the block that holds x_k (the same for absolute and signed normalisation).
 * Every minimiser is a weighted median.  The appendix derives that f falls on (x_kappa, x_kappa+1) as long as
 * sum_{k<=kappa} a_k <= sum_{k>kappa} a_k and rises afterwards, which puts the minimum at the element AFTER
 * the last kappa for which the inequality holds; its closing formula names x_kappa itself, one element early
 * (for x = 1, 2, 3 with equal weights it would give 1).  Taken here: the smallest value v among the x_k with
 *     2 * sum_{x_k <= v} a_k  >=  sum_k a_k ,
 * i.e. the lower weighted median; it minimises f (checked by brute force in the tests) and does not depend on
 * the order of equal x_k.  Weights are added as exact integers (units of 2^-24) in 128 bits.  Elements of weight
 * zero (all-zero blocks) cannot move f and are left out; a region without weight reports NaN and keeps its level.
 */
int oracle_lloyd_step_mae(const uint16_t* w, uint64_t n, uint32_t I, const double* cb, int signed_norm, double T,
                          int weight_by_max, oracle_mae_stats* out) {
    if (!w || !cb || !out) return ORACLE_ERR_ARG;
    if (!valid_block(I) || n == 0 || n % I != 0 || !valid_codebook(cb) || !(T >= 0.0)) return ORACLE_ERR_ARG;
    double xi[NLEVELS - 1];
    midpoints(cb, xi);
    const uint64_t B = n / I;
    mae_sample* all = (mae_sample*)malloc((size_t)n * sizeof(mae_sample));
    uint8_t* code_of = (uint8_t*)malloc((size_t)n);
    if (!all || !code_of) {
        free(all);
        free(code_of);
        return ORACLE_ERR_ARG;
    }
    memset(out, 0, sizeof(*out));
    /* pass 1: normalise and classify every element; 255 marks an outlier */
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < (int64_t)B; ++b) {
        float wz[256], x[256];
        uint8_t is_out[256];
        uint16_t s16;
        float m_eff;
        block_front_end(w + (uint64_t)b * I, I, signed_norm, T, wz, is_out, x, &s16, &m_eff);
        for (uint32_t i = 0; i < I; ++i) {
            uint64_t e = (uint64_t)b * I + i;
            all[e].x = x[i];
            all[e].a16 = (uint16_t)(s16 & 0x7fffu);
            code_of[e] = is_out[i] ? 255 : (uint8_t)nearest_level(x[i], xi);
        }
    }
    /* pass 2: per region, collect, sort by x and walk the cumulated weights */
    for (uint64_t e = 0; e < n; ++e) {
        if (code_of[e] == 255) {
            out->n_outliers++;
            continue;
        }
        out->cnt[code_of[e]]++;
        out->n_used++;
        out->sae += (weight_by_max ? (double)f16_to_f32(all[e].a16) : 1.0) * fabs((double)all[e].x - cb[code_of[e]]);
    }
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int l = 0; l < NLEVELS; ++l) {
        out->median[l] = NAN;
        uint64_t K = out->cnt[l];
        if (K == 0) continue;
        mae_sample* reg = (mae_sample*)malloc((size_t)K * sizeof(mae_sample));
        if (!reg) {
            failed = 1;
            continue;
        }
        uint64_t k = 0;
        for (uint64_t e = 0; e < n; ++e)
            if (code_of[e] == (uint8_t)l) reg[k++] = all[e];
        qsort(reg, (size_t)K, sizeof(mae_sample), cmp_mae_sample);
        unsigned __int128 total = 0, run = 0;
        /* appendix D (weight_by_max == 0): one unit per weight - the plain median; a block whose constant is not a
           binary16 number carries no weight either way */
        for (uint64_t j = 0; j < K; ++j) total += sample_weight(reg[j].a16, weight_by_max);
        out->den[l] = weight_by_max ? ldexp((double)total, -24) : (double)total;
        if (total != 0) {
            /* equal x are adjacent: the test is made where a value ends, on everything up to and including it */
            for (uint64_t j = 0; j < K; ++j) {
                run += sample_weight(reg[j].a16, weight_by_max);
                if (j + 1 < K && reg[j + 1].x == reg[j].x) continue;
                if (2 * run >= total) {
                    out->median[l] = (double)reg[j].x;
                    break;
                }
            }
        }
        free(reg);
    }
    free(all);
    free(code_of);
    return failed ? ORACLE_ERR_ARG : ORACLE_OK;
}

/* Maximisation step under the MAE criterion: an unpinned level whose region carries weight moves to the region's
 * weighted median (section 3.2 eq. 8). */
int oracle_codebook_update_mae(const oracle_mae_stats* st, uint16_t pinned_mask, double* cb) {
    if (!st || !cb) return ORACLE_ERR_ARG;
    for (int l = 0; l < NLEVELS; ++l) {
        if ((pinned_mask >> l) & 1u) continue;
        if (st->median[l] == st->median[l]) cb[l] = st->median[l];
    }
    return ORACLE_OK;
}

/* Thread count the Lloyd pass will use (for the reported CPU baseline). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
