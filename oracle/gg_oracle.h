/*
 * gg_oracle.h -- reference ("oracle") implementation of the generalized-Gaussian
 * (GG) constrained tensor pass, for TESTING ONLY.
 *
 * This is test infrastructure: a plain, slow, single-threaded, sequential CPU
 * implementation in C99 with double accumulators.  Only the test-suite, the
 * smoke check and the cpu_baseline leg of the benchmark may call it.  It shares
 * no source, header, table or helper with the HIP library; the structs below
 * are the oracle's own and deliberately differ from the library's.
 *
 * Notation (the paper writes scale = beta and shape = nu in Eq. 1-2; here, as in
 * the rest of this repository, alpha = scale and beta = shape):
 *
 *   f(x; alpha, beta) = beta / (2 alpha Gamma(1/beta)) * exp(-(|x|/alpha)^beta)   [Eq. 1, mu = 0]
 *   alpha = sigma * sqrt(Gamma(1/beta) / Gamma(3/beta))                          [Eq. 2]
 *   E[x^2] = alpha^2 Gamma(3/beta) / Gamma(1/beta)                               [Eq. 3]
 *
 * Pinned parts (see tests/test_oracle_*.py): rho(), solve, fit, Map, EG length,
 * histogram/entropy/bit count, penalty gradient, Philox4x32-10, sampler,
 * init scale.  Nothing in this file is "parity unpinned".
 */
#ifndef GG_ORACLE_H
#define GG_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element types of an input buffer */
#define ORC_F32 0
#define ORC_BF16 1

/* rounding of x/Delta to an integer: the paper's STE forward is floor (Sec. 4.2) */
#define ORC_ROUND_FLOOR 0
#define ORC_ROUND_NEAREST_EVEN 1

/* condition bits */
#define ORC_EMPTY 1u          /* n == 0 */
#define ORC_DEGENERATE 2u     /* sum x^2 == 0: no spread, beta := 2, alpha := 0 */
#define ORC_BETA_CLAMPED_LO 4u
#define ORC_BETA_CLAMPED_HI 8u
#define ORC_NONFINITE 16u     /* a NaN/Inf reached the sums (fit) or a NaN product (quantize) */
#define ORC_SATURATED 32u     /* some |x/Delta| exceeded 2^30 and was clamped */

#define ORC_BETA_MIN 0.05
#define ORC_BETA_MAX 20.0

typedef struct {
    double sum_abs;   /* S1 = sum |x_i|            */
    double sum_sq;    /* S2 = sum x_i^2            */
    uint64_t n;       /* element count (zeros included) */
    double beta;      /* shape, double precision   */
    double alpha;     /* scale, double precision   */
    uint32_t flags;
} orc_fit_t;

typedef struct {
    uint64_t eg_bits;    /* sum of Exp-Golomb-k code lengths            */
    uint64_t n;          /* element count                               */
    uint64_t n_clamped;  /* symbols that fell in the overflow bin but are larger than it */
    double entropy_bits; /* empirical entropy of the (clamped) histogram, bits/symbol */
    uint32_t u_max;      /* largest mapped symbol                       */
    uint32_t fl_bits;    /* fixed-length bits = max(1, bit_length(u_max)) */
    uint32_t flags;
} orc_rate_t;

/* ---- GG statistics (Eq. 1-3) ------------------------------------------- */
double orc_rho(double beta);                               /* (E|x|)^2 / E[x^2] of a GGD with shape beta */
double orc_solve_beta(double rho, uint32_t *flags);        /* inverse of orc_rho on [0.05, 20] by bisection */
double orc_alpha_from_m2(double m2, double beta);          /* Eq. 2 with sigma^2 = m2 */
double orc_init_alpha(int64_t d_in, double shape, double xi); /* Eq. 5 scale of GG initialisation */
void orc_moments(const void *x, int dtype, int64_t n, double *sum_abs, double *sum_sq);
void orc_fit_from_moments(double sum_abs, double sum_sq, uint64_t n, orc_fit_t *out);
void orc_fit(const void *x, int dtype, int64_t n, orc_fit_t *out);

/* ---- quantiser, Map, Exp-Golomb rate (Sec. 4.2) ------------------------ */
int32_t orc_quantize_one(float x, float inv_delta, int round_mode, uint32_t *flags);
uint32_t orc_map(int32_t q);
uint32_t orc_eg_len(uint32_t u, int k);
/* hist may be NULL (nbins ignored); symbols may be NULL. hist is overwritten. */
void orc_quantize_rate(const void *x, int dtype, int64_t n, float delta, int eg_k, int round_mode,
                       int32_t nbins, uint64_t *hist, int32_t *symbols, orc_rate_t *out);

/* ---- GG-prior rate penalty gradient ------------------------------------ */
void orc_penalty_grad(const void *w, int dtype, int64_t n, float alpha, float beta, float lambda,
                      float *grad, int accumulate);

/* ---- counter-based RNG and GG sampler ---------------------------------- */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
/* element i uses counter {attempt, stream, lo(offset+i), hi(offset+i)}, key {lo(seed), hi(seed)} */
/* fp32 -> bf16 bits, round to nearest even, NaN kept quiet (what orc_sample stores for ORC_BF16) */
void orc_round_bf16(const float *x, int64_t n, uint16_t *out);
void orc_sample(void *out, int dtype, int64_t n, float alpha, float beta,
                uint64_t seed, uint32_t stream, uint64_t offset);
/* total attempts of the rejection step over the same n draws */
uint64_t orc_sample_attempts(int64_t n, float beta, uint64_t seed, uint32_t stream, uint64_t offset);

/* ---- whole pass over a segmented flat buffer --------------------------- */
/* offsets[S+1] element offsets; per segment: fit, Delta = (float)alpha / delta_div (or delta[s]
 * when delta_div <= 0), rate with no histogram; optional penalty (grad NULL = none). */
void orc_fused_segmented(const void *x, int dtype, const int64_t *offsets, int32_t S,
                         float delta_div, const float *delta, int eg_k, int round_mode,
                         float lambda, float *grad, int accumulate,
                         orc_fit_t *fits, orc_rate_t *rates);

/* ---- GCT element-wise update (Algorithm 2, with the rate gradient of Sec. 4.3) ---- */
void orc_gct_update(float *w, const float *g, float *g_hat_prev, int64_t n,
                    float eta, float lambda, float eps, float inv_delta, int eg_k,
                    int64_t n_rate, int first_step);

/* ---- gradient of the mean EG-k length w.r.t. the quantised tensor (ACT backward, Sec. 4.2/4.3) ----
 * grad[i] (+)= scale * 4 inv_delta / (n_rate ln 2) * sign(x_i) / (u_i + 2^k) */
void orc_rate_grad(const void *x, int dtype, int64_t n, float inv_delta, int eg_k, int64_t n_rate,
                   float scale, float *grad, int accumulate);

/* ---- Exp-Golomb bit stream (encoder / decoder) -------------------------- */
/* returns number of bits written; out must hold (bits+7)/8 bytes, zero-initialised by callee */
uint64_t orc_eg_encode(const uint32_t *u, int64_t n, int eg_k, uint8_t *out, uint64_t out_bytes);
int64_t orc_eg_decode(const uint8_t *in, uint64_t n_bits, int eg_k, uint32_t *u, int64_t max_n);
/* out[i] (=|+=) q[i] * delta in fp32: the reconstruction level of the quantiser of Sec. 4.2 */
void orc_dequantize(const int32_t *q, int64_t n, float delta, float *out, int accumulate);

/* ---- compression ratio against fixed-length coding (Sec. 5.1): 1 - mean_bits / fl_bits ---- */
double orc_compression_ratio(double mean_bits, double fl_bits);

/* ---- Huffman mean code length from a histogram -------------------------- */
double orc_huffman_mean_bits(const uint64_t *hist, int32_t nbins);

#ifdef __cplusplus
}
#endif
#endif
