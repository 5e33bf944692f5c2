/*
 * gg_oracle.c -- plain CPU reference of the generalized-Gaussian (GG) tensor pass.
 *
 * TEST INFRASTRUCTURE ONLY (see gg_oracle.h).  Single thread, sequential index
 * order, double accumulators, libm only.  Written to be checked against the
 * paper by eye: every function names the passage it follows and performs the
 * steps in that order, with no blocking, fusion or reordering.
 *
 * Build: gcc -O2 -std=c99 -fPIC -shared (no -ffast-math; denormals are kept).
 */
#include "gg_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* element access: bf16 -> fp32 is exact (the 16 bits are the high half)      */
/* ------------------------------------------------------------------------- */
static float load_elem(const void *x, int dtype, int64_t i)
{
    if (dtype == ORC_BF16) {
        uint32_t bits = (uint32_t)((const uint16_t *)x)[i] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return f;
    }
    return ((const float *)x)[i];
}

/* round-to-nearest-even fp32 -> bf16 (NaN kept quiet) */
static uint16_t to_bf16(float f)
{
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    if ((bits & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((bits >> 16) | 0x0040u);
    uint32_t lsb = (bits >> 16) & 1u;
    bits += 0x7fffu + lsb;
    return (uint16_t)(bits >> 16);
}

/* the rounding the sampler applies to its bf16 outputs, on an array (for the tests) */
void orc_round_bf16(const float *x, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = to_bf16(x[i]);
}

/* ------------------------------------------------------------------------- */
/* GG statistics                                                              */
/* ------------------------------------------------------------------------- */

/* Moment ratio of a zero-mean GGD with shape b.  From Eq. 1:
 *   E|x|  = alpha Gamma(2/b)/Gamma(1/b),   E[x^2] = alpha^2 Gamma(3/b)/Gamma(1/b)  (Eq. 3)
 * so rho(b) = (E|x|)^2 / E[x^2] = Gamma(2/b)^2 / (Gamma(1/b) Gamma(3/b)), free of alpha. */
static double log_rho(double b)
{
    return 2.0 * lgamma(2.0 / b) - lgamma(1.0 / b) - lgamma(3.0 / b);
}

double orc_rho(double beta)
{
    return exp(log_rho(beta));
}

/* Invert rho on [ORC_BETA_MIN, ORC_BETA_MAX].  rho is strictly increasing in b
 * (0 as b -> 0, 3/4 as b -> inf), so plain bisection on log rho converges. */
double orc_solve_beta(double rho, uint32_t *flags)
{
    double target = log(rho);
    double lo = ORC_BETA_MIN, hi = ORC_BETA_MAX;
    if (!(target > log_rho(lo))) {
        if (flags) *flags |= ORC_BETA_CLAMPED_LO;
        return lo;
    }
    if (!(target < log_rho(hi))) {
        if (flags) *flags |= ORC_BETA_CLAMPED_HI;
        return hi;
    }
    for (int it = 0; it < 200; ++it) {
        double mid = 0.5 * (lo + hi);
        if (log_rho(mid) < target)
            lo = mid;
        else
            hi = mid;
        if (hi - lo < 1e-12 * lo)
            break;
    }
    return 0.5 * (lo + hi);
}

/* Eq. 2 with sigma^2 replaced by the second sample moment m2. */
double orc_alpha_from_m2(double m2, double beta)
{
    return sqrt(m2 * exp(lgamma(1.0 / beta) - lgamma(3.0 / beta)));
}

/* Eq. 5: scale of the GG initialisation of a linear layer with fan-in d_in,
 * activation correction xi: sqrt(xi/d_in * Gamma(1/nu)/Gamma(3/nu)). */
double orc_init_alpha(int64_t d_in, double shape, double xi)
{
    return sqrt(xi / (double)d_in * exp(lgamma(1.0 / shape) - lgamma(3.0 / shape)));
}

void orc_moments(const void *x, int dtype, int64_t n, double *sum_abs, double *sum_sq)
{
    double s1 = 0.0, s2 = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        float v = load_elem(x, dtype, i);
        s1 += (double)fabsf(v);
        s2 += (double)v * (double)v;
    }
    *sum_abs = s1;
    *sum_sq = s2;
}

void orc_fit_from_moments(double sum_abs, double sum_sq, uint64_t n, orc_fit_t *out)
{
    out->sum_abs = sum_abs;
    out->sum_sq = sum_sq;
    out->n = n;
    out->beta = 0.0;
    out->alpha = 0.0;
    out->flags = 0;
    if (n == 0) {
        out->flags = ORC_EMPTY;
        return;
    }
    if (!isfinite(sum_abs) || !isfinite(sum_sq)) {
        out->flags = ORC_NONFINITE;
        out->beta = 2.0;
        return;
    }
    if (sum_sq == 0.0) {
        out->flags = ORC_DEGENERATE;
        out->beta = 2.0;
        return;
    }
    double m1 = sum_abs / (double)n;
    double m2 = sum_sq / (double)n;
    double rho = m1 * m1 / m2;
    out->beta = orc_solve_beta(rho, &out->flags);
    out->alpha = orc_alpha_from_m2(m2, out->beta);
}

void orc_fit(const void *x, int dtype, int64_t n, orc_fit_t *out)
{
    double s1, s2;
    orc_moments(x, dtype, n, &s1, &s2);
    orc_fit_from_moments(s1, s2, (uint64_t)n, out);
}

/* ------------------------------------------------------------------------- */
/* quantiser, Map, Exp-Golomb length (Sec. 4.2)                               */
/* ------------------------------------------------------------------------- */

/* Quant(x) = STE(x / Delta): the forward value of the straight-through
 * estimator x - sg(x - floor(x)) is floor(x).  The paper's step 2^-n is
 * generalised to any positive fp32 Delta via one fp32 multiply by 1/Delta.
 * NaN products give symbol 0; the product is clamped to +-2^30 before the
 * integer conversion. */
int32_t orc_quantize_one(float x, float inv_delta, int round_mode, uint32_t *flags)
{
    volatile float prod = x * inv_delta; /* volatile: one fp32 rounding, never fused or widened */
    float t = prod;
    if (t != t) {
        if (flags) *flags |= ORC_NONFINITE;
        return 0;
    }
    const float lim = 1073741824.0f; /* 2^30 */
    if (t > lim) t = lim;
    if (t < -lim) t = -lim;
    float r = (round_mode == ORC_ROUND_NEAREST_EVEN) ? rintf(t) : floorf(t);
    return (int32_t)r;
}

/* Map of Sec. 4.2: negative -> -2q (even), zero -> 0, positive -> 2q-1 (odd). */
uint32_t orc_map(int32_t q)
{
    if (q < 0) return (uint32_t)(-2 * (int64_t)q);
    if (q == 0) return 0u;
    return (uint32_t)(2 * (int64_t)q - 1);
}

/* k-th order Exp-Golomb code length of u: write v = u + 2^k in binary
 * (L = floor(log2 v) + 1 bits) preceded by L - 1 - k zeros:  2 floor(log2 v) - k + 1. */
uint32_t orc_eg_len(uint32_t u, int k)
{
    uint64_t v = (uint64_t)u + ((uint64_t)1 << k);
    uint32_t fl = 0;
    while (v > 1) {
        v >>= 1;
        ++fl;
    }
    return 2u * fl - (uint32_t)k + 1u;
}

static uint32_t bit_length(uint32_t v)
{
    uint32_t b = 0;
    while (v) {
        v >>= 1;
        ++b;
    }
    return b;
}

void orc_quantize_rate(const void *x, int dtype, int64_t n, float delta, int eg_k, int round_mode,
                       int32_t nbins, uint64_t *hist, int32_t *symbols, orc_rate_t *out)
{
    volatile float inv_v = 1.0f / delta; /* one IEEE fp32 divide */
    float inv_delta = inv_v;
    uint64_t bits = 0, clamped = 0;
    uint32_t umax = 0, flags = 0;

    if (hist)
        for (int32_t b = 0; b < nbins; ++b) hist[b] = 0;

    for (int64_t i = 0; i < n; ++i) {
        float v = load_elem(x, dtype, i);
        int32_t q = orc_quantize_one(v, inv_delta, round_mode, &flags);
        uint32_t u = orc_map(q);
        if (symbols) symbols[i] = q;
        bits += orc_eg_len(u, eg_k);
        if (u > umax) umax = u;
        if (hist) {
            if (u > (uint32_t)(nbins - 1)) {
                ++clamped;
                hist[nbins - 1] += 1;
            } else {
                hist[u] += 1;
            }
        }
    }
    if (umax >= 2147483647u) flags |= ORC_SATURATED; /* |q| reached 2^30 */
    if (n == 0) flags |= ORC_EMPTY;

    double H = 0.0;
    if (hist && n > 0) {
        for (int32_t b = 0; b < nbins; ++b) {
            if (hist[b]) {
                double p = (double)hist[b] / (double)n;
                H -= p * log2(p);
            }
        }
    }
    out->eg_bits = bits;
    out->n = (uint64_t)n;
    out->n_clamped = clamped;
    out->entropy_bits = H;
    out->u_max = umax;
    out->fl_bits = bit_length(umax) > 1u ? bit_length(umax) : 1u;
    out->flags = flags;
}

/* ------------------------------------------------------------------------- */
/* GG-prior rate penalty: lambda * d/dw (|w|/alpha)^beta                       */
/*   = lambda * beta * |w/alpha|^(beta-1) * sign(w) / alpha,  sign(0) = 0      */
/* (minus lambda times the derivative of the log of Eq. 1)                     */
/* ------------------------------------------------------------------------- */
void orc_penalty_grad(const void *w, int dtype, int64_t n, float alpha, float beta, float lambda,
                      float *grad, int accumulate)
{
    double a = (double)alpha, b = (double)beta, lam = (double)lambda;
    for (int64_t i = 0; i < n; ++i) {
        double v = (double)load_elem(w, dtype, i);
        double p;
        if (v == 0.0 || v != v) {
            p = 0.0;
        } else {
            double s = v > 0.0 ? 1.0 : -1.0;
            p = lam * b * pow(fabs(v) / a, b - 1.0) * s / a;
        }
        float p32 = (float)p;
        if (accumulate) {
            volatile float sum = grad[i] + p32; /* one fp32 add */
            grad[i] = sum;
        } else {
            grad[i] = p32;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as    */
/* easy as 1, 2, 3", SC'11): ten rounds of                                     */
/*   (c0,c1,c2,c3) <- (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0)) */
/* with the key bumped by the Weyl constants between rounds.                   */
/* ------------------------------------------------------------------------- */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = M0 * c0;
        uint64_t p1 = M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0;
        k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* 32 random bits -> uniform in (0,1): the top 23 bits plus one half, times 2^-23.
 * Exactly representable in fp32 and never 0 or 1. */
static double unit_open(uint32_t w)
{
    return ((double)(w >> 9) + 0.5) * (1.0 / 8388608.0);
}

#define ORC_MAX_ATTEMPTS 64

/* GG sample: |x| = alpha * G^(1/beta) with G ~ Gamma(1/beta, 1), random sign.
 * Gamma(a) by Marsaglia & Tsang (2000): d = a - 1/3, c = 1/sqrt(9 d), draw
 * z ~ N(0,1), v = (1 + c z)^3, accept d*v when v > 0 and
 * ln u < z^2/2 + d - d v + d ln v.  For a < 1 draw Gamma(a+1) and multiply by
 * U^(1/a).  Every attempt takes one fresh Philox block
 *   counter = {attempt, stream, lo(index), hi(index)}, key = {lo(seed), hi(seed)}:
 * words 0,1 -> Box-Muller normal, word 2 -> acceptance uniform; word 3 of
 * attempt 0 gives the sign (bit 0) and the boost uniform (top 23 bits). */

/* Shape a = 1/beta of the Gamma variate and the constants of its generator; returns whether the
 * draw is made at shape a + 1 and boosted down (a < 1). */
static int gamma_constants(float beta, double *a, double *d, double *c)
{
    *a = 1.0 / (double)beta;
    int boost = *a < 1.0;
    *d = (boost ? *a + 1.0 : *a) - 1.0 / 3.0;
    *c = 1.0 / sqrt(9.0 * *d);
    return boost;
}

/* The attempts of element `idx`: returns d*v of the accepted attempt (d if all ORC_MAX_ATTEMPTS are
 * rejected: probability < 1e-80), word 3 of attempt 0 in *w3_first, the attempts used in *used. */
static double gamma_by_attempts(double d, double c, uint64_t idx, uint32_t stream, const uint32_t key[2],
                                uint32_t *w3_first, uint32_t *used)
{
    const double two_pi = 6.283185307179586476925286766559;
    *w3_first = 0;
    for (uint32_t attempt = 0; attempt < ORC_MAX_ATTEMPTS; ++attempt) {
        uint32_t ctr[4] = {attempt, stream, (uint32_t)idx, (uint32_t)(idx >> 32)};
        uint32_t w[4];
        orc_philox4x32_10(ctr, key, w);
        if (attempt == 0) *w3_first = w[3];
        double z = sqrt(-2.0 * log(unit_open(w[0]))) * cos(two_pi * unit_open(w[1]));
        double t = 1.0 + c * z;
        double v = t * t * t;
        if (v <= 0.0) continue;
        double lu = log(unit_open(w[2]));
        if (lu < 0.5 * z * z + d - d * v + d * log(v)) {
            *used = attempt + 1;
            return d * v;
        }
    }
    *used = ORC_MAX_ATTEMPTS;
    return d;
}

void orc_sample(void *out, int dtype, int64_t n, float alpha, float beta,
                uint64_t seed, uint32_t stream, uint64_t offset)
{
    double a, d, c;
    int boost = gamma_constants(beta, &a, &d, &c);
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};

    for (int64_t i = 0; i < n; ++i) {
        uint32_t w3_first, used;
        double gam = gamma_by_attempts(d, c, offset + (uint64_t)i, stream, key, &w3_first, &used);
        /* G^(1/beta) = G^a; with the boost G = G' U^(1/a) so G^a = G'^a U */
        double mag = pow(gam, a);
        if (boost) mag *= unit_open(w3_first);
        double xval = (double)alpha * mag;
        if (w3_first & 1u) xval = -xval;
        float xf = (float)xval;
        if (dtype == ORC_BF16)
            ((uint16_t *)out)[i] = to_bf16(xf);
        else
            ((float *)out)[i] = xf;
    }
}

/* Attempts the same n draws take in total (the efficiency of the rejection step; no sample is formed). */
uint64_t orc_sample_attempts(int64_t n, float beta, uint64_t seed, uint32_t stream, uint64_t offset)
{
    double a, d, c;
    (void)gamma_constants(beta, &a, &d, &c);
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint64_t total = 0;
    for (int64_t i = 0; i < n; ++i) {
        uint32_t w3_first, used;
        (void)gamma_by_attempts(d, c, offset + (uint64_t)i, stream, key, &w3_first, &used);
        total += used;
    }
    return total;
}

/* ------------------------------------------------------------------------- */
/* whole pass over a segmented flat buffer                                    */
/* ------------------------------------------------------------------------- */
void orc_fused_segmented(const void *x, int dtype, const int64_t *offsets, int32_t S,
                         float delta_div, const float *delta, int eg_k, int round_mode,
                         float lambda, float *grad, int accumulate,
                         orc_fit_t *fits, orc_rate_t *rates)
{
    size_t esz = dtype == ORC_BF16 ? 2 : 4;
    for (int32_t s = 0; s < S; ++s) {
        int64_t lo = offsets[s], n = offsets[s + 1] - offsets[s];
        const void *xs = (const char *)x + (size_t)lo * esz;
        orc_fit(xs, dtype, n, &fits[s]);
        float a32 = (float)fits[s].alpha, b32 = (float)fits[s].beta;
        volatile float dl = delta_div > 0.0f ? a32 / delta_div : delta[s];
        memset(&rates[s], 0, sizeof rates[s]);
        rates[s].n = (uint64_t)n;
        if (n == 0) {
            rates[s].flags = ORC_EMPTY;
            rates[s].fl_bits = 1;
            continue;
        }
        if (dl > 0.0f && isfinite((double)dl))
            orc_quantize_rate(xs, dtype, n, dl, eg_k, round_mode, 0, NULL, NULL, &rates[s]);
        else
            rates[s].flags = ORC_DEGENERATE; /* no usable step: rate not evaluated */
        if (grad && a32 > 0.0f)
            orc_penalty_grad(xs, dtype, n, a32, b32, lambda, grad + lo, accumulate);
        else if (grad && !accumulate)
            for (int64_t i = 0; i < n; ++i) grad[lo + i] = 0.0f;
    }
}

/* ------------------------------------------------------------------------- */
/* GCT element-wise update (Algorithm 2).  Per parameter i at step t:         */
/*   h_i   = (1/eta) (1 - g_i / (ghat_prev_i + eps)) * 1[t >= 2]               */
/*   dR_i  = 4 inv_delta / (N ln 2) * sign(g_i) / (u_i + 2^k),                 */
/*           u_i = Map(floor(g_i * inv_delta))                                */
/*   ghat_i = g_i + lambda * dR_i * h_i   (stored for the next step)           */
/*   w_i  <- w_i - eta * ghat_i                                               */
/* dR is the derivative of the mean EG-k length (1/N) sum 2 log2(u + 2^k) with */
/* u ~ 2 |g| inv_delta; for inv_delta = 2^n it is the paper's 2^(n+2)/(N ln 2) */
/* sign(g)/Map(Quant(g)) with the 2^k the printed formula drops restored.      */
/* ------------------------------------------------------------------------- */
void orc_gct_update(float *w, const float *g, float *g_hat_prev, int64_t n,
                    float eta, float lambda, float eps, float inv_delta, int eg_k,
                    int64_t n_rate, int first_step)
{
    const double ln2 = 0.69314718055994530942;
    double coef = 4.0 * (double)inv_delta / ((double)n_rate * ln2);
    for (int64_t i = 0; i < n; ++i) {
        double gi = (double)g[i];
        double h = 0.0;
        if (!first_step)
            h = (1.0 / (double)eta) * (1.0 - gi / ((double)g_hat_prev[i] + (double)eps));
        uint32_t fl = 0;
        int32_t q = orc_quantize_one(g[i], inv_delta, ORC_ROUND_FLOOR, &fl);
        uint32_t u = orc_map(q);
        double s = gi > 0.0 ? 1.0 : (gi < 0.0 ? -1.0 : 0.0);
        double dR = coef * s / ((double)u + (double)((uint64_t)1 << eg_k));
        double ghat = gi + (double)lambda * dR * h;
        float ghat32 = (float)ghat;
        g_hat_prev[i] = ghat32;
        w[i] = (float)((double)w[i] - (double)eta * (double)ghat32);
    }
}

/* ------------------------------------------------------------------------- */
/* Gradient of the rate R = (1/N) sum_i [2 log2(u_i + 2^k) - k + 1] through    */
/* the straight-through quantiser (Sec. 4.2): d u/d x ~ 2 inv_delta sign(x),   */
/* so dR/dx_i = 4 inv_delta / (N ln 2) * sign(x_i) / (u_i + 2^k)  -- the       */
/* expression Sec. 4.3 prints as 2^(n+2)/(n ln 2) Sign(G)/Map(Quant(G)), with  */
/* the 2^k of the code length kept so that u = 0 is finite.                    */
/* ------------------------------------------------------------------------- */
void orc_rate_grad(const void *x, int dtype, int64_t n, float inv_delta, int eg_k, int64_t n_rate,
                   float scale, float *grad, int accumulate)
{
    const double ln2 = 0.69314718055994530942;
    double coef = (double)scale * 4.0 * (double)inv_delta / ((double)n_rate * ln2);
    for (int64_t i = 0; i < n; ++i) {
        float v = load_elem(x, dtype, i);
        uint32_t fl = 0;
        uint32_t u = orc_map(orc_quantize_one(v, inv_delta, ORC_ROUND_FLOOR, &fl));
        double s = v > 0.0f ? 1.0 : (v < 0.0f ? -1.0 : 0.0);
        float d = (float)(coef * s / ((double)u + (double)((uint64_t)1 << eg_k)));
        if (accumulate) {
            volatile float sum = grad[i] + d;
            grad[i] = sum;
        } else {
            grad[i] = d;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Exp-Golomb-k bit stream, MSB first: (L-1-k) zeros then the L bits of u+2^k */
/* ------------------------------------------------------------------------- */
uint64_t orc_eg_encode(const uint32_t *u, int64_t n, int eg_k, uint8_t *out, uint64_t out_bytes)
{
    uint64_t pos = 0;
    memset(out, 0, (size_t)out_bytes);
    for (int64_t i = 0; i < n; ++i) {
        uint64_t v = (uint64_t)u[i] + ((uint64_t)1 << eg_k);
        int L = 0;
        for (uint64_t t = v; t; t >>= 1) ++L;
        pos += (uint64_t)(L - 1 - eg_k); /* zero prefix */
        for (int b = L - 1; b >= 0; --b) {
            if ((pos >> 3) < out_bytes && ((v >> b) & 1u))
                out[pos >> 3] |= (uint8_t)(0x80u >> (pos & 7u));
            ++pos;
        }
    }
    return pos;
}

int64_t orc_eg_decode(const uint8_t *in, uint64_t n_bits, int eg_k, uint32_t *u, int64_t max_n)
{
    uint64_t pos = 0;
    int64_t cnt = 0;
    while (pos < n_bits && cnt < max_n) {
        int zeros = 0;
        while (pos < n_bits && !((in[pos >> 3] >> (7 - (pos & 7u))) & 1u)) {
            ++zeros;
            ++pos;
        }
        int L = zeros + eg_k + 1;
        if (pos + (uint64_t)L > n_bits) return -1;
        uint64_t v = 0;
        for (int b = 0; b < L; ++b) {
            v = (v << 1) | ((in[pos >> 3] >> (7 - (pos & 7u))) & 1u);
            ++pos;
        }
        u[cnt++] = (uint32_t)(v - ((uint64_t)1 << eg_k));
    }
    return cnt;
}

/* What a symbol of the uniform quantiser of Sec. 4.2 stands for: q * Delta, one fp32 product (the
 * quantiser's floor makes it the lower end of the cell: q Delta <= x < (q + 1) Delta).  With accumulate the
 * value is added to what is there (one fp32 add): the receiving side of a sum of coded tensors. */
void orc_dequantize(const int32_t *q, int64_t n, float delta, float *out, int accumulate)
{
    for (int64_t i = 0; i < n; ++i) {
        volatile float v = (float)q[i] * delta;
        if (accumulate) {
            volatile float sum = out[i] + v;
            out[i] = sum;
        } else {
            out[i] = v;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Huffman mean code length (the HM column of the paper's tables): repeatedly */
/* merge the two least frequent nodes; the sum of all merged weights is the   */
/* total coded length.  One distinct symbol is given a 1-bit code.            */
/* ------------------------------------------------------------------------- */
static int cmp_u64(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return x < y ? -1 : (x > y ? 1 : 0);
}

double orc_huffman_mean_bits(const uint64_t *hist, int32_t nbins)
{
    int32_t m = 0;
    uint64_t total = 0;
    for (int32_t b = 0; b < nbins; ++b)
        if (hist[b]) {
            ++m;
            total += hist[b];
        }
    if (m == 0) return 0.0;
    if (m == 1) return 1.0;
    uint64_t *leaf = (uint64_t *)malloc((size_t)m * sizeof *leaf);
    uint64_t *node = (uint64_t *)malloc((size_t)m * sizeof *node);
    int32_t j = 0;
    for (int32_t b = 0; b < nbins; ++b)
        if (hist[b]) leaf[j++] = hist[b];
    qsort(leaf, (size_t)m, sizeof *leaf, cmp_u64);
    int32_t li = 0, ni = 0, nn = 0;
    double coded = 0.0;
    for (int32_t step = 0; step < m - 1; ++step) {
        uint64_t pick[2];
        for (int t = 0; t < 2; ++t) {
            if (li < m && (ni >= nn || leaf[li] <= node[ni]))
                pick[t] = leaf[li++];
            else
                pick[t] = node[ni++];
        }
        node[nn++] = pick[0] + pick[1];
        coded += (double)(pick[0] + pick[1]);
    }
    free(leaf);
    free(node);
    return coded / (double)total;
}

/* Compression ratio of an entropy code against fixed-length coding, as tabulated in the
 * experiments: C = 1 - (mean code length) / (fixed-length bits). */
double orc_compression_ratio(double mean_bits, double fl_bits)
{
    return 1.0 - mean_bits / fl_bits;
}
