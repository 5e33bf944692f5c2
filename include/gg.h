/*
 * gg.h -- C ABI of libgg: the generalized-Gaussian (GG) constrained tensor pass for
 * AMD MI355X (gfx950).
 *
 * The pass underlies the paper's GG initialisation (Sec. 4.1), activation-constrained
 * training (ACT, Sec. 4.2, Algorithm 1) and gradient-constrained training (GCT, Sec. 4.3,
 * Algorithm 2).  Over a tensor, each row of a matrix, or each segment of a flat bucket it
 *   1. fits a zero-mean generalized Gaussian  f(x) = beta/(2 alpha Gamma(1/beta)) exp(-(|x|/alpha)^beta)
 *      (Eq. 1; the paper calls the scale beta and the shape nu -- here alpha = scale, beta = shape)
 *      from sum|x|, sum x^2 and the count, by inverting the moment ratio
 *      rho(beta) = Gamma(2/beta)^2 / (Gamma(1/beta) Gamma(3/beta)) and applying Eq. 2 for alpha;
 *   2. quantises uniformly with step Delta (forward value of the straight-through estimator of
 *      Sec. 4.2: floor), maps signed symbols to unsigned (Map, Sec. 4.2), and evaluates the
 *      order-k Exp-Golomb bit count (rate R, Sec. 4.2), the symbol histogram, its empirical
 *      entropy, and the fixed-length bits the experiments compare against (Sec. 5.1);
 *   3. evaluates the GG-prior rate penalty gradient
 *      lambda * beta * |w/alpha|^(beta-1) * sign(w) / alpha   (= lambda d/dw of the exponent of Eq. 1);
 *   4. draws GG variates |x| = alpha G^(1/beta), G ~ Gamma(1/beta, 1), from Philox4x32-10 (GG init, Eq. 5).
 *
 * Conventions
 *   - Every pointer named *_dev is DEVICE memory; *_host is HOST memory.  The caller owns all
 *     buffers, including the workspace and the result structs.  The library allocates no device
 *     memory (and no host memory outside the host helper gg_huffman_mean_bits),
 *     keeps no state between calls and never synchronises: all work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream); outputs are valid once the
 *     stream reaches that point.  Calls sharing a workspace must be ordered on one stream.
 *   - x_dev, grad_dev and symbols_dev must be 16-byte aligned; result structs 8-byte aligned.
 *   - Every function returns GG_OK or a negative error code.  Invalid arguments are detected on
 *     the host before anything is launched.  Data-dependent conditions (empty, degenerate,
 *     clamped, non-finite input) are reported per unit in the `flags` fields, never as errors.
 *   - dtype: GG_F32 (IEEE binary32) or GG_BF16 (bfloat16, widened exactly to fp32).  Any finite values, denormals
 *     included: where the fp32 square of a value would leave the fp32 range, the moment sums form it in fp64.
 */
#ifndef GG_H
#define GG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GG_OK 0
#define GG_ERR_INVALID_ARG (-1)   /* null pointer, negative size, misaligned buffer, bad parameter value */
#define GG_ERR_BAD_DTYPE (-2)
#define GG_ERR_BAD_SEGMENTS (-3)  /* offsets not non-decreasing, negative, or too many units */
#define GG_ERR_WORKSPACE (-4)     /* workspace missing or smaller than gg_workspace_bytes() says */
#define GG_ERR_HIP (-5)           /* a HIP runtime call failed (launch error) */

#define GG_F32 0
#define GG_BF16 1

#define GG_FLOOR 0          /* the paper's quantiser: q = floor(x / Delta) */
#define GG_NEAREST_EVEN 1   /* q = rint(x / Delta), ties to even */

/* per-unit condition bits */
#define GG_F_EMPTY 1u            /* the unit has no elements */
#define GG_F_DEGENERATE 2u       /* fit: sum x^2 == 0 (beta := 2, alpha := 0); rate: no usable step, rate not evaluated */
#define GG_F_BETA_CLAMPED_LO 4u  /* moment ratio below rho(GG_BETA_MIN) */
#define GG_F_BETA_CLAMPED_HI 8u  /* moment ratio above rho(GG_BETA_MAX) */
#define GG_F_NONFINITE 16u       /* fit: a sum is NaN/Inf (beta := 2, alpha := 0); rate: some x/Delta was NaN (symbol 0) */
#define GG_F_SATURATED 32u       /* rate: some |x/Delta| was clamped to 2^30 */

#define GG_BETA_MIN 0.05
#define GG_BETA_MAX 20.0
#define GG_MAX_BINS 65536
#define GG_MAX_EG_K 15

/* Result of a fit (step 1).  40 bytes. */
typedef struct {
    double sum_abs;   /* S1 = sum |x_i| (fp64 sum of fp32 per-thread partials)      */
    double sum_sq;    /* S2 = sum x_i^2                                             */
    uint64_t n;       /* number of elements, zeros included                         */
    float beta;       /* shape                                                      */
    float alpha;      /* scale, Eq. 2 with sigma^2 = S2/n                           */
    uint32_t flags;
    uint32_t _pad;
} gg_fit_t;

/* Result of a rate evaluation (step 2).  48 bytes. */
typedef struct {
    uint64_t eg_bits;     /* sum over elements of 2 floor(log2(u + 2^k)) - k + 1               */
    uint64_t n;
    uint64_t n_clamped;   /* elements with u > nbins-1 (counted in the last bin); 0 without a histogram */
    double entropy_bits;  /* -sum p log2 p over the histogram bins, bits/element; 0 without a histogram */
    uint32_t u_max;       /* largest mapped symbol (never clamped)                              */
    uint32_t fl_bits;     /* fixed-length bits: max(1, bit_length(u_max))                       */
    float delta;          /* the step that was used                                            */
    uint32_t flags;
} gg_rate_t;

const char *gg_strerror(int code);

/* Bytes of device workspace any call below needs for a buffer of n_total elements split into
 * n_units units (segments or rows; 1 for a single tensor).  nbins is accepted for forward
 * compatibility and does not currently change the size. */
int gg_workspace_bytes(int64_t n_total, int32_t n_units, int32_t nbins, size_t *bytes_out_host);

/* ---- step 1: fit --------------------------------------------------------------------------- */
/* One tensor of n elements -> out_dev[0]. */
int gg_fit(const void *x_dev, int dtype, int64_t n, gg_fit_t *out_dev,
           void *ws_dev, size_t ws_bytes, void *stream);
/* Flat bucket: unit s is x[offsets_host[s] .. offsets_host[s+1]) (element offsets, S+1 entries,
 * non-decreasing, offsets_host[0] >= 0; zero-length units are legal; S <= 2^17: the table travels to the
 * device as kernel arguments, 448 offsets per launch, read from offsets_host before the call returns).  -> out_dev[S]. */
int gg_fit_segmented(const void *x_dev, int dtype, const int64_t *offsets_host, int32_t S,
                     gg_fit_t *out_dev, void *ws_dev, size_t ws_bytes, void *stream);
/* Row-major rows x cols matrix: one fit per row -> out_dev[rows]; if total_out_dev is not NULL it
 * also receives the fit of the whole matrix (fixed-order sum of the row sums), from the same sweep. */
int gg_fit_rows(const void *x_dev, int dtype, int64_t rows, int64_t cols, gg_fit_t *out_dev,
                gg_fit_t *total_out_dev, void *ws_dev, size_t ws_bytes, void *stream);

/* ---- step 2: quantise + rate ---------------------------------------------------------------- */
/* t = x * (1/delta) in fp32 (one multiply; NaN -> 0; clamped to +-2^30); q = floor(t) or rint(t);
 * u = Map(q) = (q > 0 ? 2q-1 : -2q).  delta > 0 and finite.  eg_k in 0..15.
 * nbins = 0: no histogram (hist_dev ignored).  Otherwise 2..65536 and hist_dev[nbins] (uint64) is
 * overwritten with counts of min(u, nbins-1).  symbols_dev (int32[n]) receives q unless NULL. */
int gg_quantize_rate(const void *x_dev, int dtype, int64_t n, float delta, int eg_k, int round_mode,
                     int32_t nbins, uint64_t *hist_dev, int32_t *symbols_dev, gg_rate_t *out_dev,
                     void *ws_dev, size_t ws_bytes, void *stream);
/* Per-segment steps delta_dev[S] (device).  hist_dev is S*nbins (unit s at hist_dev + s*nbins) or
 * NULL with nbins = 0.  A unit whose step is not a positive finite number is flagged
 * GG_F_DEGENERATE and its rate is not evaluated (symbols of that unit are written as 0). */
int gg_quantize_rate_segmented(const void *x_dev, int dtype, const int64_t *offsets_host, int32_t S,
                               const float *delta_dev, int eg_k, int round_mode,
                               int32_t nbins, uint64_t *hist_dev, int32_t *symbols_dev,
                               gg_rate_t *out_dev, void *ws_dev, size_t ws_bytes, void *stream);
/* One step per row of a rows x cols matrix, no histogram. */
int gg_quantize_rate_rows(const void *x_dev, int dtype, int64_t rows, int64_t cols,
                          const float *delta_dev, int eg_k, int round_mode, int32_t *symbols_dev,
                          gg_rate_t *out_dev, void *ws_dev, size_t ws_bytes, void *stream);
/* delta_out_dev[s] = fit_dev[s].alpha / delta_div (one fp32 division), for chaining calls on device. */
int gg_delta_from_fit(const gg_fit_t *fit_dev, int32_t S, float delta_div, float *delta_out_dev,
                      void *stream);

/* ---- step 3: penalty gradient --------------------------------------------------------------- */
/* grad[i] (=|+=) lambda*beta*|w_i/alpha|^(beta-1)*sign(w_i)/alpha, sign(0) = 0.  alpha > 0,
 * beta > 0, finite.  accumulate: 0 writes, 1 adds to the existing fp32 value. */
int gg_penalty_grad(const void *w_dev, int dtype, int64_t n, float alpha, float beta, float lambda,
                    float *grad_dev, int accumulate, void *stream);
/* alpha, beta of unit s from fit_dev[s].  Units with alpha == 0 contribute 0. */
int gg_penalty_grad_segmented(const void *w_dev, int dtype, const int64_t *offsets_host, int32_t S,
                              const gg_fit_t *fit_dev, float lambda, float *grad_dev, int accumulate,
                              void *ws_dev, size_t ws_bytes, void *stream);

/* ---- step 4: sampler (GG initialisation, Sec. 4.1) ------------------------------------------ */
/* out[i] = +-alpha * G^(1/beta), G ~ Gamma(1/beta, 1) by Marsaglia-Tsang rejection (boosted for
 * shape < 1), fed by Philox4x32-10 with key = {lo(seed), hi(seed)} and counter
 * {attempt, stream_id, lo(offset+i), hi(offset+i)}: the value of element i depends on
 * (seed, stream_id, offset+i) only, never on the launch shape.  alpha >= 0, 0.05 <= beta <= 20. */
int gg_sample(void *out_dev, int dtype, int64_t n, float alpha, float beta,
              uint64_t seed, uint32_t stream_id, uint64_t offset, void *stream);
/* Raw generator output: out_dev[4*i .. 4*i+3] = Philox4x32-10 block for counter
 * {attempt, stream_id, lo(offset+i), hi(offset+i)}. */
int gg_philox_words(uint32_t *out_dev, int64_t n, uint64_t seed, uint32_t stream_id, uint64_t offset,
                    uint32_t attempt, void *stream);
/* Host helper, Eq. 5: scale of GG(0, alpha, shape) weights of a linear layer with fan-in d_in and
 * activation correction xi (1: none/sigmoid, 2: ReLU, 2/(1+k^2): leaky ReLU); shape 2 gives He init. */
double gg_init_alpha(int64_t d_in, double shape, double xi);
/* Host helper, Sec. 5.1: compression ratio against fixed-length coding, 1 - mean_bits / fl_bits. */
double gg_compression_ratio(double mean_bits, double fl_bits);

/* ---- the whole pass over a flat bucket in one call ------------------------------------------ */
/* Per unit s: fit -> fit_dev[s]; step Delta_s = fit alpha_s / delta_div (delta_div > 0) or
 * delta_dev[s] (delta_div <= 0); rate -> rate_dev[s] (skipped entirely when rate_dev is NULL);
 * optional histogram (hist_dev, S*nbins) and symbols; optional penalty gradient with the fitted
 * (alpha_s, beta_s) into grad_dev (NULL = none).  Everything stays on the device.
 * When the steps are given (delta_div <= 0, delta_dev != NULL) and no penalty is asked for, nothing
 * depends on this call's own fit and x is read ONCE: moments and rate come from the same sweep
 * (e.g. GCT monitoring with the steps of the previous training step). */
int gg_fused_segmented(const void *x_dev, int dtype, const int64_t *offsets_host, int32_t S,
                       float delta_div, const float *delta_dev, int eg_k, int round_mode,
                       int32_t nbins, uint64_t *hist_dev, int32_t *symbols_dev,
                       float lambda, float *grad_dev, int accumulate,
                       gg_fit_t *fit_dev, gg_rate_t *rate_dev,
                       void *ws_dev, size_t ws_bytes, void *stream);
/* The same with one unit per row of a rows x cols matrix (no histogram); total_fit_dev as in gg_fit_rows. */
int gg_fused_rows(const void *x_dev, int dtype, int64_t rows, int64_t cols,
                  float delta_div, const float *delta_dev, int eg_k, int round_mode,
                  int32_t *symbols_dev, float lambda, float *grad_dev, int accumulate,
                  gg_fit_t *fit_dev, gg_fit_t *total_fit_dev, gg_rate_t *rate_dev,
                  void *ws_dev, size_t ws_bytes, void *stream);

/* gg_fused_segmented for callers that cannot allocate and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and error codes, minus
 * the workspace: the scratch memory (fit partials, per-run rate slots, the unit table) is a device array of
 * GG_NOALLOC_SCRATCH_BYTES inside the library, one copy per GPU, held until the process ends.  The call makes no
 * hipMalloc / hipFree and no host allocation.  A bucket whose gg_workspace_bytes(offsets_host[S], S, 0) exceeds
 * GG_NOALLOC_SCRATCH_BYTES is refused with GG_ERR_WORKSPACE before anything is launched (16 MiB serve any bucket
 * of up to 2^31 elements in up to 4096 units; the 1.5 G-element, 253-unit gradient bucket needs 7.2 MiB).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams, or
 * different host threads) race on it and give wrong results; order them on one stream.  Nothing in the array
 * has to be cleared between calls: every slot a kernel reads has been written earlier in the same call. */
#define GG_NOALLOC_SCRATCH_BYTES (16u << 20)
int gg_fused_segmented_noalloc(const void *x_dev, int dtype, const int64_t *offsets_host, int32_t S,
                               float delta_div, const float *delta_dev, int eg_k, int round_mode,
                               int32_t nbins, uint64_t *hist_dev, int32_t *symbols_dev,
                               float lambda, float *grad_dev, int accumulate,
                               gg_fit_t *fit_dev, gg_rate_t *rate_dev, void *stream);

/* ---- companions of the pass inside the training algorithms ----------------------------------- */
/* ACT backward (Sec. 4.2) / dR/dG of Sec. 4.3: gradient of the mean order-k Exp-Golomb length
 * R = (1/n_rate) sum_i [2 log2(u_i + 2^k) - k + 1] through the straight-through quantiser,
 *   grad[i] (=|+=) scale * 4 (1/delta) / (n_rate ln 2) * sign(x_i) / (u_i + 2^k),  u_i = Map(floor(x_i / delta)).
 * For delta = 2^-n, k = 0 this is the paper's 2^(n+2)/(N ln 2) Sign/Map(Quant) with the 2^k of the code
 * length kept (finite at u = 0).  n_rate is the N of the mean (normally n).  grad_dev fp32, 16-byte aligned. */
int gg_rate_grad(const void *x_dev, int dtype, int64_t n, float delta, int eg_k, int64_t n_rate, float scale,
                 float *grad_dev, int accumulate, void *stream);

/* GCT element-wise update, Algorithm 2 (steps "approximate second-order derivatives", "equivalent
 * gradient", "weight update"), fp32, in place on w_dev and ghat_prev_dev:
 *   h = first_step ? 0 : (1/eta) (1 - g/(ghat_prev + eps));  ghat = g + lambda * dR/dg * h  (dR/dg as in
 *   gg_rate_grad with scale 1);  ghat_prev <- ghat;  w <- w - eta * ghat.
 * The per-epoch decay lambda <- alpha_decay * lambda is the caller's scalar.  eta > 0. */
int gg_gct_update(float *w_dev, const float *g_dev, float *ghat_prev_dev, int64_t n, float eta, float lambda,
                  float eps, float delta, int eg_k, int64_t n_rate, int first_step, void *stream);
/* The same over a flat bucket with one step per unit (delta_dev[S], e.g. from gg_delta_from_fit) and
 * n_rate = the unit's length.  A unit without a positive finite step gets no rate term (plain SGD). */
int gg_gct_update_segmented(float *w_dev, const float *g_dev, float *ghat_prev_dev, const int64_t *offsets_host,
                            int32_t S, const float *delta_dev, float eta, float lambda, float eps, int eg_k,
                            int first_step, void *ws_dev, size_t ws_bytes, void *stream);

/* Order-k Exp-Golomb bit stream of quantised symbols q (as written by the rate sweep): symbol i is
 * (L-1-k) zero bits followed by the L bits of Map(q_i) + 2^k, most significant bit first, bytes filled from
 * their most significant bit.  The stream's length in bits equals gg_rate_t.eg_bits of the same symbols.
 * symbols_dev: n int32, 16-byte aligned.  stream_dev: room for stream_bytes (a multiple of 4, 4-byte
 * aligned); the 32-bit words up to the one holding the last bit are written (that one zero-padded), bytes
 * beyond it are left as they were.  If the stream does not fit, tiles that would overflow are left out
 * (compare *total_bits_dev with 8*stream_bytes).
 * block_offsets_dev: gg_eg_workspace_bytes(n) bytes, 8-byte aligned; on return its first T + 1 entries,
 * T = ceil(n / GG_EG_TILE), are the index for parallel decoding: entry b is the bit offset of symbol
 * GG_EG_TILE*b, entry T the total (the rest of the buffer is scratch).  total_bits_dev may be NULL.
 * gg_eg_decode takes those T + 1 entries; it reads only words that hold bits of the indexed tiles, whatever
 * the stream contains; symbols_dev (out) 16-byte aligned. */
#define GG_EG_TILE 256
int gg_eg_workspace_bytes(int64_t n, size_t *bytes_out_host);
int gg_eg_encode(const int32_t *symbols_dev, int64_t n, int eg_k, uint8_t *stream_dev, uint64_t stream_bytes,
                 uint64_t *block_offsets_dev, uint64_t *total_bits_dev, void *stream);
int gg_eg_decode(const uint8_t *stream_dev, const uint64_t *block_offsets_dev, int64_t n, int eg_k,
                 int32_t *symbols_dev, void *stream);
/* Decoding straight to values: out[i] (=|+=) q_i * delta in fp32, q_i the decoded symbol -- the lower end of the
 * quantiser's cell (Sec. 4.2: q = floor(x / delta), so q delta <= x < (q + 1) delta), one fp32 product, and with
 * accumulate != 0 one fp32 add onto the existing value (summing the coded tensors of several senders).  No symbol
 * array in memory.  delta > 0 and finite; out_dev fp32, 16-byte aligned; the rest as for gg_eg_decode. */
int gg_eg_decode_dequant(const uint8_t *stream_dev, const uint64_t *block_offsets_dev, int64_t n, int eg_k, float delta,
                         float *out_dev, int accumulate, void *stream);
/* The same for the stream of a flat bucket (gg_eg_encode_segmented): element i of unit s becomes q_i * delta_dev[s];
 * a unit without a positive finite step was coded as zeros and decodes to zeros.  n is offsets_host[S]; offsets
 * and ws_dev as in gg_fit_segmented (the workspace receives the unit table), except that offsets_host[0] must be 0
 * (GG_ERR_BAD_SEGMENTS otherwise): the stream holds every element of the buffer, so the units must cover it. */
int gg_eg_decode_dequant_segmented(const uint8_t *stream_dev, const uint64_t *block_offsets_dev, const int64_t *offsets_host,
                                   int32_t S, int eg_k, const float *delta_dev, float *out_dev, int accumulate, void *ws_dev,
                                   size_t ws_bytes, void *stream);
/* The same stream straight from a tensor: symbol i is the quantised x_i (the rate sweep's arithmetic: one
 * fp32 product with 1/delta, NaN -> 0, clamp to +-2^30, GG_FLOOR or GG_NEAREST_EVEN), so the stream is bit for
 * bit what gg_quantize_rate's symbols would give and its length the eg_bits of that call, with no symbol
 * array in memory.  x_dev 16-byte aligned, delta > 0 and finite; buffers as for gg_eg_encode. */
int gg_eg_encode_tensor(const void *x_dev, int dtype, int64_t n, float delta, int round_mode, int eg_k,
                        uint8_t *stream_dev, uint64_t stream_bytes, uint64_t *block_offsets_dev,
                        uint64_t *total_bits_dev, void *stream);
/* The same for a flat bucket with one step per unit (delta_dev[S], e.g. from gg_delta_from_fit; offsets as in
 * gg_fit_segmented): one stream for the whole bucket, equal to the stream of gg_quantize_rate_segmented's
 * symbols; a unit without a positive finite step contributes symbol 0 for every element.  ws_dev as for the
 * segmented calls (it receives the unit table).  offsets_host[0] must be 0 (GG_ERR_BAD_SEGMENTS otherwise): the
 * stream codes the elements 0 .. offsets_host[S) of x_dev, each with the step of the unit that holds it. */
int gg_eg_encode_segmented(const void *x_dev, int dtype, const int64_t *offsets_host, int32_t S,
                           const float *delta_dev, int round_mode, int eg_k, uint8_t *stream_dev,
                           uint64_t stream_bytes, uint64_t *block_offsets_dev, uint64_t *total_bits_dev,
                           void *ws_dev, size_t ws_bytes, void *stream);

/* Host helper: mean Huffman code length in bits/symbol of a histogram (the HM column of the paper's
 * tables, Sec. 5.1); 0 for an empty histogram, 1 when a single symbol occurs. */
int gg_huffman_mean_bits(const uint64_t *hist_host, int32_t nbins, double *mean_bits_out_host);

#ifdef __cplusplus
}
#endif
#endif /* GG_H */
