// gg_kernels.hip -- HIP kernels and the C ABI of libgg (see include/gg.h).
//
// Launch structure of one pass over a buffer cut into units (segments / rows / one tensor):
//   k_upload_i64      segment offsets and per-unit chunk prefix -> workspace (through kernel args)
//   k_fit_partials    the buffer is cut into chunks of <= kChunk elements of one unit; each block
//                     owns a run of consecutive chunks: sum|x|, sum x^2 in fp32 per lane and chunk,
//                     fp64 lane totals, combined across the block per (run, unit) piece -> partials
//   k_fit_finalize    one wave per unit: fixed-order fp64 sum of its partials, 64-way parallel
//                     bracketing of the moment-ratio equation, Eq. 2 for alpha; derives the
//                     unit's quantiser / penalty parameters and clears its rate record
//   k_quant           re-reads x: quantise, Map, Exp-Golomb bits, u_max, optional LDS-privatised
//                     histogram, symbols, penalty gradient; a unit inside one run gets its rate record
//                     from that block, a unit that several runs share one slot of sums per run
//   k_rate_reduce     folds the per-run rate sums of units that several runs share into their records
//   k_rate_finalize   the same, plus the histogram entropy in fp64 (when a histogram was asked for)
// All reductions are order-fixed (floating point) or integer, so results are reproducible.

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <atomic>
#include <cmath>
#include <type_traits>

#include "../../include/gg.h"
#include "gg_device.h"
#include "gg_geometry.h"

// 128-bit loads each lane keeps in flight in the two sweeps (tuned on MI355X)
#ifndef GG_U_FIT
#define GG_U_FIT 8
#endif
#ifndef GG_U_QUANT
#define GG_U_QUANT 4
#endif
#ifndef GG_ROW_BATCH
#define GG_ROW_BATCH 2            // rows of a matrix a wave fits with one solve (wave-per-row pass)
#endif
#ifndef GG_ROW_BATCH_BYTES
#define GG_ROW_BATCH_BYTES 16384  // and the bytes of rows it may hold in cache between its two sweeps
#endif

namespace gg {

constexpr int kMaxDevices = 64;   // devices of one process the per-device caches below have room for

// ---------------------------------------------------------------------------------------------
// sweep 1: moments
// ---------------------------------------------------------------------------------------------
struct FitBody {
    float s1[4] = {0.f, 0.f, 0.f, 0.f};
    float s2[4] = {0.f, 0.f, 0.f, 0.f};
    template <int W>
    __device__ __forceinline__ void vec(const float (&v)[W], int64_t) {
#pragma unroll
        for (int j = 0; j < W; ++j) {
            s1[j & 3] += fabsf(v[j]);
            s2[j & 3] = __builtin_fmaf(v[j], v[j], s2[j & 3]);
        }
    }
    __device__ __forceinline__ void one(float v, int64_t) {
        s1[0] += fabsf(v);
        s2[0] = __builtin_fmaf(v, v, s2[0]);
    }
};

// The fp32 squares of a lane's share leave the representable range when all of its values lie below about 1e-19
// (the squares vanish) or one above about 1e19 (its square is infinite).  The sums tell: a sum of squares below
// 2^-90 next to a positive sum of magnitudes (had even one square been in range, the sum would be there too, and
// the at most 64 vanished ones beside it would be 2^-54 of it), or an infinite sum.  Such a share -- in practice
// a whole tensor that lives at such a scale, or none -- is summed again with the squares formed in fp64.
struct FitBody64 {
    double s1 = 0.0, s2 = 0.0;
    template <int W>
    __device__ __forceinline__ void vec(const float (&v)[W], int64_t) {
#pragma unroll
        for (int j = 0; j < W; ++j) { const double d = (double)v[j]; s1 += fabs(d); s2 = fma(d, d, s2); }
    }
    __device__ __forceinline__ void one(float v, int64_t) { const double d = (double)v; s1 += fabs(d); s2 = fma(d, d, s2); }
};

__device__ __forceinline__ bool fit_sums_left_range(const float (&s1)[4], const float (&s2)[4]) {
    const float a = (s1[0] + s1[1]) + (s1[2] + s1[3]), b = (s2[0] + s2[1]) + (s2[2] + s2[3]);
    return (a > 0.f && b < 0x1p-90f) || a == __builtin_inff() || b == __builtin_inff();
}

// the lane's sums of one walk as doubles (d1, d2 are added to); E, GROUP and the range as in the walk that filled `fb`
template <typename E, int GROUP>
__device__ __forceinline__ void add_lane_moments(const float (&s1)[4], const float (&s2)[4], const typename E::type *__restrict__ x,
                                                 int64_t start, int len, double &d1, double &d2) {
    if (fit_sums_left_range(s1, s2)) {             // per lane: the walk has no barrier in it
        FitBody64 wide;
        process_chunk<E, 1, FitBody64, GROUP>(x, start, len, wide);
        d1 += wide.s1; d2 += wide.s2;
    } else {
        d1 += ((double)s1[0] + (double)s1[1]) + ((double)s1[2] + (double)s1[3]);
        d2 += ((double)s2[0] + (double)s2[1]) + ((double)s2[2] + (double)s2[3]);
    }
}

// A block owns a run of consecutive chunks.  Lanes keep fp32 sums per chunk (<= 16 terms each) and
// fold them into fp64 lane totals; lanes are combined only when the run leaves a unit or ends.
// The combined value of a (run, unit) piece goes to the slot of the piece's first chunk, which is
// max(first chunk of the unit, first chunk of the run): k_fit_finalize visits exactly those slots.
template <typename T>
__global__ __launch_bounds__(kBlock) void k_fit_partials(SegView sv, const T *__restrict__ x,
                                                         double2 *__restrict__ partials, int64_t n_chunks,
                                                         int32_t chunks_per_block) {
    __shared__ double red[2][kWaves];
    const int tid = threadIdx.x;
    const int64_t first = (int64_t)blockIdx.x * chunks_per_block;
    int64_t last = first + chunks_per_block;
    if (last > n_chunks) last = n_chunks;
    if (first >= last) return;

    double d1 = 0.0, d2 = 0.0;
    auto flush = [&](int64_t slot) {
        const double a = wave_reduce(d1, OpAdd());
        const double b = wave_reduce(d2, OpAdd());
        if ((tid & 63) == 0) { red[0][tid >> 6] = a; red[1][tid >> 6] = b; }
        __syncthreads();
        if (tid == 0) {
            double2 r;
            r.x = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
            r.y = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
            partials[slot] = r;
        }
        __syncthreads();
        d1 = 0.0; d2 = 0.0;
    };

    RunCursor cur;
    cur.init(sv, first, last);
    int piece_seg = cur.L.seg;
    int64_t piece_first = first;
    for (; cur.valid(); cur.next(sv)) {
        if (cur.L.seg != piece_seg) {
            flush(piece_first);
            piece_first = cur.chunk; piece_seg = cur.L.seg;
        }
        FitBody body;
        process_chunk<Elem<T>, GG_U_FIT>(x, cur.L.start, cur.L.len, body);
        add_lane_moments<Elem<T>, kBlock>(body.s1, body.s2, x, cur.L.start, cur.L.len, d1, d2);
    }
    flush(piece_first);
}

// cubic Lagrange through (xs[k], ys[k]), k = 0..3, evaluated at x, over the common denominator: one division.
// The node differences here are 1e-5 .. 1 (table values a grid step apart), so the products stay far inside
// the fp64 range.
__device__ __forceinline__ double lagrange4(const double (&xs)[4], const double (&ys)[4], double x) {
    double num[4], den[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        num[k] = ys[k]; den[k] = 1.0;
#pragma unroll
        for (int m = 0; m < 4; ++m)
            if (m != k) { num[k] *= x - xs[m]; den[k] *= xs[k] - xs[m]; }
    }
    const double d01 = den[0] * den[1], d23 = den[2] * den[3];
    const double top = (num[0] * den[1] + num[1] * den[0]) * d23 + (num[2] * den[3] + num[3] * den[2]) * d01;
    return top / (d01 * d23);
}

// the same for equally spaced nodes x0, x0 + h, x0 + 2h, x0 + 3h: the denominators are -6, 2, -2, 6 times h^3
__device__ __forceinline__ double lagrange4_uniform(double x0, double h, const double (&ys)[4], double x) {
    const double t = (x - x0) / h;                     // node k sits at t = k
    const double t0 = t, t1 = t - 1.0, t2 = t - 2.0, t3 = t - 3.0;
    return ys[0] * (t1 * t2 * t3) * (-1.0 / 6.0) + ys[1] * (t0 * t2 * t3) * 0.5 + ys[2] * (t0 * t1 * t3) * (-0.5) +
           ys[3] * (t0 * t1 * t2) * (1.0 / 6.0);
}

// The moment ratio of a GGD is rho(b) = Gamma(2/b)^2 / (Gamma(1/b) Gamma(3/b)) (from Eq. 1, 3).  Its curve is
// tabulated at build time (gen_solve_curve.py) on a uniform grid in l = ln b,
//   kSolveCurve[j] = { ln rho(b_j), lgamma(1/b_j) - lgamma(3/b_j) },  b_j = exp(l_min + j h),  j = 0..kSolveTable,
// and a unit's root is found by locating its interval (two 64-way probes by a wave, or a binary search by a
// lane) and inverse cubic interpolation through the four surrounding points: error 7e-12 relative in b,
// 2e-10 in the log of the scale factor of Eq. 2.  No launch, no workspace and no run-time state: the curve
// is part of the code object.
struct alignas(16) CurvePoint { double x, y; };
__device__ const CurvePoint kSolveCurve[kSolveTable + 1] = {
#include "gg_solve_curve.inc"
};

// beta and alpha from four consecutive table points j0 .. j0+3 around the root
__device__ __forceinline__ void finish_from_points(int j0, const double (&fs)[4], const double (&as)[4], double target, double m2,
                                                   gg_fit_t &f) {
    const double l_min = log(GG_BETA_MIN), h = (log(GG_BETA_MAX) - l_min) / (double)kSolveTable;
    double ls[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) ls[k] = l_min + h * (double)(j0 + k);
    const double l = lagrange4(fs, ls, target);          // inverse interpolation: l as a function of log rho
    f.beta = (float)exp(l);
    f.alpha = (float)sqrt(m2 * exp(lagrange4_uniform(ls[0], h, as, l)));   // Eq. 2 with sigma^2 = m2
}

// first of the four points used for the interval j (table[j].x <= target < table[j+1].x)
__device__ __forceinline__ int first_point(int j) {
    const int j0 = j - 1;
    return j0 < 0 ? 0 : (j0 > kSolveTable - 3 ? kSolveTable - 3 : j0);
}

__device__ __forceinline__ void finish_from_table(int j, double target, double m2, gg_fit_t &f) {
    const int j0 = first_point(j);
    double fs[4], as[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const CurvePoint t = kSolveCurve[j0 + k];
        fs[k] = t.x; as[k] = t.y;
    }
    finish_from_points(j0, fs, as, target, m2, f);
}

// common head of the table solvers; returns true when the root has to be searched
__device__ __forceinline__ bool fit_head(double s1, double s2, uint64_t n, gg_fit_t &f, double &target, double &m2) {
    f.sum_abs = s1; f.sum_sq = s2; f.n = n; f.beta = 0.f; f.alpha = 0.f; f.flags = 0; f._pad = 0;
    if (n == 0) { f.flags = GG_F_EMPTY; return false; }
    if (!isfinite(s1) || !isfinite(s2)) { f.flags = GG_F_NONFINITE; f.beta = 2.f; return false; }
    if (s2 == 0.0) { f.flags = GG_F_DEGENERATE; f.beta = 2.f; return false; }
    const double m1 = s1 / (double)n;
    m2 = s2 / (double)n;
    target = log(m1 * m1 / m2);
    // outside the curve the shape is clamped to the end of the supported range; Eq. 2 then takes that end's factor
    int end;
    if (!(target > kSolveCurve[0].x)) { end = 0; f.beta = (float)GG_BETA_MIN; f.flags = GG_F_BETA_CLAMPED_LO; }
    else if (!(target < kSolveCurve[kSolveTable].x)) { end = kSolveTable; f.beta = (float)GG_BETA_MAX; f.flags = GG_F_BETA_CLAMPED_HI; }
    else return true;
    f.alpha = (float)sqrt(m2 * exp(kSolveCurve[end].y));
    return false;
}

// one lane per unit: binary search of the interval
__device__ __forceinline__ void solve_fit_lane(double s1, double s2, uint64_t n, gg_fit_t &f) {
    const CurvePoint *__restrict__ table = kSolveCurve;
    double target, m2;
    if (!fit_head(s1, s2, n, f, target, m2)) return;
    int lo = 0, hi = kSolveTable;            // table[lo].x <= target < table[hi].x
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (table[mid].x <= target) lo = mid; else hi = mid;
    }
    finish_from_table(lo, target, m2, f);
}

// one wave per unit (all 64 lanes, identical arguments): two rounds of 64 probes locate the interval
__device__ __forceinline__ void solve_fit_wave(double s1, double s2, uint64_t n, gg_fit_t &f) {
    static_assert(kSolveTable == 64 * 64, "two 64-way rounds cover the table");
    const CurvePoint *__restrict__ table = kSolveCurve;
    const int lane = threadIdx.x & 63;
    double target, m2;
    if (!fit_head(s1, s2, n, f, target, m2)) return;
    int c1 = __popcll(__ballot(table[64 * lane].x <= target));
    c1 = c1 < 1 ? 1 : c1;
    const int coarse = 64 * (c1 - 1);
    const CurvePoint t2 = table[coarse + lane];
    int c2 = __popcll(__ballot(t2.x <= target));
    c2 = c2 < 1 ? 1 : c2;
    const int j0 = first_point(coarse + c2 - 1);
    if (j0 >= coarse && j0 + 3 <= coarse + 63) {          // the four points are in this round's lanes
        double fs[4], as[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) { fs[k] = __shfl(t2.x, j0 - coarse + k, 64); as[k] = __shfl(t2.y, j0 - coarse + k, 64); }
        finish_from_points(j0, fs, as, target, m2, f);
    } else {
        finish_from_table(coarse + c2 - 1, target, m2, f);
    }
}

// A batch of up to kRowBatch units per wave, lane r holding the sums of unit r (r < nr).  Only the search of
// the interval needs the whole wave (two table probes per unit, the first probe shared by the batch);
// the fp64 work in front of it (logarithm of the moment ratio) and behind it (interpolation, Eq. 2) is done
// once, lane r working for unit r.  Must be called by all 64 lanes.
constexpr int kRowBatch = GG_ROW_BATCH;
__device__ __forceinline__ void solve_fit_batch(double s1, double s2, uint64_t n, int nr, gg_fit_t &f) {
    static_assert(kSolveTable == 64 * 64, "two 64-way rounds cover the table");
    const CurvePoint *__restrict__ table = kSolveCurve;
    const int lane = threadIdx.x & 63;
    double target = 0.0, m2 = 0.0;
    bool search = false;
    if (lane < nr) search = fit_head(s1, s2, n, f, target, m2);
    const double probe = table[64 * lane].x;
    double tr[kRowBatch];
    int coarse[kRowBatch];
    double fine[kRowBatch];
#pragma unroll
    for (int r = 0; r < kRowBatch; ++r) {      // any target, even a NaN of an idle lane, stays inside the table
        tr[r] = __shfl(target, r, 64);
        int c1 = __popcll(__ballot(probe <= tr[r]));
        c1 = c1 < 1 ? 1 : c1;
        coarse[r] = 64 * (c1 - 1);
        fine[r] = table[coarse[r] + lane].x;
    }
    int j = 0;
#pragma unroll
    for (int r = 0; r < kRowBatch; ++r) {
        int c2 = __popcll(__ballot(fine[r] <= tr[r]));
        c2 = c2 < 1 ? 1 : c2;
        if (lane == r) j = coarse[r] + c2 - 1;
    }
    if (search) finish_from_table(j, target, m2, f);
}

// ---------------------------------------------------------------------------------------------
// The same root with the transcendental functions in fp32, for the wave-per-row kernel, where a fit costs as much
// as reading the row: about 150 instructions instead of about 300 double-precision ones (half rate).  Every lane
// of the wave takes the same arguments.  What keeps the result at 3e-7 relative (the fp64 solvers: 2e-7 after
// rounding to fp32; the bar is 1e-4):
//   * ln v of a double v = m 2^e as e ln 2 + ln m, the first term and the sum in fp64, ln m by v_log_f32 with
//     |ln m| < 0.7: 6e-8 absolute;
//   * the interpolation on differences to the table (x_k - target, a_k - a_1 formed in fp64, then fp32): the
//     quantities interpolated are a grid step wide, so fp32 rounding is 1e-7 of 1.5e-3;
//   * alpha = 2^k 2^r with k + r = log2(e) * (ln m2 + a) / 2 split in fp64, 2^r by v_exp_f32 with |r| <= 1/2.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ double ln_by_parts(double v) {      // v > 0, finite
    const int e = __builtin_amdgcn_frexp_exp(v);
    const float m = (float)__builtin_amdgcn_frexp_mant(v);       // [0.5, 1)
    return (double)e * 0.69314718055994530942 + (double)(0.69314718056f * __builtin_amdgcn_logf(m));
}

__device__ __forceinline__ float exp_by_parts(double ln_v) {    // e^ln_v as a float
    const double y = ln_v * 1.44269504088896340736;
    const double k = __builtin_rint(y);
    const float r = (float)(y - k);                              // |r| <= 1/2, exact difference
    return ldexpf(__builtin_amdgcn_exp2f(r), (int)k);
}

__device__ __forceinline__ void solve_fit_wave_f32(double s1, double s2, uint64_t n, gg_fit_t &f) {
    static_assert(kSolveTable == 64 * 64, "two 64-way rounds cover the table");
    const CurvePoint *__restrict__ table = kSolveCurve;
    const int lane = threadIdx.x & 63;
    f.sum_abs = s1; f.sum_sq = s2; f.n = n; f.beta = 0.f; f.alpha = 0.f; f.flags = 0; f._pad = 0;
    if (n == 0) { f.flags = GG_F_EMPTY; return; }
    if (!isfinite(s1) || !isfinite(s2)) { f.flags = GG_F_NONFINITE; f.beta = 2.f; return; }
    if (s2 == 0.0) { f.flags = GG_F_DEGENERATE; f.beta = 2.f; return; }
    const double ln_n = ln_by_parts((double)n);
    const double ln_m2 = ln_by_parts(s2) - ln_n;
    const double target = 2.0 * (ln_by_parts(s1) - ln_n) - ln_m2;                  // ln of the moment ratio (s1 > 0 since s2 > 0)
    if (!(target > table[0].x)) { f.beta = (float)GG_BETA_MIN; f.flags = GG_F_BETA_CLAMPED_LO; f.alpha = exp_by_parts(0.5 * (ln_m2 + table[0].y)); return; }
    if (!(target < table[kSolveTable].x)) { f.beta = (float)GG_BETA_MAX; f.flags = GG_F_BETA_CLAMPED_HI; f.alpha = exp_by_parts(0.5 * (ln_m2 + table[kSolveTable].y)); return; }
    int c1 = __popcll(__ballot(table[64 * lane].x <= target));
    c1 = c1 < 1 ? 1 : c1;
    const int coarse = 64 * (c1 - 1);
    const CurvePoint t2 = table[coarse + lane];
    int c2 = __popcll(__ballot(t2.x <= target));
    c2 = c2 < 1 ? 1 : c2;
    const int j0 = first_point(coarse + c2 - 1);
    double fs[4], as[4];
    if (j0 >= coarse && j0 + 3 <= coarse + 63) {          // the four points are in this round's lanes
#pragma unroll
        for (int k = 0; k < 4; ++k) { fs[k] = __shfl(t2.x, j0 - coarse + k, 64); as[k] = __shfl(t2.y, j0 - coarse + k, 64); }
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) { const CurvePoint t = table[j0 + k]; fs[k] = t.x; as[k] = t.y; }
    }
    // inverse interpolation in node units: tau = sum_k k w_k, w_k = prod_{m != k} d_m / (d_m - d_k), d_k = x_k - target
    float d[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) d[k] = (float)(fs[k] - target);
    float tau = 0.f;
#pragma unroll
    for (int k = 1; k < 4; ++k) {
        float num = (float)k, den = 1.f;
#pragma unroll
        for (int m = 0; m < 4; ++m)
            if (m != k) { num *= d[m]; den *= d[m] - d[k]; }
        tau += num / den;
    }
    const double l_min = log(GG_BETA_MIN), h = (log(GG_BETA_MAX) - l_min) / (double)kSolveTable;   // constants
    const float l = (float)(l_min + h * (double)j0) + (float)h * tau;
    f.beta = __builtin_amdgcn_exp2f(l * 1.44269504089f);
    // the scale factor of Eq. 2 at tau: cubic through a_k - a_1 on the nodes 0, 1, 2, 3
    const float e0 = (float)(as[0] - as[1]), e2 = (float)(as[2] - as[1]), e3 = (float)(as[3] - as[1]);
    const float t0 = tau, t1 = tau - 1.f, t2f = tau - 2.f, t3 = tau - 3.f;
    const float da = e0 * (t1 * t2f * t3) * (-1.f / 6.f) + e2 * (t0 * t1 * t3) * (-0.5f) + e3 * (t0 * t1 * t2f) * (1.f / 6.f);
    f.alpha = exp_by_parts(0.5 * (ln_m2 + as[1] + (double)da));                     // Eq. 2 with sigma^2 = m2
}

// where the step and the penalty parameters of a unit come from
struct PrepArgs {
    const gg_fit_t *fit;       // device fits (penalty parameters, and alpha for delta_div > 0) or nullptr
    const float *delta_dev;    // device per-unit steps or nullptr
    float delta_div;           // > 0: Delta = alpha / delta_div
    float delta_scalar;        // used when delta_div <= 0 and delta_dev == nullptr
    float lambda;
    SegParam *params;          // device out
    gg_rate_t *rate;           // device out (cleared) or nullptr
    int want_pen;
    uint64_t *hist;            // histograms to clear for the sweep that follows (S * nbins counts), or nullptr
    int32_t nbins;
};

__device__ __forceinline__ void prepare_unit(const PrepArgs &a, int seg, int64_t n, float alpha, float beta) {
    SegParam p;
    p.flags = 0; p.ticket = 0; p._pad = 0;
    float delta;
    if (a.delta_div > 0.f) delta = (float)((double)alpha / (double)a.delta_div);  // == one fp32 division
    else delta = a.delta_dev ? a.delta_dev[seg] : a.delta_scalar;
    const bool ok = delta > 0.f && isfinite(delta);
    p.delta = delta;
    p.inv_delta = ok ? (float)(1.0 / (double)delta) : 0.f;                        // == 1.0f / delta
    if (!ok) p.flags |= kSkipRate;
    if (a.want_pen && alpha > 0.f && isfinite(alpha) && isfinite(beta)) {
        p.inv_alpha = (float)(1.0 / (double)alpha);
        p.pen_coef = (float)((double)a.lambda * (double)beta / (double)alpha);
        p.beta_m1 = beta - 1.0f;
    } else {
        p.inv_alpha = 0.f; p.pen_coef = 0.f; p.beta_m1 = 0.f;
        p.flags |= kPenZero;
    }
    a.params[seg] = p;
    if (a.rate) {
        gg_rate_t r;
        r.eg_bits = 0; r.n = (uint64_t)n; r.n_clamped = 0; r.entropy_bits = 0.0;
        r.u_max = 0; r.delta = delta;
        r.flags = n == 0 ? GG_F_EMPTY : (ok ? 0u : GG_F_DEGENERATE);
        r.fl_bits = (r.flags & GG_F_DEGENERATE) ? 0u : 1u;   // max(1, bit_length(u_max)); the sweep raises it
        a.rate[seg] = r;
    }
}

constexpr int kFitFinalizeThreads = 256;
__global__ __launch_bounds__(kFitFinalizeThreads) void k_fit_finalize(SegView sv, const double2 *__restrict__ partials,
                                                                      int32_t chunks_per_block, gg_fit_t *__restrict__ out,
                                                                      PrepArgs prep, int do_prep) {
    __shared__ double red[2][kFitFinalizeThreads / 64];
    const int seg = blockIdx.x, tid = threadIdx.x;
    const int64_t c0 = unit_chunk0(sv, seg), c1 = unit_chunk1(sv, seg);
    double s1 = 0.0, s2 = 0.0;
    if (c1 > c0) {
        // one piece per run that overlaps the unit; thread-strided over runs, ascending: a fixed order
        const int64_t r0 = c0 / chunks_per_block, r1 = (c1 - 1) / chunks_per_block;
#pragma unroll 8
        for (int64_t r = r0 + tid; r <= r1; r += kFitFinalizeThreads) {    // loads of several rounds in flight; the order of the sums stays
            const int64_t run_first = r * chunks_per_block;
            const double2 p = partials[run_first > c0 ? run_first : c0];
            s1 += p.x; s2 += p.y;
        }
    }
    s1 = wave_reduce(s1, OpAdd());
    s2 = wave_reduce(s2, OpAdd());
    if ((tid & 63) == 0) { red[0][tid >> 6] = s1; red[1][tid >> 6] = s2; }
    const int64_t n = unit_len(sv, seg);
    if (do_prep && prep.hist) {          // the unit's histogram starts at zero; the stores overlap the solve
        uint64_t *bins = prep.hist + (int64_t)seg * prep.nbins;
        for (int b = tid; b < prep.nbins; b += kFitFinalizeThreads) bins[b] = 0;
    }
    __syncthreads();
    if (tid >= 64) return;               // the first wave solves (all its lanes, identical arguments)
    s1 = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
    s2 = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    gg_fit_t f;
    solve_fit_wave(s1, s2, (uint64_t)n, f);
    if (tid == 0) {
        out[seg] = f;
        if (do_prep) prepare_unit(prep, seg, n, f.alpha, f.beta);
    }
}

// the same finalisation with one lane per unit (many small units)
__global__ __launch_bounds__(64) void k_fit_finalize_lanes(SegView sv, const double2 *__restrict__ partials,
                                                           int32_t chunks_per_block, gg_fit_t *__restrict__ out,
                                                           PrepArgs prep, int do_prep) {
    const int seg = blockIdx.x * 64 + threadIdx.x;
    if (seg >= sv.S) return;
    const int64_t c0 = unit_chunk0(sv, seg), c1 = unit_chunk1(sv, seg);
    double s1 = 0.0, s2 = 0.0;
    if (c1 > c0) {
        const int64_t r0 = c0 / chunks_per_block, r1 = (c1 - 1) / chunks_per_block;
        for (int64_t r = r0; r <= r1; ++r) {
            const int64_t run_first = r * chunks_per_block;
            const double2 p = partials[run_first > c0 ? run_first : c0];
            s1 += p.x; s2 += p.y;
        }
    }
    const int64_t n = unit_len(sv, seg);
    gg_fit_t f;
    solve_fit_lane(s1, s2, (uint64_t)n, f);
    out[seg] = f;
    if (do_prep) prepare_unit(prep, seg, n, f.alpha, f.beta);
}

// fit of the whole matrix from the per-row sums: thread-strided ascending sums, fixed tree across the
// block, solve by the first wave
constexpr int kTotalThreads = 1024;
__global__ __launch_bounds__(kTotalThreads) void k_fit_total(const gg_fit_t *__restrict__ rows, int64_t n_rows,
                                                             gg_fit_t *__restrict__ out) {
    __shared__ double red1[kTotalThreads / 64], red2[kTotalThreads / 64];
    __shared__ uint64_t redn[kTotalThreads / 64];
    const int tid = threadIdx.x;
    double s1 = 0.0, s2 = 0.0;
    uint64_t n = 0;
    for (int64_t r = tid; r < n_rows; r += kTotalThreads) { s1 += rows[r].sum_abs; s2 += rows[r].sum_sq; n += rows[r].n; }
    s1 = wave_reduce(s1, OpAdd());
    s2 = wave_reduce(s2, OpAdd());
    n = wave_reduce(n, OpAdd());
    if ((tid & 63) == 0) { red1[tid >> 6] = s1; red2[tid >> 6] = s2; redn[tid >> 6] = n; }
    __syncthreads();
    if (tid < 64) {
        s1 = 0.0; s2 = 0.0; n = 0;
        for (int w = 0; w < kTotalThreads / 64; ++w) { s1 += red1[w]; s2 += red2[w]; n += redn[w]; }
        gg_fit_t f;
        solve_fit_wave(s1, s2, n, f);
        if (tid == 0) out[0] = f;
    }
}

// the same from the sums the waves of k_rows leave (fewer and smaller than the row records)
__global__ __launch_bounds__(kTotalThreads) void k_fit_total_waves(const double2 *__restrict__ sums, int64_t n_waves, uint64_t n_elems,
                                                                   gg_fit_t *__restrict__ out) {
    __shared__ double red1[kTotalThreads / 64], red2[kTotalThreads / 64];
    const int tid = threadIdx.x;
    double s1 = 0.0, s2 = 0.0;
    for (int64_t w = tid; w < n_waves; w += kTotalThreads) { s1 += sums[w].x; s2 += sums[w].y; }
    s1 = wave_reduce(s1, OpAdd());
    s2 = wave_reduce(s2, OpAdd());
    if ((tid & 63) == 0) { red1[tid >> 6] = s1; red2[tid >> 6] = s2; }
    __syncthreads();
    if (tid < 64) {
        s1 = 0.0; s2 = 0.0;
        for (int w = 0; w < kTotalThreads / 64; ++w) { s1 += red1[w]; s2 += red2[w]; }
        gg_fit_t f;
        solve_fit_wave(s1, s2, n_elems, f);
        if (tid == 0) out[0] = f;
    }
}

// parameters for calls that do not fit first (one thread per unit)
__global__ void k_seg_prepare(SegView sv, PrepArgs prep) {
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (prep.hist) {                     // the histograms of the sweep that follows start at zero
        const int64_t words = (int64_t)sv.S * prep.nbins;
        for (int64_t i = gid; i < words; i += (int64_t)gridDim.x * blockDim.x) prep.hist[i] = 0;
    }
    if (gid >= sv.S) return;
    const int seg = (int)gid;
    float alpha = 0.f, beta = 0.f;
    if (prep.fit) { alpha = prep.fit[seg].alpha; beta = prep.fit[seg].beta; }
    prepare_unit(prep, seg, unit_len(sv, seg), alpha, beta);
}

__global__ void k_delta_from_fit(const gg_fit_t *__restrict__ fit, int32_t S, float delta_div,
                                 float *__restrict__ out) {
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s < S) out[s] = (float)((double)fit[s].alpha / (double)delta_div);
}

// ---------------------------------------------------------------------------------------------
// sweep 2: quantise / rate / histogram / symbols / penalty
// ---------------------------------------------------------------------------------------------
struct QuantArgs {
    const SegParam *params;   // device per-unit parameters, or nullptr to use `single`
    SegParam single;
    gg_rate_t *rate;          // device, per unit (RATE)
    uint32_t eg_add;          // 2^k
    uint32_t eg_const;        // 63 - k:  len(u) = eg_const - 2 clz(u + 2^k)
    // EXTRA
    int32_t *symbols;
    uint64_t *hist;           // S * nbins
    int32_t nbins;
    int32_t lbins;            // bins privatised in LDS
    int32_t cbins;            // k_hist: bins of the column layout (each in kHistCopies copies)
    int32_t lds_words;        // k_hist: 32-bit counters in LDS, either layout with its spare counter(s)
    // PEN
    float *grad;
    int accumulate;
    // FIT
    double2 *partials;
    RatePiece *pieces;        // RATE: per-run slots for units that several runs share
    PartSlot *part_slots;     // RATE with a written stream: one slot per block (k_quant_parts)
    // work split
    int64_t n_chunks;
    int32_t chunks_per_block;
    int32_t parts;            // element-wise sweeps: blocks per chunk
};

constexpr int32_t kQLimI = 1 << 30;   // |q| <= 2^30

// Saturating float -> int conversion of the hardware: NaN gives 0, out-of-range values give
// INT_MIN / INT_MAX (a plain C cast would be undefined for those inputs).
__device__ __forceinline__ int32_t cvt_i32_sat(float r) {
    int32_t m;
    asm("v_cvt_i32_f32 %0, %1" : "=v"(m) : "v"(r));
    return m;
}

// v_log_f32 / v_exp_f32 with the denormal range of the argument rescaled
__device__ __forceinline__ float log2_full(float t) {
    const bool tiny = t < 0x1p-100f;
    const float l = __builtin_amdgcn_logf(tiny ? t * 0x1p+64f : t);
    return tiny ? l - 64.0f : l;
}

// Outputs are written once and not re-read by this library: streaming (non-temporal) stores.  Every
// output-writing kernel handles four elements per lane, so a wave's store instruction covers 1 KiB
// of whole cache lines; with eight per lane each instruction would cover only every other 16
// bytes, and such partial-line streaming stores were measured to halve the write bandwidth.
template <int W, typename V>
__device__ __forceinline__ void stream_store(V v, V *p) {
    static_assert(W == 4, "output-writing kernels use four elements per lane");
    __builtin_nontemporal_store(v, p);
}
template <int W, typename V>
__device__ __forceinline__ V stream_load(const V *p) {
    static_assert(W == 4, "output-writing kernels use four elements per lane");
    return __builtin_nontemporal_load(p);
}

template <int MODE, bool RATE, bool PEN, bool EXTRA, bool FIT = false>
struct QuantBody {
    // moment sums of the current chunk when the sweep also fits (FIT): the one-sweep mode
    float s1[4] = {0.f, 0.f, 0.f, 0.f};
    float s2[4] = {0.f, 0.f, 0.f, 0.f};
    // unit parameters
    float inv_delta, inv_alpha, beta_m1, pen_coef;
    bool pen_live, hist_live;
    uint32_t eg_add;
    // outputs
    int32_t *symbols; float *grad; int accumulate;
    uint32_t *lds_hist; uint64_t *ghist; uint32_t last_bin, lbins;
    uint32_t fast_lim = 0;     // min(lbins, last_bin) while a histogram is live, else 0: symbols below it need no further test
    // per-lane accumulators
    uint32_t clz_sum = 0, u_max = 0, n_clamped = 0, n_last = 0;
    bool nan_seen = false;
    // MODE bit 0: 0 = floor, 1 = nearest-even.  MODE bit 1 (only with k = 0 and neither histogram nor
    // symbols): the code length is read off the float exponent of |q| instead of the integer symbol:
    //   q > 0: u + 1 = 2q;  q < 0: u + 1 = 2|q| + 1;  both have floor(log2(u + 1)) = 1 + floor(log2 |q|),
    // and floor(log2 |q|) is the biased exponent of the integer-valued float |q| minus 127.  With 0.5
    // standing in for q = 0 (exponent 126), len(u) = 2 floor(log2(u+1)) + 1 = 2 e - 251 for every element.
    // u_max follows from the extremes of r = -q, since Map grows with |q| on either side of zero.
    static constexpr bool kNearest = (MODE & 1) != 0;
    static constexpr bool kExp0 = (MODE & 2) != 0;
    static_assert(!kExp0 || (RATE && !EXTRA), "the exponent path forms no integer symbol: nothing to count in bins or to store");
    uint32_t exp_sum = 0;
    float r_max = 0.f, r_min = 0.f;      // 0 is neutral: Map(0) = 0

    __device__ __forceinline__ void quant_exp0(float x) {
        const float t = x * inv_delta;                 // the one fp32 rounding of the quantiser
        nan_seen |= (t != t);
        const float r = kNearest ? rintf(-t) : ceilf(-t);                       // -q, not yet clamped; NaN stays NaN
        const float a = __builtin_amdgcn_fmed3f(fabsf(r), 0.5f, 1073741824.0f);  // |q| in [1, 2^30], 0.5 for q = 0 and NaN
        exp_sum += __float_as_uint(a) >> 23;
        r_max = fmaxf(r_max, r);                       // NaN operands are ignored by v_max / v_min
        r_min = fminf(r_min, r);
    }

    // largest symbol seen by this lane on the exponent path
    __device__ __forceinline__ uint32_t exp0_u_max() const {
        uint32_t best = 0;
        const float ends[2] = {r_max, r_min};
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            int32_t m = cvt_i32_sat(ends[e]);
            m = m < -kQLimI ? -kQLimI : (m > kQLimI ? kQLimI : m);
            const uint32_t u = ((uint32_t)m << 1) ^ (uint32_t)(m >> 31);
            best = u > best ? u : best;
        }
        return best;
    }

    // Symbols past the block-private bins go straight to the unit's histogram, except the last bin: it
    // collects every clamped symbol, and atomics of many blocks on that one address serialise, so each lane
    // counts its hits and the block adds them once.
    __device__ __forceinline__ void hist_rare(uint32_t u) {
        const uint32_t bin = u < last_bin ? u : last_bin;
        n_clamped += u > last_bin ? 1u : 0u;
        if (bin < lbins) atomicAdd(&lds_hist[bin], 1u);
        else if (bin == last_bin) n_last += 1u;
        else atomicAdd(reinterpret_cast<unsigned long long *>(&ghist[bin]), 1ull);
    }

    __device__ __forceinline__ int32_t quant(float x) {
        const float t = x * inv_delta;                 // the one fp32 rounding of the quantiser
        nan_seen |= (t != t);
        // m = -q: floor(t) = -ceil(-t), rint is odd-symmetric.  The conversion maps NaN to 0 and
        // saturates, so clamping the integer to +-2^30 equals clamping t before rounding.
        const float r = kNearest ? rintf(-t) : ceilf(-t);
        int32_t m = cvt_i32_sat(r);
        m = m < -kQLimI ? -kQLimI : (m > kQLimI ? kQLimI : m);
        // Map(q) = q > 0 ? 2q-1 : -2q  is the zig-zag code of m = -q
        const uint32_t u = ((uint32_t)m << 1) ^ (uint32_t)(m >> 31);
        clz_sum += (uint32_t)__builtin_clz(u + eg_add);
        u_max = u > u_max ? u : u_max;
        if constexpr (EXTRA) {
            // Common case first: the symbol is its own bin (not clamped) and the bin is block-private -- one
            // compare and one LDS increment.  Everything else (clamping bin, bins beyond the private ones)
            // is rare and handled apart, so that the common path carries no further tests.
            if (u < fast_lim) atomicAdd(&lds_hist[u], 1u);
            else if (hist_live) hist_rare(u);
        }
        return -m;
    }

    __device__ __forceinline__ float penalty(float w) {
        const float a = fabsf(w);
        const float e = __builtin_amdgcn_exp2f(beta_m1 * log2_full(a * inv_alpha));
        float p = pen_coef * e;
        p = w < 0.f ? -p : p;
        return (a > 0.f && pen_live) ? p : 0.f;       // sign(0) = 0; NaN inputs give 0
    }

    template <int W>
    __device__ __forceinline__ void vec(const float (&v)[W], int64_t idx) {
        if constexpr (FIT) {
#pragma unroll
            for (int j = 0; j < W; ++j) {
                s1[j & 3] += fabsf(v[j]);
                s2[j & 3] = __builtin_fmaf(v[j], v[j], s2[j & 3]);
            }
        }
        if constexpr (RATE && kExp0) {
#pragma unroll
            for (int j = 0; j < W; ++j) quant_exp0(v[j]);
        } else if constexpr (RATE) {
            int32_t q[W];
#pragma unroll
            for (int j = 0; j < W; ++j) q[j] = quant(v[j]);
            if constexpr (EXTRA) {
                if (symbols) {
#pragma unroll
                    for (int j = 0; j < W; j += 4) {
                        gg_i4 qv = {q[j], q[j + 1], q[j + 2], q[j + 3]};
                        stream_store<W>(qv, reinterpret_cast<gg_i4 *>(symbols + idx + j));
                    }
                }
            }
        }
        if constexpr (PEN) {
#pragma unroll
            for (int j = 0; j < W; j += 4) {
                gg_f4 g = {penalty(v[j]), penalty(v[j + 1]), penalty(v[j + 2]), penalty(v[j + 3])};
                gg_f4 *dst = reinterpret_cast<gg_f4 *>(grad + idx + j);
                if (accumulate) g += stream_load<W>(dst);
                stream_store<W>(g, dst);
            }
        }
    }

    __device__ __forceinline__ void one(float v, int64_t idx) {
        if constexpr (FIT) {
            s1[0] += fabsf(v);
            s2[0] = __builtin_fmaf(v, v, s2[0]);
        }
        if constexpr (RATE && kExp0) {
            quant_exp0(v);
        } else if constexpr (RATE) {
            const int32_t q = quant(v);
            if constexpr (EXTRA) { if (symbols) symbols[idx] = q; }
        }
        if constexpr (PEN) {
            const float g = penalty(v);
            grad[idx] = accumulate ? grad[idx] + g : g;
        }
    }
};

// A block owns a run of consecutive chunks.  Lane accumulators (bit-length sum, u_max, NaN seen,
// clamped count) live across chunks and are combined only when the run leaves a unit or ends: into the
// unit's rate record when the whole unit lies in this run, else into the run's slot for a unit that other
// runs share (k_rate_reduce / k_rate_finalize fold the slots).  Many blocks finishing on one record with
// atomics cost a single-tensor sweep of 67 M elements 25-35 us of 55-80.
// With FIT the same sweep also accumulates the moments exactly as k_fit_partials does (one-sweep mode:
// the steps are given up front, so nothing has to wait for the fit).
template <typename T, int MODE, bool RATE, bool PEN, bool EXTRA, bool FIT = false>
__global__ __launch_bounds__(kBlock) void k_quant(SegView sv, const T *__restrict__ x, QuantArgs a) {
    extern __shared__ uint32_t lds_hist[];
    __shared__ uint64_t red64[kWaves];
    __shared__ uint32_t red[4][kWaves];
    __shared__ double redd[2][kWaves];
    const int tid = threadIdx.x;
    if constexpr (!RATE && !FIT) {
        // element-wise (penalty only): many short blocks, `parts` of them per chunk, nothing to combine
        const int64_t chunk = blockIdx.x / a.parts;
        if (chunk >= a.n_chunks) return;
        const ChunkLoc L = locate(sv, chunk);
        int64_t start; int len;
        if (!chunk_part(L.start, L.len, (int)(blockIdx.x - chunk * a.parts), a.parts, start, len)) return;
        QuantBody<MODE, RATE, PEN, EXTRA, FIT> body;
        body.eg_add = a.eg_add; body.symbols = nullptr; body.grad = a.grad; body.accumulate = a.accumulate;
        body.lds_hist = nullptr; body.ghist = nullptr; body.last_bin = 0; body.lbins = 0; body.hist_live = false;
        const SegParam P = a.params ? a.params[L.seg] : a.single;
        body.inv_delta = P.inv_delta; body.inv_alpha = P.inv_alpha; body.beta_m1 = P.beta_m1;
        body.pen_coef = P.pen_coef; body.pen_live = !(P.flags & kPenZero);
        // 4096 elements per block at the default split: four loads per lane, all issued at once
        if constexpr (sizeof(T) == 2) process_chunk<ElemBf16x4, 4>(x, start, len, body);
        else process_chunk<Elem<T>, 4>(x, start, len, body);
        return;
    }
    const int64_t first = (int64_t)blockIdx.x * a.chunks_per_block;
    int64_t last = first + a.chunks_per_block;
    if (last > a.n_chunks) last = a.n_chunks;
    if (first >= last) return;

    const bool want_hist = EXTRA && a.hist != nullptr;
    if (want_hist) {
        for (int b = tid; b < a.lbins; b += kBlock) lds_hist[b] = 0;
        __syncthreads();
    }

    QuantBody<MODE, RATE, PEN, EXTRA, FIT> body;
    body.eg_add = a.eg_add;
    body.symbols = a.symbols; body.grad = a.grad; body.accumulate = a.accumulate;
    body.lds_hist = lds_hist;
    body.last_bin = (uint32_t)(a.nbins > 0 ? a.nbins - 1 : 0);
    body.lbins = (uint32_t)a.lbins;

    int piece_seg = -1;
    bool rate_live = false, piece_shared = false, piece_flushed = false;
    int64_t piece_elems = 0, piece_first = first;
    int32_t piece_chunks = 0;
    double d1 = 0.0, d2 = 0.0;     // FIT: fp64 lane totals of the (run, unit) piece

    auto flush = [&](bool piece_ends) {   // fold the lanes of this piece into the unit's record
        if constexpr (FIT) {
            if (piece_seg >= 0 && piece_ends) {   // same slot convention as k_fit_partials
                const double sa = wave_reduce(d1, OpAdd());
                const double sb = wave_reduce(d2, OpAdd());
                if ((tid & 63) == 0) { redd[0][tid >> 6] = sa; redd[1][tid >> 6] = sb; }
                __syncthreads();
                if (tid == 0) {
                    double2 r;
                    r.x = (redd[0][0] + redd[0][1]) + (redd[0][2] + redd[0][3]);
                    r.y = (redd[1][0] + redd[1][1]) + (redd[1][2] + redd[1][3]);
                    a.partials[piece_first] = r;
                }
                __syncthreads();
                d1 = 0.0; d2 = 0.0;
            }
        }
        if constexpr (RATE) {
            if (piece_seg >= 0) {
                constexpr bool kExp0 = decltype(body)::kExp0;
                // wave results of all sums through LDS at once: one barrier, every thread combines in wave order
                const uint64_t lsum_w = wave_reduce((uint64_t)(kExp0 ? body.exp_sum : body.clz_sum), OpAdd());
                const uint32_t um_w = wave_reduce(kExp0 ? body.exp0_u_max() : body.u_max, OpMax());
                const uint32_t nan_w = wave_reduce((uint32_t)body.nan_seen, OpOr());
                uint32_t ncl_w = 0, nlast_w = 0;
                if constexpr (EXTRA) {
                    ncl_w = wave_reduce(body.n_clamped, OpAdd());
                    nlast_w = wave_reduce(body.n_last, OpAdd());
                }
                if ((tid & 63) == 0) {
                    const int w = tid >> 6;
                    red64[w] = lsum_w; red[0][w] = um_w; red[1][w] = nan_w;
                    if constexpr (EXTRA) { red[2][w] = ncl_w; red[3][w] = nlast_w; }
                }
                __syncthreads();
                uint64_t lsum = red64[0];
                uint32_t um = red[0][0], nan = red[1][0], ncl = 0, nlast = 0;
                if constexpr (EXTRA) { ncl = red[2][0]; nlast = red[3][0]; }
#pragma unroll
                for (int w = 1; w < kWaves; ++w) {
                    lsum += red64[w]; um = red[0][w] > um ? red[0][w] : um; nan |= red[1][w];
                    if constexpr (EXTRA) { ncl += red[2][w]; nlast += red[3][w]; }
                }
                if (tid == 0 && rate_live) {
                    // sum of 63-k-2 clz(u+2^k), or with k = 0 on the exponent path of 2e-251
                    const uint64_t bits = kExp0 ? 2ull * lsum - 251ull * (uint64_t)piece_elems
                                                : (uint64_t)piece_elems * a.eg_const - 2ull * lsum;
                    const uint32_t fl = (nan ? GG_F_NONFINITE : 0u) | (um >= 2147483647u ? GG_F_SATURATED : 0u);
                    if (piece_shared) {
                        // other runs hold pieces of this unit: leave the sums in this run's slot
                        RatePiece *s = a.pieces + 2 * (int64_t)blockIdx.x + (piece_first == first ? 0 : 1);
                        RatePiece v;
                        v.bits = bits; v.u_max = um; v.n_clamped = ncl; v.flags = fl; v._pad[0] = v._pad[1] = 0;
                        if (piece_flushed) {
                            v.bits += s->bits; v.u_max = um > s->u_max ? um : s->u_max; v.n_clamped += s->n_clamped; v.flags |= s->flags;
                        }
                        *s = v;
                    } else {
                        // the whole unit lies in this run: its record is this block's alone
                        gg_rate_t *r = a.rate + piece_seg;
                        r->eg_bits += bits;
                        const uint32_t m = um > r->u_max ? um : r->u_max;
                        r->u_max = m;
                        if (m) r->fl_bits = 32u - (uint32_t)__builtin_clz(m);
                        r->n_clamped += ncl;
                        if (fl) r->flags |= fl;
                    }
                    if (nlast) atomicAdd(reinterpret_cast<unsigned long long *>(&body.ghist[body.last_bin]), (unsigned long long)nlast);
                }
                piece_flushed = true;
                if (want_hist && rate_live) {   // merge the block-private bins into the unit's histogram
                    uint64_t *g = a.hist + (int64_t)piece_seg * a.nbins;
                    // bins above the largest symbol this block saw are still zero
                    const int touched = um < (uint32_t)a.lbins ? (int)um + 1 : a.lbins;
                    for (int b = tid; b < touched; b += kBlock) {
                        const uint32_t c = lds_hist[b];
                        if (c) {
                            atomicAdd(reinterpret_cast<unsigned long long *>(&g[b]), (unsigned long long)c);
                            lds_hist[b] = 0;
                        }
                    }
                }
                __syncthreads();   // the LDS slots (and bins) are free for the next piece
            }
        }
        body.clz_sum = 0; body.u_max = 0; body.n_clamped = 0; body.n_last = 0; body.nan_seen = false;
        body.exp_sum = 0; body.r_max = 0.f; body.r_min = 0.f;
        piece_elems = 0; piece_chunks = 0;
    };

    RunCursor cur;
    for (cur.init(sv, first, last); cur.valid(); cur.next(sv)) {
        if (cur.L.seg != piece_seg || piece_chunks >= 32768) {
            flush(cur.L.seg != piece_seg);
            if (cur.L.seg != piece_seg) {
                piece_first = cur.chunk;
                piece_flushed = false;
                // does the unit reach into another run?
                const int64_t c0 = unit_chunk0(sv, cur.L.seg), c1 = unit_chunk1(sv, cur.L.seg);
                piece_shared = c0 < first || c1 > last;
            }
            piece_seg = cur.L.seg;
            const SegParam P = a.params ? a.params[piece_seg] : a.single;
            rate_live = RATE && !(P.flags & kSkipRate);
            body.inv_delta = P.inv_delta; body.inv_alpha = P.inv_alpha; body.beta_m1 = P.beta_m1;
            body.pen_coef = P.pen_coef; body.pen_live = !(P.flags & kPenZero);
            body.hist_live = want_hist && rate_live;
            body.fast_lim = body.hist_live ? (body.lbins < body.last_bin ? body.lbins : body.last_bin) : 0u;
            body.ghist = want_hist ? a.hist + (int64_t)piece_seg * a.nbins : nullptr;
        }
        // kernels that write one 4-byte output per element read bf16 eight bytes per lane (see ElemBf16x4)
        if constexpr (sizeof(T) == 2 && (PEN || EXTRA))
            process_chunk<ElemBf16x4, 8>(x, cur.L.start, cur.L.len, body);
        else
            process_chunk<Elem<T>, GG_U_QUANT>(x, cur.L.start, cur.L.len, body);
        if constexpr (FIT) {   // per chunk: <= 16-term fp32 lane sums into the fp64 lane totals
            add_lane_moments<Elem<T>, kBlock>(body.s1, body.s2, x, cur.L.start, cur.L.len, d1, d2);
#pragma unroll
            for (int j = 0; j < 4; ++j) { body.s1[j] = 0.f; body.s2[j] = 0.f; }
        }
        piece_elems += cur.L.len;
        piece_chunks += 1;
    }
    flush(true);
}

// The rate sweep that also writes a stream (penalty gradient and / or symbols; no histogram) as short blocks:
// a stream that writes as much as it reads moves fastest in blocks of 16 KiB, all loads of a block issued at
// once (a plain copy: 5.8 TB/s against 5.1-5.4 TB/s for 64 KiB per block or resident runs on MI355X).  Block
// chunk * parts + part takes part `part` of chunk `chunk` and leaves its sums in slot [blockIdx.x].
// With HIST the block also counts its symbols in private LDS bins and adds the bins it touched to the unit's histogram
// when it ends: the shape for tensors of a few chunks, where one block per chunk would leave most of the machine idle
// (a 4 MB tensor is 64 chunks for 256 compute units) and each block would be a chain of four load rounds.
template <typename T, int MODE, bool PEN, bool SYM, bool HIST = false>
__global__ __launch_bounds__(kBlock) void k_quant_parts(SegView sv, const T *__restrict__ x, QuantArgs a) {
    extern __shared__ uint32_t lds_hist[];
    __shared__ uint32_t red[5][kWaves];
    const int tid = threadIdx.x;
    const int64_t chunk = blockIdx.x / a.parts;
    if (chunk >= a.n_chunks) return;
    const ChunkLoc L = locate(sv, chunk);
    const SegParam P = a.params ? a.params[L.seg] : a.single;
    const bool rate_live = !(P.flags & kSkipRate);
    int64_t start; int len;
    const bool any = chunk_part(L.start, L.len, (int)(blockIdx.x - chunk * a.parts), a.parts, start, len);
    if constexpr (HIST) {
        for (int b = tid; b < a.lbins; b += kBlock) lds_hist[b] = 0;
        __syncthreads();
    }
    uint32_t lsum = 0, um = 0, nan = 0, ncl = 0, nlast = 0;
    uint64_t *ghist = HIST ? a.hist + (int64_t)L.seg * a.nbins : nullptr;
    if (any) {                                 // uniform over the block
        QuantBody<MODE, true, PEN, SYM || HIST> body;
        body.eg_add = a.eg_add;
        body.symbols = a.symbols; body.grad = a.grad; body.accumulate = a.accumulate;
        body.lds_hist = nullptr; body.ghist = nullptr; body.last_bin = 0; body.lbins = 0; body.hist_live = false;
        if constexpr (HIST) {
            body.lds_hist = lds_hist; body.ghist = ghist; body.last_bin = (uint32_t)(a.nbins - 1); body.lbins = (uint32_t)a.lbins;
            body.hist_live = rate_live;
            body.fast_lim = rate_live ? (body.lbins < body.last_bin ? body.lbins : body.last_bin) : 0u;
        }
        body.inv_delta = P.inv_delta; body.inv_alpha = P.inv_alpha; body.beta_m1 = P.beta_m1;
        body.pen_coef = P.pen_coef; body.pen_live = !(P.flags & kPenZero);
        if constexpr (sizeof(T) == 2) process_chunk<ElemBf16x4, 4>(x, start, len, body);
        else process_chunk<Elem<T>, 4>(x, start, len, body);
        // at most 4096 x 32 (leading zeros) or 4096 x 157 (exponents): fits 32 bits
        lsum = wave_reduce(decltype(body)::kExp0 ? body.exp_sum : body.clz_sum, OpAdd());
        um = wave_reduce(decltype(body)::kExp0 ? body.exp0_u_max() : body.u_max, OpMax());
        nan = wave_reduce((uint32_t)body.nan_seen, OpOr());
        if constexpr (HIST) {
            ncl = wave_reduce(body.n_clamped, OpAdd());
            nlast = wave_reduce(body.n_last, OpAdd());
        }
    }
    if ((tid & 63) == 0) {
        red[0][tid >> 6] = lsum; red[1][tid >> 6] = um; red[2][tid >> 6] = nan;
        if constexpr (HIST) { red[3][tid >> 6] = ncl; red[4][tid >> 6] = nlast; }
    }
    __syncthreads();                           // also: every increment of the private bins is done
    uint32_t m = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) m = red[1][w] > m ? red[1][w] : m;
    if (tid == 0) {
        PartSlot v{0u, 0u, 0u, 0u};
        if (any && rate_live) {
            uint32_t l = 0, f = 0, c = 0, nl = 0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                l += red[0][w]; f |= red[2][w];
                if constexpr (HIST) { c += red[3][w]; nl += red[4][w]; }
            }
            // sum of 63 - k - 2 clz(u + 2^k), or with k = 0 on the exponent path of 2 e - 251
            v.bits = (MODE & 2) ? 2u * l - 251u * (uint32_t)len : (uint32_t)len * a.eg_const - 2u * l;
            v.u_max = m;
            v.flags = (f ? GG_F_NONFINITE : 0u) | (m >= 2147483647u ? GG_F_SATURATED : 0u);
            v.n_clamped = c;
            if constexpr (HIST) {              // the clamping bin: counted per lane, added once per block
                if (nl) atomicAdd(reinterpret_cast<unsigned long long *>(&ghist[a.nbins - 1]), (unsigned long long)nl);
            }
        }
        a.part_slots[blockIdx.x] = v;
    }
    if constexpr (HIST) {
        if (any && rate_live) {                // bins above the largest symbol this block saw are still zero
            const int touched = m < (uint32_t)a.lbins ? (int)m + 1 : a.lbins;
#ifndef GG_HIST_PARTS_NOMERGE   // tuning builds (timing only: wrong counts)
            for (int b = tid; b < touched; b += kBlock) {
                const uint32_t c = lds_hist[b];
                if (c) atomicAdd(reinterpret_cast<unsigned long long *>(&ghist[b]), (unsigned long long)c);
            }
#endif
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Rate sweep with a histogram and nothing else to write (the entropy / Huffman statistics of a tensor): one
// workgroup of 1024 threads per compute unit shares ONE set of block-private counters -- 128 KiB of the 160 KiB
// of LDS -- so that sixteen waves hide each other's loads and the counters are merged into the unit's histogram
// once per compute unit instead of once per small block.
//
// What LDS increments cost here is bank conflicts, not their number: scattered over plain bins a wave's 64
// increments take about 21 cycles, in distinct banks they are free next to the load stream.  So the counters
// have two layouts, chosen per piece (block, unit) from 4096 of its elements:
//   columns  bins 0 .. 1022, each kept in 32 copies, copy (lane mod 32): a half-wave never meets in a bank.
//            For quantised GG data nearly every symbol is below 1023 (the shape makes the distribution peaked);
//            the few beyond go to the unit's histogram one by one.
//   plain    up to 32768 bins, one copy: any distribution.
// The layout changes the speed only: both count every element exactly.
//
// The common path spends 8 vector instructions and one LDS increment per element, without a branch: with r = -q
// (an integer-valued float) the symbol is u = 2|r| - [r < 0] = |2r + 1/2| - 1/2, and f = |2r + 1/2| + (C - 1/2)
// with C = 1.5 * 2^e is exact while it stays below 2^(e+1) and carries u, times the byte stride of a bin, in its
// low mantissa bits (e = 21: stride 4, e = 16: stride 128).  Codes are clamped to the first counter the layout
// does not have (a spare one), and the largest code of a group of elements tells whether any of them needs the
// exact integer route of the general sweep (NaN, symbols past the counters or past the histogram): only then
// is the group looked at again.  Bit count and largest symbol of the elements counted in the block's counters
// are derived from the counters when they are merged -- a bin IS its symbol.
// ---------------------------------------------------------------------------------------------
#ifndef GG_HIST_THREADS
#define GG_HIST_THREADS 1024
#endif
constexpr int kHistThreads = GG_HIST_THREADS;
constexpr int kHistWaves = kHistThreads / 64;
#ifndef GG_HIST_MAX_LDS_BINS
#define GG_HIST_MAX_LDS_BINS 32768
#endif
constexpr int kHistMaxLdsBins = GG_HIST_MAX_LDS_BINS;   // plain layout: private bins (128 KiB)
#ifndef GG_HIST_COPIES
#define GG_HIST_COPIES 32
#endif
constexpr int kHistCopies = GG_HIST_COPIES;         // column layout: copies of a bin, one per bank
constexpr int kHistColumnBins = kHistMaxLdsBins / kHistCopies - 1;   // and its bins (one more column is the spare counter)
#ifndef GG_HIST_RARE_MAX
#define GG_HIST_RARE_MAX 8
#endif
constexpr uint32_t kHistSampleRareMax = GG_HIST_RARE_MAX;   // symbols past the columns among them (of 4096) that still choose the columns

typedef __attribute__((address_space(3))) uint32_t lds_u32_t;
// LDS byte address of a __shared__ object, and an increment of the 32-bit counter at an LDS byte address
__device__ __forceinline__ uint32_t lds_address(uint32_t *p) { return (uint32_t)(uintptr_t)(lds_u32_t *)p; }
__device__ __forceinline__ void lds_increment(uint32_t byte_address) {
    __hip_atomic_fetch_add((lds_u32_t *)(uintptr_t)byte_address, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

#ifndef GG_HIST_RUNS_PER_BLOCK
#define GG_HIST_RUNS_PER_BLOCK 1
#endif
#ifndef GG_HIST_U
#define GG_HIST_U 4       // 16-byte loads a lane keeps in flight
#endif

// STRIDE = bytes from one bin to the next: 4 (plain) or 4 * kHistCopies (columns)
template <bool NEAREST, int STRIDE>
struct HistBody {
    static constexpr int kExp = 23 - (STRIDE == 4 ? 2 : (STRIDE == 128 ? 7 : 8));     // one unit in the last place of C is 1 / STRIDE
    static_assert(STRIDE == 4 || STRIDE == 128 || STRIDE == 256, "plain bins, or 32 / 64 copies");
    static constexpr uint32_t kMagicBits = ((uint32_t)(kExp + 127) << 23) | 0x400000u;  // C = 1.5 * 2^kExp
    float inv_delta, magic_m_half;   // C - 1/2
    uint32_t lim_bits;               // kMagicBits + STRIDE * fast_lim: codes from here on are not counted in the block's counters
    uint32_t lds_bins;               // LDS byte address of this lane's copy of bin 0
    uint64_t *ghist;
    uint32_t last_bin, fast_lim, eg_add, eg_const;
    // what does not come out of the block's counters
    uint64_t rare_bits = 0;
    uint32_t rare_umax = 0, n_clamped = 0, n_last = 0;
    bool nan_seen = false;

    __device__ __forceinline__ void setup(float inv_delta_, uint32_t lds_base, uint32_t fast_lim_) {
        inv_delta = inv_delta_; fast_lim = fast_lim_;
        magic_m_half = __uint_as_float(kMagicBits) - 0.5f;
        lim_bits = kMagicBits + (uint32_t)STRIDE * fast_lim_;
        lds_bins = lds_base + (STRIDE == 4 ? 0u : 4u * (threadIdx.x & (uint32_t)(STRIDE / 4 - 1)));
    }

    // C + u as a bit pattern: kMagicBits + STRIDE u while exact, larger (as an unsigned number) for larger symbols and NaN
    __device__ __forceinline__ uint32_t code(float x, float &t, float &r) const {
        t = x * inv_delta;                                            // the one fp32 rounding of the quantiser
        r = NEAREST ? rintf(-t) : ceilf(-t);
        const float g = __builtin_fmaf(r, 2.0f, 0.5f);                // exact while |r| < 2^22
        return __float_as_uint(fabsf(g) + magic_m_half);              // exact below 2^(kExp+1), monotone beyond
    }

    // the exact integer route of the general sweep, for an element the block's counters do not take
    __device__ __forceinline__ void rare(float t, float r) {
        nan_seen |= (t != t);
        int32_t m = cvt_i32_sat(r);                                   // NaN -> 0, saturating
        m = m < -kQLimI ? -kQLimI : (m > kQLimI ? kQLimI : m);
        const uint32_t u = ((uint32_t)m << 1) ^ (uint32_t)(m >> 31);
        if (u < fast_lim) { lds_increment(lds_bins + (uint32_t)STRIDE * u); return; }   // a NaN's symbol 0: counted and priced through its bin
        rare_bits += eg_const - 2u * (uint32_t)__builtin_clz(u + eg_add);
        rare_umax = u > rare_umax ? u : rare_umax;
        if (u >= last_bin) { n_last += 1u; n_clamped += u > last_bin ? 1u : 0u; }
        else atomicAdd(reinterpret_cast<unsigned long long *>(&ghist[u]), 1ull);   // fast_lim <= u < last_bin
    }

    template <int W>
    __device__ __forceinline__ void vec(const float (&v)[W], int64_t) {
        uint32_t top = 0;
        const uint32_t base = lds_bins - kMagicBits;
#pragma unroll
        for (int j = 0; j < W; ++j) {
            float t, r;
            const uint32_t b = code(v[j], t, r);
            top = b > top ? b : top;
            lds_increment((b < lim_bits ? b : lim_bits) + base);      // its bin, or the spare counter
        }
        if (top >= lim_bits) {
#pragma unroll
            for (int j = 0; j < W; ++j) {
                float t, r;
                if (code(v[j], t, r) >= lim_bits) rare(t, r);
            }
        }
    }
    __device__ __forceinline__ void one(float v, int64_t) {
        float t, r;
        const uint32_t b = code(v, t, r);
        if (b < lim_bits) lds_increment(b + (lds_bins - kMagicBits));
        else rare(t, r);
    }
};

struct HistPiece {           // what a block knows about the piece it is on (uniform over the block)
    const SegParam *P;
    uint64_t *ghist;
    uint32_t last_bin;
};

// one sub-piece [e0, e) in layout STRIDE: count, then merge the block's counters into the unit's histogram.
// Leaves the piece's sums in red64 / red (combined by thread 0 of the caller).
template <typename T> using HistWalk = AheadWalk<Elem<T>, GG_HIST_U, kHistThreads>;

template <typename T, bool NEAREST, int STRIDE>
__device__ __forceinline__ void hist_sub_piece(HistWalk<T> &walk, const QuantArgs &a, const HistPiece &pc,
                                               uint32_t *lds_hist, uint32_t fast_lim, uint64_t *red64, uint32_t (*red)[kHistWaves]) {
    const int tid = threadIdx.x;
    HistBody<NEAREST, STRIDE> body;
    body.setup(pc.P->inv_delta, lds_address(lds_hist), fast_lim);
    body.ghist = pc.ghist; body.last_bin = pc.last_bin; body.eg_add = a.eg_add; body.eg_const = a.eg_const;
    walk.run(body);
    __syncthreads();                                  // every increment of this piece is in the counters
    // merge: a thread's bins, ascending; their elements' code lengths and the largest symbol come with them
    uint64_t bits = body.rare_bits;
    uint32_t um = body.rare_umax;
    for (uint32_t b = tid; b < fast_lim; b += kHistThreads) {
        uint32_t c;
        if constexpr (STRIDE == 4) {
            c = lds_hist[b];
            if (c) lds_hist[b] = 0;
        } else {                                      // the copies of bin b, starting at copy b so that the lanes of a wave stay in distinct banks
            constexpr int kCopies = STRIDE / 4;
            uint32_t *row = lds_hist + b * kCopies;
            c = 0;
#pragma unroll 8
            for (int k = 0; k < kCopies; ++k) {
                const int kk = (k + (int)b) & (kCopies - 1);
                c += row[kk];
                row[kk] = 0;
            }
        }
        if (c) {
            atomicAdd(reinterpret_cast<unsigned long long *>(&pc.ghist[b]), (unsigned long long)c);
            bits += (uint64_t)c * (a.eg_const - 2u * (uint32_t)__builtin_clz(b + a.eg_add));
            um = b > um ? b : um;
        }
    }
    // the spare counter(s) too: the next piece may use the other layout, where these words are bins
    if (tid < STRIDE / 4) lds_hist[fast_lim * (STRIDE / 4) + tid] = 0;
    bits = wave_reduce(bits, OpAdd());
    um = wave_reduce(um, OpMax());
    const uint32_t nan_w = wave_reduce((uint32_t)body.nan_seen, OpOr());
    const uint32_t ncl_w = wave_reduce(body.n_clamped, OpAdd());
    const uint32_t nlast_w = wave_reduce(body.n_last, OpAdd());
    if ((tid & 63) == 0) {
        const int w = tid >> 6;
        red64[w] = bits; red[0][w] = um; red[1][w] = nan_w; red[2][w] = ncl_w; red[3][w] = nlast_w;
    }
    __syncthreads();
}

template <typename T, bool NEAREST>
__global__ __launch_bounds__(kHistThreads) void k_hist(SegView sv, const T *__restrict__ x, QuantArgs a) {
    extern __shared__ __align__(16) uint32_t lds_hist[];
    __shared__ uint64_t red64[kHistWaves];
    __shared__ uint32_t red[4][kHistWaves];
    const int tid = threadIdx.x;
    const int64_t first = (int64_t)blockIdx.x * a.chunks_per_block;
    int64_t last = first + a.chunks_per_block;
    if (last > a.n_chunks) last = a.n_chunks;
    if (first >= last) return;
    const uint32_t last_bin = (uint32_t)(a.nbins - 1);
    const uint32_t fast_plain = (uint32_t)a.lbins < last_bin ? (uint32_t)a.lbins : last_bin;
    const uint32_t fast_cols = (uint32_t)a.cbins < last_bin ? (uint32_t)a.cbins : last_bin;
    bool lds_clear = false;
    int64_t chunk = first;
    while (chunk < last) {                                    // one piece per unit the run touches
        const ChunkLoc L = locate(sv, chunk);
        const int64_t c0u = unit_chunk0(sv, L.seg), c1u = unit_chunk1(sv, L.seg);
        const int64_t stop = c1u < last ? c1u : last;         // chunks [chunk, stop) of this unit are the block's
        const bool piece_shared = c0u < first || c1u > last;
        const bool first_slot = chunk == first;
        int64_t e0 = L.start, e1 = L.start + (stop - chunk) * kChunk;
        const int64_t uend = unit_end(sv, L.seg);
        if (e1 > uend) e1 = uend;
        const SegParam P = a.params ? a.params[L.seg] : a.single;
        chunk = stop;
        if (P.flags & kSkipRate) continue;                    // no usable step: nothing to count (uniform over the block)
        HistPiece pc{&P, a.hist + (int64_t)L.seg * a.nbins, last_bin};

        bool flushed = false;
        while (e0 < e1) {                                     // 32-bit counters and lane sums: at most 2^30 elements at a time
            const int64_t e = e1 - e0 > (1LL << 30) ? e0 + (1LL << 30) : e1;
            HistWalk<T> walk;
            walk.begin(x, e0, (int)(e - e0));                 // the first loads travel while the counters are cleared
            if (!lds_clear) {
                gg_u4 *z = reinterpret_cast<gg_u4 *>(lds_hist);
                for (int b = tid; b < (a.lds_words + 3) / 4; b += kHistThreads) z[b] = gg_u4{0u, 0u, 0u, 0u};
                lds_clear = true;                             // from here on every merge leaves them cleared
            }
            // Which layout?  The first vector of every lane (8192 or 4096 elements at the head of the piece) tells.
            bool columns = false;
            if (fast_cols > 0) {
                HistBody<NEAREST, 4 * kHistCopies> probe;
                probe.setup(P.inv_delta, 0u, fast_cols);
                uint32_t beyond = 0;
                walk.peek([&](const float (&v)[Elem<T>::W]) {
#pragma unroll
                    for (int j = 0; j < Elem<T>::W; ++j) {
                        float t, r;
                        beyond += probe.code(v[j], t, r) >= probe.lim_bits ? 1u : 0u;
                    }
                });
                beyond = wave_reduce(beyond, OpAdd());
                if ((tid & 63) == 0) red[0][tid >> 6] = beyond;
                __syncthreads();                              // also: the counters are cleared
                uint32_t all = 0;
#pragma unroll
                for (int w = 0; w < kHistWaves; ++w) all += red[0][w];
                // the same sum in every thread; taken from the first lane so that the branch below is a scalar one
                columns = (uint32_t)__builtin_amdgcn_readfirstlane((int)all) * 4096u <= kHistSampleRareMax * (uint32_t)(kHistThreads * Elem<T>::W);
            }
            __syncthreads();
#ifdef GG_HIST_FORCE_PLAIN     // tuning builds
            columns = false;
#endif
#ifdef GG_HIST_FORCE_COLUMNS
            columns = fast_cols > 0;
#endif
            if (columns) hist_sub_piece<T, NEAREST, 4 * kHistCopies>(walk, a, pc, lds_hist, fast_cols, red64, red);
            else hist_sub_piece<T, NEAREST, 4>(walk, a, pc, lds_hist, fast_plain, red64, red);
            if (tid == 0) {
                uint64_t tb = 0; uint32_t tu = 0, tn = 0, tc = 0, tl = 0;
                for (int w = 0; w < kHistWaves; ++w) {
                    tb += red64[w]; tu = red[0][w] > tu ? red[0][w] : tu; tn |= red[1][w]; tc += red[2][w]; tl += red[3][w];
                }
                const uint32_t fl = (tn ? GG_F_NONFINITE : 0u) | (tu >= 2147483647u ? GG_F_SATURATED : 0u);
                if (piece_shared) {                           // other runs hold pieces of this unit: this run's slot
                    RatePiece *sl = a.pieces + 2 * (int64_t)blockIdx.x + (first_slot ? 0 : 1);
                    RatePiece v;
                    v.bits = tb; v.u_max = tu; v.n_clamped = tc; v.flags = fl; v._pad[0] = v._pad[1] = 0;
                    if (flushed) { v.bits += sl->bits; v.u_max = tu > sl->u_max ? tu : sl->u_max; v.n_clamped += sl->n_clamped; v.flags |= sl->flags; }
                    *sl = v;
                } else {                                      // the whole unit lies in this run: its record is this block's alone
                    gg_rate_t *r = a.rate + L.seg;
                    r->eg_bits += tb;
                    const uint32_t m = tu > r->u_max ? tu : r->u_max;
                    r->u_max = m;
                    if (m) r->fl_bits = 32u - (uint32_t)__builtin_clz(m);
                    r->n_clamped += tc;
                    if (fl) r->flags |= fl;
                }
                if (tl) atomicAdd(reinterpret_cast<unsigned long long *>(&pc.ghist[last_bin]), (unsigned long long)tl);
            }
            flushed = true;
            e0 = e;
            __syncthreads();                                  // the reduction slots and the (cleared) counters are free again
        }
    }
}

// ---------------------------------------------------------------------------------------------
// wave-per-row pass.  For matrices whose rows fit a few cache lines per lane (activations: one row
// per token) a wave owns a row outright: it sums the moments, solves the fit, derives the row's
// step and immediately quantises the row again while it is still in cache.  Short rows are taken
// two at a time, so that the fp64 part of the solve runs once for both (lane r works for row r).
// No workspace, no atomics, no second kernel; HBM sees each element once.
// ---------------------------------------------------------------------------------------------
constexpr int64_t kRowWaveMax = 16384;   // elements per row this path takes
constexpr int64_t kRowBatchBytes = GG_ROW_BATCH_BYTES; // bytes of rows a wave holds in cache between its two sweeps

struct RowsArgs {
    int64_t rows, cols;
    gg_fit_t *fit;            // per-row fits (written when do_fit)
    gg_rate_t *rate;          // per-row rate records (RATE)
    const float *delta_dev;   // per-row steps when delta_div <= 0
    float delta_div, lambda;
    uint32_t eg_add, eg_const;
    int32_t *symbols; float *grad; int accumulate;
    int do_fit;
    int batch;                // rows per wave and solve, 1..kRowBatch (set by the launcher)
    double2 *wave_sums;       // per wave of the grid: sum |x|, sum x^2 over its rows (for the whole-matrix fit), or nullptr
    int64_t wave_sums_cap;    // host: entries wave_sums has room for
    gg_fit_t *total_out;      // host: where the whole-matrix fit goes (launched behind the row kernel), or nullptr
};

template <typename T, int MODE, bool RATE, bool PEN, bool EXTRA>
__global__ __launch_bounds__(kBlock) void k_rows(const T *__restrict__ x, RowsArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t n_waves = (int64_t)gridDim.x * kWaves;
    const int len = (int)a.cols;
    const int batch = a.batch;       // rows a wave takes at a time, 1..kRowBatch: one lane-parallel solve per batch
    double tot1 = 0.0, tot2 = 0.0;   // lane r: sums over the r-th rows of this wave's batches
    for (int64_t row0 = ((int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6)) * batch; row0 < a.rows; row0 += n_waves * batch) {
        const int nr = a.rows - row0 < batch ? (int)(a.rows - row0) : batch;
        // lane r < nr works for row row0 + r from here to the second sweep
        float alpha = 0.f, beta = 0.f;
        if (a.do_fit) {
            double my_s1 = 0.0, my_s2 = 0.0;
#pragma unroll
            for (int r = 0; r < kRowBatch; ++r) {
                if (r >= nr) break;
                FitBody fb;
                // cached loads: the row is read again a few microseconds later by this same wave
                process_chunk<Elem<T, !(RATE || PEN)>, 4, FitBody, 64>(x, (row0 + r) * a.cols, len, fb);
                double s1 = 0.0, s2 = 0.0;
                add_lane_moments<Elem<T, !(RATE || PEN)>, 64>(fb.s1, fb.s2, x, (row0 + r) * a.cols, len, s1, s2);
                s1 = wave_reduce(s1, OpAdd());
                s2 = wave_reduce(s2, OpAdd());
                if (lane == r) { my_s1 = s1; my_s2 = s2; }
            }
            gg_fit_t f;
            solve_fit_batch(my_s1, my_s2, (uint64_t)len, nr, f);
            if (lane < nr) { a.fit[row0 + lane] = f; alpha = f.alpha; beta = f.beta; }
            tot1 += my_s1; tot2 += my_s2;
        }
        if constexpr (RATE || PEN) {
            // the per-row constants of the second sweep, again one lane per row
            float delta = 0.f;
            if constexpr (RATE)
                if (lane < nr) delta = a.delta_div > 0.f ? (float)((double)alpha / (double)a.delta_div) : a.delta_dev[row0 + lane];
            const bool ok = delta > 0.f && isfinite(delta);
            const float inv_delta = ok ? (float)(1.0 / (double)delta) : 0.f;
            const bool pen_live = PEN && alpha > 0.f && isfinite(alpha) && isfinite(beta);
            const float inv_alpha = pen_live ? (float)(1.0 / (double)alpha) : 0.f;
            const float pen_coef = pen_live ? (float)((double)a.lambda * (double)beta / (double)alpha) : 0.f;
            const float beta_m1 = pen_live ? beta - 1.0f : 0.f;
#pragma unroll
            for (int r = 0; r < kRowBatch; ++r) {
                if (r >= nr) break;
                const int64_t row = row0 + r, start = row * a.cols;
                const float delta_r = __shfl(delta, r, 64);
                const bool ok_r = __shfl((int)ok, r, 64) != 0;
                QuantBody<MODE, RATE, PEN, EXTRA> body;
                body.eg_add = a.eg_add;
                body.symbols = a.symbols; body.grad = a.grad; body.accumulate = a.accumulate;
                body.lds_hist = nullptr; body.ghist = nullptr; body.last_bin = 0; body.lbins = 0; body.hist_live = false;
                body.inv_delta = __shfl(inv_delta, r, 64);
                body.pen_live = __shfl((int)pen_live, r, 64) != 0;
                body.inv_alpha = __shfl(inv_alpha, r, 64);
                body.pen_coef = __shfl(pen_coef, r, 64);
                body.beta_m1 = __shfl(beta_m1, r, 64);
                if constexpr (sizeof(T) == 2 && (PEN || EXTRA))
                    process_chunk<ElemBf16x4, 8, decltype(body), 64>(x, start, len, body);
                else
                    process_chunk<Elem<T>, 4, decltype(body), 64>(x, start, len, body);
                if constexpr (RATE) {
                    constexpr bool kExp0 = decltype(body)::kExp0;
                    const uint64_t lsum = wave_reduce((uint64_t)(kExp0 ? body.exp_sum : body.clz_sum), OpAdd());
                    const uint32_t um = wave_reduce(kExp0 ? body.exp0_u_max() : body.u_max, OpMax());
                    const uint32_t nan = wave_reduce((uint32_t)body.nan_seen, OpOr());
                    if (lane == 0) {
                        gg_rate_t rr;
                        rr.n = (uint64_t)len; rr.n_clamped = 0; rr.entropy_bits = 0.0; rr.delta = delta_r;
                        if (ok_r) {
                            rr.eg_bits = kExp0 ? 2ull * lsum - 251ull * (uint64_t)len : (uint64_t)len * a.eg_const - 2ull * lsum;
                            rr.u_max = um;
                            rr.fl_bits = um ? 32u - (uint32_t)__builtin_clz(um) : 1u;
                            rr.flags = (nan ? GG_F_NONFINITE : 0u) | (um >= 2147483647u ? GG_F_SATURATED : 0u);
                        } else {
                            rr.eg_bits = 0; rr.u_max = 0; rr.fl_bits = 0; rr.flags = GG_F_DEGENERATE;
                        }
                        a.rate[row] = rr;
                    }
                }
            }
        }
    }
    if (a.wave_sums) {               // every wave of the grid, also one without rows: the reader adds them all
        tot1 = wave_reduce(tot1, OpAdd());
        tot2 = wave_reduce(tot2, OpAdd());
        if (lane == 0) a.wave_sums[(int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6)] = make_double2(tot1, tot2);
    }
}

// Rows of at most 8 KiB whose byte length is a multiple of 16 (activations: a few thousand bf16 per token), fit +
// rate and nothing to write per element: the wave keeps its row in registers -- NV 16-byte vectors per lane --
// between the two sweeps, so memory sees every element exactly once whatever the caches hold, and the fit between
// the sweeps is the fp32-based one (no batching of rows: a fit costs less than a tenth of the row's sweeps).
#ifndef GG_ROWS_REG_WAVES
#define GG_ROWS_REG_WAVES 4
#endif
template <typename T, int NV, bool NEAREST>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(GG_ROWS_REG_WAVES, 8))) void k_rows_reg(const T *__restrict__ x, RowsArgs a) {
    using E = Elem<T, true>;                       // streaming loads: nothing is read twice
    using Raw = typename E::raw;
    constexpr int W = E::W;
    const int lane = threadIdx.x & 63;
    const int64_t n_waves = (int64_t)gridDim.x * kWaves;
    const int len = (int)a.cols;
    const int nvec = len / W;                      // the launcher takes only rows of whole vectors, NV = ceil(nvec / 64)
    const int padded = NV * 64 * W - len;          // elements a short last group is filled up with (zeros)
    // Loads are never predicated per lane (a predicated load makes the compiler wait for each one by itself):
    // lanes past the end of a short last group read the row's last vector again and zero it afterwards.
    auto load_row = [&](int64_t row, Raw (&dst)[NV]) {
        const T *__restrict__ p = x + row * a.cols;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int i = lane + 64 * v;
            dst[v] = E::loadv(p + (int64_t)((v < NV - 1 || i < nvec) ? i : nvec - 1) * W);
        }
    };
    double tot1 = 0.0, tot2 = 0.0;

    // one row from the registers `cur`; the wave's next row, if there is one, starts travelling into `nxt` on the way
    auto do_row = [&](int64_t row, Raw (&cur)[NV], Raw (&nxt)[NV]) {
        if (padded && lane + 64 * (NV - 1) >= nvec) cur[NV - 1] = Raw{};
        // sweep 1: moments, at most 16 terms per fp32 partial sum
        FitBody fb;
#pragma unroll
        for (int v = 0; v < NV; ++v) { float e[W]; E::unpack(cur[v], e); fb.vec(e, 0); }
        // (squares out of the fp32 range: the lane reads its share of the row again and forms them in fp64 -- a loop
        // that is not unrolled, so that this rare path costs the kernel no registers)
        double s1 = 0.0, s2 = 0.0;
        add_lane_moments<E, 64>(fb.s1, fb.s2, x, row * a.cols, len, s1, s2);
        s1 = wave_reduce(s1, OpAdd());
        s2 = wave_reduce(s2, OpAdd());
        gg_fit_t f;
        solve_fit_wave_f32(s1, s2, (uint64_t)len, f);
        if (lane == 0) a.fit[row] = f;
        tot1 += s1; tot2 += s2;
        // the row's step: one correctly rounded fp32 division each, as on the host
        const float delta = a.delta_div > 0.f ? f.alpha / a.delta_div : a.delta_dev[row];
        const bool ok = delta > 0.f && isfinite(delta);
        float inv_delta = ok ? 1.0f / delta : 0.f;
        asm volatile("" : "+v"(inv_delta));        // formed here, not where it is first used
        // The next row starts travelling now, after everything above that waits for memory (a wait behind a conditional
        // load waits for all loads): the registers the fit needed are free, and the second sweep and the reductions
        // behind it take about as long as the loads.
        __builtin_amdgcn_sched_barrier(0);         // (keeps the instruction scheduler from moving the division below the loads)
        if (row + n_waves < a.rows) load_row(row + n_waves, nxt);
        // sweep 2 from the registers.  The empty statements keep the compiler from carrying the widened fp32 values of
        // sweep 1 over the fit (twice or four times the registers of the packed row); they are formed again here.
#pragma unroll
        for (int v = 0; v < NV; ++v) asm volatile("" : "+v"(cur[v].x), "+v"(cur[v].y), "+v"(cur[v].z), "+v"(cur[v].w));
        // The exponent path (see QuantBody) two elements at a time: three-operand add, max and min.  Whether the row holds
        // a NaN is known from its sum of magnitudes, so no element is tested for it.
        uint32_t exp_sum = 0;
        float r_max = 0.f, r_min = 0.f;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            float e[W];
            E::unpack(cur[v], e);
#pragma unroll
            for (int j = 0; j < W; j += 2) {
                const float r0 = NEAREST ? rintf(-(e[j] * inv_delta)) : ceilf(-(e[j] * inv_delta));
                const float r1 = NEAREST ? rintf(-(e[j + 1] * inv_delta)) : ceilf(-(e[j + 1] * inv_delta));
                const float a0 = __builtin_amdgcn_fmed3f(fabsf(r0), 0.5f, 1073741824.0f);
                const float a1 = __builtin_amdgcn_fmed3f(fabsf(r1), 0.5f, 1073741824.0f);
                exp_sum += (__float_as_uint(a0) >> 23) + (__float_as_uint(a1) >> 23);
                r_max = fmaxf(fmaxf(r_max, r0), r1);       // NaN operands are ignored by v_max / v_min
                r_min = fminf(fminf(r_min, r0), r1);
            }
        }
        QuantBody<2, true, false, false> ends;     // (for the largest symbol from the two extremes of -q)
        ends.r_max = r_max; ends.r_min = r_min;
        // the zeros a short last group was filled up with were counted as symbol 0: exponent 126
        const uint64_t lsum = wave_reduce((uint64_t)exp_sum, OpAdd()) - 126ull * (uint64_t)padded;
        const uint32_t um = wave_reduce(ends.exp0_u_max(), OpMax());
        if (lane == 0) {
            gg_rate_t rr;
            rr.n = (uint64_t)len; rr.n_clamped = 0; rr.entropy_bits = 0.0; rr.delta = delta;
            if (ok) {
                rr.eg_bits = 2ull * lsum - 251ull * (uint64_t)len;
                rr.u_max = um;
                rr.fl_bits = um ? 32u - (uint32_t)__builtin_clz(um) : 1u;
                // an element is NaN exactly when the row's sum of magnitudes is (an infinite element makes it infinite, not NaN)
                rr.flags = (s1 != s1 ? GG_F_NONFINITE : 0u) | (um >= 2147483647u ? GG_F_SATURATED : 0u);
            } else {
                rr.eg_bits = 0; rr.u_max = 0; rr.fl_bits = 0; rr.flags = GG_F_DEGENERATE;
            }
            a.rate[row] = rr;
        }
    };

    // the wave index as a scalar, so that the branches on the row number are scalar branches
    int64_t row = (int64_t)blockIdx.x * kWaves + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    Raw ra[NV], rb[NV];                            // two register sets taking turns
    if (row < a.rows) load_row(row, ra);
    while (row < a.rows) {
        do_row(row, ra, rb);
        row += n_waves;
        if (row >= a.rows) break;
        do_row(row, rb, ra);
        row += n_waves;
    }
    if (a.wave_sums && lane == 0)     // every wave of the grid, also one without rows: the reader adds them all
        a.wave_sums[(int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6)] = make_double2(tot1, tot2);
}

// ---------------------------------------------------------------------------------------------
// Rate records of units that several runs share: the sweep left one slot per run (see RatePiece); these
// kernels fold them, in run order, into the record.  Units inside a single run are final already.
// ---------------------------------------------------------------------------------------------
struct PieceSum {
    uint64_t bits = 0, n_clamped = 0;
    uint32_t u_max = 0, flags = 0;
    __device__ __forceinline__ void add(const RatePiece &p) {
        bits += p.bits; u_max = p.u_max > u_max ? p.u_max : u_max; n_clamped += p.n_clamped; flags |= p.flags;
    }
};

// runs r0 .. r1 that overlap the chunks [c0, c1) of a unit; shared iff r0 < r1
__device__ __forceinline__ const RatePiece &piece_slot(const RatePiece *pieces, int64_t run, int32_t cpb, int64_t c0) {
    return pieces[2 * run + (run * cpb >= c0 ? 0 : 1)];   // the piece starts with the run unless the unit starts later
}

__device__ __forceinline__ void store_piece_sum(gg_rate_t *r, const PieceSum &t) {
    r->eg_bits = t.bits;
    r->u_max = t.u_max;
    r->fl_bits = t.u_max ? 32u - (uint32_t)__builtin_clz(t.u_max) : 1u;
    r->n_clamped = t.n_clamped;
    if (t.flags) r->flags |= t.flags;
}

// one workgroup per unit
__global__ __launch_bounds__(kBlock) void k_rate_reduce(SegView sv, const RatePiece *__restrict__ pieces, int32_t cpb,
                                                        gg_rate_t *__restrict__ rate) {
    __shared__ uint64_t red_bits[kWaves], red_ncl[kWaves];
    __shared__ uint32_t red_u[2][kWaves];
    const int seg = blockIdx.x, tid = threadIdx.x;
    const int64_t c0 = unit_chunk0(sv, seg), c1 = unit_chunk1(sv, seg);
    if (c1 <= c0) return;
    const int64_t r0 = c0 / cpb, r1 = (c1 - 1) / cpb;
    if (r0 == r1) return;
    gg_rate_t *r = rate + seg;
    if (r->flags & (GG_F_DEGENERATE | GG_F_EMPTY)) return;       // no rate was evaluated: the slots are stale
    PieceSum t;
#pragma unroll 4
    for (int64_t run = r0 + tid; run <= r1; run += kBlock) t.add(piece_slot(pieces, run, cpb, c0));
    t.bits = block_reduce(t.bits, OpAdd(), red_bits);
    t.u_max = block_reduce(t.u_max, OpMax(), red_u[0]);
    t.n_clamped = block_reduce(t.n_clamped, OpAdd(), red_ncl);
    t.flags = block_reduce(t.flags, OpOr(), red_u[1]);
    if (tid == 0) store_piece_sum(r, t);
}

// one lane per unit (many small units: few of them are shared, and those by few runs)
__global__ __launch_bounds__(64) void k_rate_reduce_lanes(SegView sv, const RatePiece *__restrict__ pieces, int32_t cpb,
                                                          gg_rate_t *__restrict__ rate) {
    const int seg = blockIdx.x * 64 + threadIdx.x;
    if (seg >= sv.S) return;
    const int64_t c0 = unit_chunk0(sv, seg), c1 = unit_chunk1(sv, seg);
    if (c1 <= c0) return;
    const int64_t r0 = c0 / cpb, r1 = (c1 - 1) / cpb;
    if (r0 == r1) return;
    gg_rate_t *r = rate + seg;
    if (r->flags & (GG_F_DEGENERATE | GG_F_EMPTY)) return;
    PieceSum t;
    for (int64_t run = r0; run <= r1; ++run) t.add(piece_slot(pieces, run, cpb, c0));
    store_piece_sum(r, t);
}

// the same for the slots of k_quant_parts: the blocks of a unit are consecutive, parts per chunk
template <int THREADS>
__device__ __forceinline__ void fold_part_slots(const PartSlot *__restrict__ slots, int64_t i0, int64_t i1, int t, PieceSum &acc) {
    const gg_u4 *__restrict__ p = reinterpret_cast<const gg_u4 *>(slots);
    for (int64_t i = i0 + t; i < i1; i += 8 * THREADS) {          // eight 16-byte loads in flight per thread
        gg_u4 v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int64_t j = i + (int64_t)k * THREADS;
            v[k] = j < i1 ? p[j] : gg_u4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            acc.bits += v[k].x; acc.u_max = v[k].y > acc.u_max ? v[k].y : acc.u_max; acc.flags |= v[k].z; acc.n_clamped += v[k].w;
        }
    }
}

constexpr int kPartReduceThreads = 1024;
__global__ __launch_bounds__(kPartReduceThreads) void k_rate_reduce_parts(SegView sv, const PartSlot *__restrict__ slots, int32_t parts,
                                                                          gg_rate_t *__restrict__ rate) {
    __shared__ uint64_t red_bits[kPartReduceThreads / 64];
    __shared__ uint32_t red_u[2][kPartReduceThreads / 64];
    const int seg = blockIdx.x, tid = threadIdx.x;
    const int64_t c0 = unit_chunk0(sv, seg), c1 = unit_chunk1(sv, seg);
    if (c1 <= c0) return;
    gg_rate_t *r = rate + seg;
    if (r->flags & (GG_F_DEGENERATE | GG_F_EMPTY)) return;       // no rate was evaluated
    PieceSum t;
    fold_part_slots<kPartReduceThreads>(slots, c0 * parts, c1 * parts, tid, t);
    t.bits = wave_reduce(t.bits, OpAdd());
    t.u_max = wave_reduce(t.u_max, OpMax());
    t.flags = wave_reduce(t.flags, OpOr());
    if ((tid & 63) == 0) { red_bits[tid >> 6] = t.bits; red_u[0][tid >> 6] = t.u_max; red_u[1][tid >> 6] = t.flags; }
    __syncthreads();
    if (tid == 0) {
        PieceSum all;
        for (int w = 0; w < kPartReduceThreads / 64; ++w) {
            all.bits += red_bits[w]; all.u_max = red_u[0][w] > all.u_max ? red_u[0][w] : all.u_max; all.flags |= red_u[1][w];
        }
        store_piece_sum(r, all);
    }
}

// one wave per unit (many small units)
__global__ __launch_bounds__(kBlock) void k_rate_reduce_parts_waves(SegView sv, const PartSlot *__restrict__ slots, int32_t parts,
                                                                    gg_rate_t *__restrict__ rate) {
    const int seg = blockIdx.x * kWaves + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (seg >= sv.S) return;
    const int64_t c0 = unit_chunk0(sv, seg), c1 = unit_chunk1(sv, seg);
    if (c1 <= c0) return;
    gg_rate_t *r = rate + seg;
    if (r->flags & (GG_F_DEGENERATE | GG_F_EMPTY)) return;
    PieceSum t;
    fold_part_slots<64>(slots, c0 * parts, c1 * parts, lane, t);
    t.bits = wave_reduce(t.bits, OpAdd());
    t.u_max = wave_reduce(t.u_max, OpMax());
    t.flags = wave_reduce(t.flags, OpOr());
    if (lane == 0) store_piece_sum(r, t);
}

// With a histogram: the same folding, then the entropy of the unit's bins.  `split` workgroups share a unit:
// workgroup j takes the bins [1024 (i split + j), 1024 (i split + j + 1)), i = 0, 1, ..., a thread one bin of each,
// and leaves the sum of its terms (lane-strided ascending, fixed tree: the same bits whatever the timing) in
// parts[seg * split + j]; the workgroup that delivers last adds the parts in the order of j and writes the
// record.  No workgroup waits for another.
constexpr int kFinalizeThreads = 1024;
constexpr int kFinalizeSplitMax = 8;
__global__ __launch_bounds__(kFinalizeThreads) void k_rate_finalize(SegView sv, const RatePiece *__restrict__ pieces, int32_t cpb,
                                                                    gg_rate_t *__restrict__ rate,
                                                                    const uint64_t *__restrict__ hist, int32_t nbins,
                                                                    SegParam *__restrict__ params, double *__restrict__ parts, int split,
                                                                    const PartSlot *__restrict__ slots, int32_t slot_parts) {
    __shared__ double red[kFinalizeThreads / 64];
    __shared__ uint64_t red_bits[kFinalizeThreads / 64], red_ncl[kFinalizeThreads / 64];
    __shared__ uint32_t red_u[2][kFinalizeThreads / 64];
    const int seg = blockIdx.x / split, part = blockIdx.x - seg * split, tid = threadIdx.x;
    gg_rate_t *r = rate + seg;
    const uint32_t flags = r->flags;
    const uint64_t n = r->n;
    const bool live = n > 0 && !(flags & GG_F_DEGENERATE);
    const int64_t c0 = unit_chunk0(sv, seg), c1 = unit_chunk1(sv, seg);
    const int64_t r0 = c1 > c0 ? c0 / cpb : 0, r1 = c1 > c0 ? (c1 - 1) / cpb : 0;
    // a sweep of short blocks left a slot per block (slot_parts of them per chunk): every unit is folded from those
    const bool shared = live && (slot_parts > 0 ? c1 > c0 : r0 < r1);           // uniform over the block
    if (shared) {                                  // every workgroup of the unit folds the slots: it needs the largest symbol
        PieceSum t;
        if (slot_parts > 0) fold_part_slots<kFinalizeThreads>(slots, c0 * slot_parts, c1 * slot_parts, tid, t);
        else for (int64_t run = r0 + tid; run <= r1; run += kFinalizeThreads) t.add(piece_slot(pieces, run, cpb, c0));
        t.bits = wave_reduce(t.bits, OpAdd());
        t.u_max = wave_reduce(t.u_max, OpMax());
        t.n_clamped = wave_reduce(t.n_clamped, OpAdd());
        t.flags = wave_reduce(t.flags, OpOr());
        if ((tid & 63) == 0) {
            red_bits[tid >> 6] = t.bits; red_u[0][tid >> 6] = t.u_max; red_ncl[tid >> 6] = t.n_clamped; red_u[1][tid >> 6] = t.flags;
        }
    }
    // bins above the unit's largest symbol are empty (a clamped symbol makes the largest >= nbins - 1): skip them
    uint32_t um = r->u_max;                        // final for a unit inside one run
    if (shared) {                                  // uniform over the block
        __syncthreads();
        um = 0;
        for (int w = 0; w < kFinalizeThreads / 64; ++w) um = red_u[0][w] > um ? red_u[0][w] : um;
    }
    const int used = um < (uint32_t)(nbins - 1) ? (int)um + 1 : nbins;
    double h = 0.0;
    if (live) {
        const uint64_t *g = hist + (int64_t)seg * nbins;
        const double inv_n = 1.0 / (double)n;
        for (int b = part * kFinalizeThreads + tid; b < used; b += split * kFinalizeThreads) {
            const uint64_t c = g[b];
            if (c) { const double p = (double)c * inv_n; h -= p * log2(p); }
        }
    }
    h = wave_reduce(h, OpAdd());
    if ((tid & 63) == 0) red[tid >> 6] = h;
    __syncthreads();
    if (tid == 0) {
        h = 0.0;
        for (int w = 0; w < kFinalizeThreads / 64; ++w) h += red[w];
        uint32_t before = 0;
        if (split > 1) {
            // deliver: the part, then (release) the ticket; whoever finds every other ticket taken reads (acquire) the parts
            __hip_atomic_store(reinterpret_cast<uint64_t *>(&parts[(int64_t)seg * split + part]), (uint64_t)__double_as_longlong(h),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            before = __hip_atomic_fetch_add(&params[seg].ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (before == (uint32_t)(split - 1)) {
            if (split > 1) {
                h = 0.0;
                for (int j = 0; j < split; ++j)
                    h += __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<uint64_t *>(&parts[(int64_t)seg * split + j]),
                                                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                __hip_atomic_store(&params[seg].ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // as it was found
            }
            if (shared) {
                PieceSum t;
                for (int w = 0; w < kFinalizeThreads / 64; ++w) {
                    t.bits += red_bits[w]; t.u_max = red_u[0][w] > t.u_max ? red_u[0][w] : t.u_max;
                    t.n_clamped += red_ncl[w]; t.flags |= red_u[1][w];
                }
                store_piece_sum(r, t);
            }
            r->entropy_bits = h;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// sampler
// ---------------------------------------------------------------------------------------------
constexpr int kMaxAttempts = 64;

struct SampleArgs {
    float alpha, a /* 1/beta */, d, c;
    int boost;
    uint32_t key0, key1, stream_id;
    uint64_t offset;
    int64_t n;
};

// One Marsaglia-Tsang attempt for element idx: true and the Gamma variate on acceptance.  w3 is the fourth
// Philox word of the attempt (sign and boost uniform are taken from attempt 0).
__device__ __forceinline__ bool gg_attempt(const SampleArgs &s, uint64_t idx, uint32_t attempt, float &gam, uint32_t &w3) {
    uint32_t w[4];
    philox4x32_10(attempt, s.stream_id, (uint32_t)idx, (uint32_t)(idx >> 32), s.key0, s.key1, w);
    w3 = w[3];
    // Box-Muller: v_cos_f32 takes its argument in revolutions
    const float rad = sqrtf(-2.0f * 0.69314718056f * __builtin_amdgcn_logf(unit_open(w[0])));
    const float z = rad * __builtin_amdgcn_cosf(unit_open(w[1]));
    const float t = 1.0f + s.c * z;
    const float v = t * t * t;
    if (v <= 0.f) return false;
    const float lu = 0.69314718056f * __builtin_amdgcn_logf(unit_open(w[2]));
    const float lv = 0.69314718056f * __builtin_amdgcn_logf(v);
    gam = s.d * v;
    return lu < 0.5f * z * z + s.d - s.d * v + s.d * lv;
}

// x from the accepted Gamma variate: G^(1/beta); with the boost G = G' U^beta so G^(1/beta) = G'^(1/beta) U
__device__ __forceinline__ float gg_finish(const SampleArgs &s, float gam, uint32_t w3_first) {
    float mag = __builtin_amdgcn_exp2f(s.a * __builtin_amdgcn_logf(gam));
    if (s.boost) mag *= unit_open(w3_first);
    const float xv = s.alpha * mag;
    return (w3_first & 1u) ? -xv : xv;
}

template <typename T>
__device__ __forceinline__ void gg_store(T *__restrict__ out, int64_t i, float v) {
    if constexpr (sizeof(T) == 2) out[i].bits = f32_to_bf16_rne(v);
    else out[i] = v;
}

// A wave draws kSampleRounds x 64 consecutive elements.  Every element's first attempt runs with all lanes
// busy; the few rejected ones (2-5 %) are queued in LDS and retried together, lanes packed, attempt after
// attempt -- instead of the whole wave looping until its slowest lane is through (twice the work on average).
// Element i always uses the Philox blocks (attempt, stream, i), so the result does not depend on this order.
#ifndef GG_SAMPLE_ROUNDS
#define GG_SAMPLE_ROUNDS 16
#endif
constexpr int kSampleRounds = GG_SAMPLE_ROUNDS;
constexpr int kSampleSpan = 64 * kSampleRounds;

template <typename T>
__global__ __launch_bounds__(kBlock) void k_sample(T *__restrict__ out, SampleArgs s) {
    __shared__ int64_t q_idx[kWaves][kSampleSpan];
    __shared__ uint32_t q_w3[kWaves][kSampleSpan];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t below = (1ull << lane) - 1ull;               // lanes before this one
    const int64_t n_waves = (int64_t)gridDim.x * kWaves;
    int64_t *qi = q_idx[wave];
    uint32_t *qw = q_w3[wave];
    for (int64_t base = ((int64_t)blockIdx.x * kWaves + wave) * kSampleSpan; base < s.n; base += n_waves * kSampleSpan) {
        int count = 0;                                          // queued elements (uniform over the wave)
#pragma unroll 2
        for (int r = 0; r < kSampleRounds; ++r) {
            const int64_t i = base + r * 64 + lane;
            const bool there = i < s.n;
            float gam = s.d;
            uint32_t w3 = 0;
            const bool ok = gg_attempt(s, s.offset + (uint64_t)i, 0u, gam, w3);
            if (there && ok) gg_store(out, i, gg_finish(s, gam, w3));
            const bool again = there && !ok;
            const uint64_t m = __ballot(again);
            if (again) { const int p = count + (int)__popcll(m & below); qi[p] = i; qw[p] = w3; }
            count += (int)__popcll(m);
        }
        for (uint32_t attempt = 1; attempt < (uint32_t)kMaxAttempts && count > 0; ++attempt) {
            int kept = 0;
            for (int b = 0; b < count; b += 64) {               // entries are read before any of this batch is re-queued
                const bool have = b + lane < count;
                const int64_t i = have ? qi[b + lane] : 0;
                const uint32_t w3_first = have ? qw[b + lane] : 0u;
                float gam = s.d;
                uint32_t w3;
                const bool ok = gg_attempt(s, s.offset + (uint64_t)i, attempt, gam, w3);
                if (have && ok) gg_store(out, i, gg_finish(s, gam, w3_first));
                const bool again = have && !ok;
                const uint64_t m = __ballot(again);
                if (again) { const int p = kept + (int)__popcll(m & below); qi[p] = i; qw[p] = w3_first; }
                kept += (int)__popcll(m);
            }
            count = kept;
        }
        // every attempt rejected (probability below 1e-80): the mode of the proposal stands in
        for (int b = 0; b < count; b += 64)
            if (b + lane < count) gg_store(out, qi[b + lane], gg_finish(s, s.d, qw[b + lane]));
    }
}

__global__ __launch_bounds__(kBlock) void k_philox_words(uint32_t *__restrict__ out, int64_t n, uint32_t key0, uint32_t key1,
                                                         uint32_t stream_id, uint64_t offset, uint32_t attempt) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        const uint64_t idx = offset + (uint64_t)i;
        uint32_t w[4];
        philox4x32_10(attempt, stream_id, (uint32_t)idx, (uint32_t)(idx >> 32), key0, key1, w);
        *reinterpret_cast<uint4 *>(out + 4 * i) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// =============================================================================================
// host side
// =============================================================================================
// Runs (blocks) per compute unit of the sweeps that reduce.  With no atomics in their epilogues (fit: one
// slot per piece; rate: records or run slots) several waves of blocks per compute unit balance the finish
// times better than one resident wave: 32-96 measured 1.5 % faster than 8 on the 1.5 G-element bucket, 128
// and more slower again.  Sweeps with block-private histogram bins stay at one resident wave: every block
// has its bins to merge.
#ifndef GG_FIT_RUNS_PER_CU
#define GG_FIT_RUNS_PER_CU 32
#endif
#ifndef GG_RATE_RUNS_PER_CU
#define GG_RATE_RUNS_PER_CU 64
#endif
#ifndef GG_RATE_PEN_RUNS_PER_CU
#define GG_RATE_PEN_RUNS_PER_CU 512   // rate sums and a written stream: short blocks win (one chunk each up to 2.1 G elements)
#endif
#ifndef GG_HIST_BLOCKS_PER_CU
#define GG_HIST_BLOCKS_PER_CU 8
#endif

// per-unit sums of the pieces written by a sweep that used `chunks_per_block`, and the solve
static int launch_fit_finalize(const Geometry &g, int32_t chunks_per_block, gg_fit_t *out, const PrepArgs *prep,
                               hipStream_t st) {
    if (g.S == 0) return GG_OK;
    PrepArgs p{};
    if (prep) p = *prep;
    if (g.S >= kManyUnits) {
        hipLaunchKernelGGL(k_fit_finalize_lanes, dim3((unsigned)((g.S + 63) / 64)), dim3(64), 0, st, g.sv, g.partials(),
                           chunks_per_block, out, p, prep ? 1 : 0);
    } else {
        hipLaunchKernelGGL(k_fit_finalize, dim3((unsigned)g.S), dim3(kFitFinalizeThreads), 0, st, g.sv, g.partials(), chunks_per_block, out,
                           p, prep ? 1 : 0);
    }
    return check_launch();
}

static int launch_fit(const Geometry &g, const void *x, int dtype, gg_fit_t *out, const PrepArgs *prep, hipStream_t st) {
    const RunSplit rs = split_runs(g.n_chunks, GG_FIT_RUNS_PER_CU);
    if (g.n_chunks > 0) {
        int rc = by_dtype(dtype, [&](auto *tag) {
            using T = std::remove_const_t<std::remove_pointer_t<decltype(tag)>>;
            hipLaunchKernelGGL(k_fit_partials<T>, dim3((unsigned)rs.blocks), dim3(kBlock), 0, st, g.sv,
                               static_cast<const T *>(x), g.partials(), g.n_chunks, rs.chunks_per_block);
            return check_launch();
        });
        if (rc != GG_OK) return rc;
    }
    return launch_fit_finalize(g, rs.chunks_per_block, out, prep, st);
}

struct QuantOpts {
    bool rate = false, pen = false;
    int eg_k = 0, round_mode = GG_FLOOR;
    int32_t nbins = 0;
    uint64_t *hist = nullptr;
    int32_t *symbols = nullptr;
    float *grad = nullptr;
    int accumulate = 0;
    gg_rate_t *rate_out = nullptr;
    const SegParam *params = nullptr;
    SegParam single{};
    bool fit_too = false;              // one-sweep mode: the rate sweep also writes moment partials
    bool hist_cleared = false;         // the kernel that prepared the units has cleared the histograms already
    int32_t chunks_per_block_out = 1;  // the run length the sweep used (the fit finalisation needs it)
    int32_t parts_out = 0;             // > 0: the sweep ran as short blocks and left one slot per block (k_quant_parts)
};

#ifndef GG_PEN_PARTS
#define GG_PEN_PARTS 4   // element-wise sweeps: blocks per chunk of 16384 elements
#endif
#ifndef GG_LDS_BINS
#define GG_LDS_BINS 12288
#endif
constexpr int kMaxLdsBins = GG_LDS_BINS;   // block-private bins (4 bytes each); higher symbols go to atomics on the unit's histogram
#ifndef GG_HIST_PARTS_MAX_CHUNKS
#define GG_HIST_PARTS_MAX_CHUNKS 192       // up to 3 M elements: histogram (+ symbols / penalty) as short blocks (equal at 4 M, slower from 8 M)
#endif
constexpr int64_t kHistPartsMaxChunks = GG_HIST_PARTS_MAX_CHUNKS;
#ifndef GG_HIST_PARTS
#define GG_HIST_PARTS 2
#endif
constexpr int kHistParts = GG_HIST_PARTS;  // blocks per chunk there (at most kStreamParts: the slot area is sized for that)
static_assert(kHistParts >= 1 && kHistParts <= kStreamParts, "slots");
constexpr int kHistPartsLdsBins = 4096;    // private bins of such a block (cleared and merged per 4096 elements)

template <typename T, int MODE, bool RATE, bool PEN, bool EXTRA, bool FIT = false>
static int launch_quant_inst(const Geometry &g, const void *x, QuantOpts &o, hipStream_t st) {
    QuantArgs a{};
    a.partials = g.ws ? g.partials() : nullptr;
    a.pieces = g.ws ? g.rate_pieces() : nullptr;
    a.params = o.params; a.single = o.single; a.rate = o.rate_out;
    a.eg_add = 1u << o.eg_k; a.eg_const = 63u - (uint32_t)o.eg_k;
    a.symbols = o.symbols; a.hist = o.hist; a.nbins = o.nbins;
    a.lbins = o.hist ? (o.nbins < kMaxLdsBins ? o.nbins : kMaxLdsBins) : 0;
    a.grad = o.grad; a.accumulate = o.accumulate;
    a.n_chunks = g.n_chunks;
    const size_t lds = (size_t)a.lbins * sizeof(uint32_t);
    // A sweep that only writes per-element results (no sums to combine) runs fastest as many short blocks: a
    // plain copy reaches 5.8 TB/s with 16 KiB per block against 5.1 TB/s with resident runs on MI355X.  Sweeps
    // that reduce keep one run per resident block (their per-block epilogue costs more than the balance gains).
    RunSplit rs;
    a.parts = 1;
    if constexpr (RATE && !FIT && EXTRA) {
        // a histogram over a few chunks only (a tensor of some megabytes): short blocks with private bins, or one
        // block per chunk would leave most of the compute units idle
        if (lds > 0 && g.n_chunks <= kHistPartsMaxChunks) {
            a.parts = kHistParts;
            a.part_slots = g.ws ? g.part_slots() : nullptr;
            if (!a.part_slots) return GG_ERR_WORKSPACE;
            if (a.lbins > kHistPartsLdsBins) a.lbins = kHistPartsLdsBins;
            o.parts_out = a.parts;
            hipLaunchKernelGGL((k_quant_parts<T, MODE, PEN, true, true>), dim3((unsigned)(g.n_chunks * a.parts)), dim3(kBlock),
                               (size_t)a.lbins * sizeof(uint32_t), st, g.sv, static_cast<const T *>(x), a);
            return check_launch();
        }
    }
    if constexpr (RATE && !FIT && (PEN || EXTRA)) {
        if (lds == 0) {              // rate sums and a written stream, no histogram: short blocks, one slot each
            a.parts = kStreamParts;
            a.part_slots = g.ws ? g.part_slots() : nullptr;
            if (!a.part_slots) return GG_ERR_WORKSPACE;
            if (g.n_chunks > 2147483647LL / a.parts) return GG_ERR_INVALID_ARG;
            o.parts_out = a.parts;
            hipLaunchKernelGGL((k_quant_parts<T, MODE, PEN, EXTRA>), dim3((unsigned)(g.n_chunks * a.parts)), dim3(kBlock), 0, st,
                               g.sv, static_cast<const T *>(x), a);
            return check_launch();
        }
    }
    if (!RATE && !FIT) {
        a.parts = GG_PEN_PARTS;      // 4096 elements per block = 256 lanes x 4 loads x 4 elements
        if (g.n_chunks > 2147483647LL / a.parts) return GG_ERR_INVALID_ARG;
        rs = RunSplit{g.n_chunks * a.parts, 1};
    }
    else if (lds > 0) rs = split_runs(g.n_chunks, resident_blocks(k_quant<T, MODE, RATE, PEN, EXTRA, FIT>, lds, GG_HIST_BLOCKS_PER_CU));
    else if (PEN || a.symbols) rs = split_runs(g.n_chunks, GG_RATE_PEN_RUNS_PER_CU);   // a written stream
    else rs = split_runs(g.n_chunks, GG_RATE_RUNS_PER_CU);
    if (RATE && (rs.blocks > kMaxRuns || !a.pieces)) return GG_ERR_WORKSPACE;
    a.chunks_per_block = rs.chunks_per_block;
    o.chunks_per_block_out = rs.chunks_per_block;
    hipLaunchKernelGGL((k_quant<T, MODE, RATE, PEN, EXTRA, FIT>), dim3((unsigned)rs.blocks), dim3(kBlock), lds, st, g.sv,
                       static_cast<const T *>(x), a);
    return check_launch();
}

template <typename T, int MODE>
static int launch_quant_mode(const Geometry &g, const void *x, QuantOpts &o, hipStream_t st) {
    const bool extra = o.hist || o.symbols;
    if constexpr ((MODE & 2) != 0) {   // exponent path: rate sums without the integer symbol, with or without the penalty
        if (o.pen) return launch_quant_inst<T, MODE, true, true, false>(g, x, o, st);
        if (o.fit_too) return launch_quant_inst<T, MODE, true, false, false, true>(g, x, o, st);
        return launch_quant_inst<T, MODE, true, false, false>(g, x, o, st);
    } else {
        if (o.fit_too && o.rate && !o.pen)
            return extra ? launch_quant_inst<T, MODE, true, false, true, true>(g, x, o, st)
                         : launch_quant_inst<T, MODE, true, false, false, true>(g, x, o, st);
        if (o.rate && !o.pen && !extra) return launch_quant_inst<T, MODE, true, false, false>(g, x, o, st);
        if (o.rate && o.pen && !extra) return launch_quant_inst<T, MODE, true, true, false>(g, x, o, st);
        if (o.rate && !o.pen && extra) return launch_quant_inst<T, MODE, true, false, true>(g, x, o, st);
        if (o.rate && o.pen && extra) return launch_quant_inst<T, MODE, true, true, true>(g, x, o, st);
        return GG_ERR_INVALID_ARG;
    }
}

// LDS a workgroup may use on the current device (a property of the device; asked once per device)
static size_t lds_per_block() {
    static std::atomic<size_t> cached[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 64u << 10;
    size_t v = cached[dev].load(std::memory_order_relaxed);
    if (v) return v;
    int bytes = 0;
    if (hipDeviceGetAttribute(&bytes, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess || bytes <= 0) bytes = 64 << 10;
    cached[dev].store((size_t)bytes, std::memory_order_relaxed);
    return (size_t)bytes;
}

// the histogram-only rate sweep: one workgroup of 1024 threads per compute unit (two where the bins leave room)
template <typename T, bool NEAREST>
static int launch_hist_inst(const Geometry &g, const void *x, QuantOpts &o, hipStream_t st) {
    QuantArgs a{};
    a.pieces = g.ws ? g.rate_pieces() : nullptr;
    if (!a.pieces) return GG_ERR_WORKSPACE;
    a.params = o.params; a.single = o.single; a.rate = o.rate_out;
    a.eg_add = 1u << o.eg_k; a.eg_const = 63u - (uint32_t)o.eg_k;
    a.hist = o.hist; a.nbins = o.nbins;
    const size_t room = (lds_per_block() - 1024) / sizeof(uint32_t);   // counters, beside the kernel's own reduction slots
    // plain layout: a counter per bin and a spare one; column layout: kHistCopies counters per bin and a spare column
    int64_t lbins = o.nbins < kHistMaxLdsBins ? o.nbins : kHistMaxLdsBins;
    if ((size_t)lbins + 1 > room) lbins = (int64_t)room - 1;
    int64_t cbins = o.nbins - 1 < kHistColumnBins ? o.nbins - 1 : kHistColumnBins;
    if ((size_t)(cbins + 1) * kHistCopies > room) cbins = (int64_t)(room / kHistCopies) - 1;
    if (cbins < 0) cbins = 0;
    const int64_t words = lbins + 1 > (cbins + 1) * kHistCopies ? lbins + 1 : (cbins + 1) * kHistCopies;
    a.lbins = (int32_t)lbins; a.cbins = (int32_t)cbins; a.lds_words = (int32_t)words;
    const size_t lds = (size_t)((words + 3) / 4 * 4) * sizeof(uint32_t);   // cleared 16 bytes at a time
    auto kernel = k_hist<T, NEAREST>;
    // (the attribute is a property of the kernel on the device and only ever raised: asked for once per size)
    static std::atomic<uint64_t> lds_allowed[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GG_ERR_HIP;
    if (lds > (48u << 10) && lds > lds_allowed[dev].load(std::memory_order_relaxed)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return GG_ERR_HIP;
        }
        lds_allowed[dev].store(lds, std::memory_order_relaxed);
    }
    int per_cu = workgroups_per_cu(reinterpret_cast<const void *>(kernel), kHistThreads, lds);
    if (per_cu > 2) per_cu = 2;
    // a few runs per resident workgroup: the compute units finish at different times, and a workgroup that met
    // a piece it has to count in plain bins takes longer than its neighbours
    const RunSplit rs = split_runs(g.n_chunks, per_cu * GG_HIST_RUNS_PER_BLOCK);
    if (rs.blocks > kMaxRuns) return GG_ERR_WORKSPACE;
    a.n_chunks = g.n_chunks; a.chunks_per_block = rs.chunks_per_block;
    o.chunks_per_block_out = rs.chunks_per_block;
    hipLaunchKernelGGL(kernel, dim3((unsigned)rs.blocks), dim3(kHistThreads), lds, st, g.sv, static_cast<const T *>(x), a);
    return check_launch();
}

static int launch_quant(const Geometry &g, const void *x, int dtype, QuantOpts &o, hipStream_t st) {
    if (g.n_chunks == 0) return GG_OK;
    return by_dtype(dtype, [&](auto *tag) {
        using T = std::remove_const_t<std::remove_pointer_t<decltype(tag)>>;
        if (!o.rate) return launch_quant_inst<T, GG_FLOOR, false, true, false>(g, x, o, st);
#ifndef GG_NO_HIST_KERNEL   // tuning builds
        if (o.hist && !o.symbols && !o.pen && !o.fit_too)
            return o.round_mode == GG_FLOOR ? launch_hist_inst<T, false>(g, x, o, st) : launch_hist_inst<T, true>(g, x, o, st);
#endif
        // kernel MODE: bit 0 = rounding, bit 1 = exponent-based lengths (k = 0, no histogram, no symbols)
#ifdef GG_NO_EXP0   // tuning builds
        const bool exp0 = false;
#else
        const bool exp0 = o.eg_k == 0 && !o.hist && !o.symbols;
#endif
        if (o.round_mode == GG_FLOOR) return exp0 ? launch_quant_mode<T, 2>(g, x, o, st) : launch_quant_mode<T, 0>(g, x, o, st);
        return exp0 ? launch_quant_mode<T, 3>(g, x, o, st) : launch_quant_mode<T, 1>(g, x, o, st);
    });
}


// after a rate sweep: fold the run slots of shared units into their records; with a histogram also the entropy
static int launch_rate_finalize(const Geometry &g, gg_rate_t *rate, const uint64_t *hist, int32_t nbins, int32_t cpb,
                                int32_t parts, hipStream_t st) {
    if (g.S == 0 || g.n_chunks == 0) return GG_OK;
    if (hist) {
        // few units: several workgroups share a unit's bins (their parts go where the moment partials were; the fit
        // that read those has run).  Many units keep the machine busy with a workgroup each.
        int split = 1;
        if (g.S <= 32 && nbins > kFinalizeThreads) {
            split = (nbins + kFinalizeThreads - 1) / kFinalizeThreads;
            if (split > kFinalizeSplitMax) split = kFinalizeSplitMax;
            if ((size_t)g.S * split * sizeof(double) > g.wl.partials_bytes) split = 1;
        }
        hipLaunchKernelGGL(k_rate_finalize, dim3((unsigned)(g.S * split)), dim3(kFinalizeThreads), 0, st, g.sv, g.rate_pieces(), cpb,
                           rate, hist, nbins, g.params(), reinterpret_cast<double *>(g.partials()), split,
                           parts > 0 ? g.part_slots() : nullptr, parts);
        return check_launch();
    }
    if (parts > 0) {                                     // short blocks: every unit's record comes from its slots
        if (g.S >= kManyUnits)
            hipLaunchKernelGGL(k_rate_reduce_parts_waves, dim3((unsigned)((g.S + kWaves - 1) / kWaves)), dim3(kBlock), 0, st, g.sv,
                               g.part_slots(), parts, rate);
        else
            hipLaunchKernelGGL(k_rate_reduce_parts, dim3((unsigned)g.S), dim3(kPartReduceThreads), 0, st, g.sv, g.part_slots(),
                               parts, rate);
        return check_launch();
    }
    if (g.n_chunks <= cpb) return GG_OK;                 // a single run: nothing is shared
    if (g.S >= kManyUnits)
        hipLaunchKernelGGL(k_rate_reduce_lanes, dim3((unsigned)((g.S + 63) / 64)), dim3(64), 0, st, g.sv, g.rate_pieces(), cpb,
                           rate);
    else
        hipLaunchKernelGGL(k_rate_reduce, dim3((unsigned)g.S), dim3(kBlock), 0, st, g.sv, g.rate_pieces(), cpb, rate);
    return check_launch();
}

static int launch_seg_prepare(const Geometry &g, const PrepArgs &p, hipStream_t st) {
    if (g.S == 0) return GG_OK;
    int64_t blocks = (g.S + 255) / 256;
    if (p.hist) {                        // enough threads to clear the histograms too
        int64_t want = ((int64_t)g.S * p.nbins + 2047) / 2048;
        if (want > 2048) want = 2048;
        if (want > blocks) blocks = want;
    }
    hipLaunchKernelGGL(k_seg_prepare, dim3((unsigned)blocks), dim3(256), 0, st, g.sv, p);
    return check_launch();
}

// wave-per-row launch: enough blocks to fill the machine, each wave strides over rows
template <typename T, int MODE, bool RATE, bool PEN, bool EXTRA>
static int launch_rows_inst(const void *x, RowsArgs a, hipStream_t st) {
    const int bpc = resident_blocks(k_rows<T, MODE, RATE, PEN, EXTRA>, 0, 8);
    const int64_t cap = (int64_t)kComputeUnits * bpc;
    // Rows of a batch are read again from cache after the solve: keep a batch within kRowBatchBytes, and
    // batch only while every resident wave still gets one.
    int batch = 1;
    while (batch < kRowBatch && a.cols * (int64_t)sizeof(T) * (2 * batch) <= kRowBatchBytes && a.rows >= cap * kWaves * (2 * batch))
        batch *= 2;
    a.batch = batch;
    const int64_t per_block = (int64_t)kWaves * batch;
    int64_t blocks = (a.rows + per_block - 1) / per_block;
    if (blocks > cap) blocks = cap;
    // the whole-matrix fit: from the sums the waves leave when the workspace has room for them (fewer and
    // smaller than the row records), else from the row records
    const bool want_total = a.total_out != nullptr && a.do_fit;
    const bool by_waves = want_total && a.wave_sums != nullptr && a.wave_sums_cap >= blocks * kWaves;
    if (!by_waves) a.wave_sums = nullptr;
    hipLaunchKernelGGL((k_rows<T, MODE, RATE, PEN, EXTRA>), dim3((unsigned)blocks), dim3(kBlock), 0, st,
                       static_cast<const T *>(x), a);
    if (want_total) {
        if (by_waves)
            hipLaunchKernelGGL(k_fit_total_waves, dim3(1), dim3(kTotalThreads), 0, st, (const double2 *)a.wave_sums, blocks * kWaves,
                               (uint64_t)(a.rows * a.cols), a.total_out);
        else
            hipLaunchKernelGGL(k_fit_total, dim3(1), dim3(kTotalThreads), 0, st, (const gg_fit_t *)a.fit, a.rows, a.total_out);
    }
    return check_launch();
}

template <typename T, int MODE>
static int launch_rows_mode(const void *x, const RowsArgs &a, bool rate, bool pen, bool extra, hipStream_t st) {
    if constexpr ((MODE & 2) != 0) {
        return launch_rows_inst<T, MODE, true, false, false>(x, a, st);
    } else {
        if (rate && !pen && !extra) return launch_rows_inst<T, MODE, true, false, false>(x, a, st);
        if (rate && pen && !extra) return launch_rows_inst<T, MODE, true, true, false>(x, a, st);
        if (rate && !pen && extra) return launch_rows_inst<T, MODE, true, false, true>(x, a, st);
        if (rate && pen && extra) return launch_rows_inst<T, MODE, true, true, true>(x, a, st);
        return GG_ERR_INVALID_ARG;
    }
}

static bool rows_take_wave_path(int64_t rows, int64_t cols) { return rows > 0 && cols > 0 && cols <= kRowWaveMax; }

// rows that fit a wave's registers (k_rows_reg): whole 16-byte vectors, at most 8 per lane; order-0 code lengths
constexpr int64_t kRowRegBytes = 8192;
template <typename T, bool NEAREST>
static int launch_rows_reg(const void *x, RowsArgs a, hipStream_t st) {
    const int64_t vecs = a.cols * (int64_t)sizeof(T) / 16;
    const int nv = (int)((vecs + 63) / 64);
    auto go = [&](auto kernel) {
        const int bpc = resident_blocks(kernel, 0, 8);
        const int64_t cap_waves = (int64_t)kComputeUnits * bpc * kWaves;
        const int64_t waves = a.rows < cap_waves ? a.rows : cap_waves;
        const int64_t blocks = (waves + kWaves - 1) / kWaves;
        const bool want_total = a.total_out != nullptr;
        if (want_total && !(a.wave_sums != nullptr && a.wave_sums_cap >= blocks * kWaves)) return -1;   // the caller takes the general kernel
        if (!want_total) a.wave_sums = nullptr;
        hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kBlock), 0, st, static_cast<const T *>(x), a);
        if (want_total)
            hipLaunchKernelGGL(k_fit_total_waves, dim3(1), dim3(kTotalThreads), 0, st, (const double2 *)a.wave_sums, blocks * kWaves,
                               (uint64_t)(a.rows * a.cols), a.total_out);
        return check_launch();
    };
    switch (nv) {
        case 1: return go(k_rows_reg<T, 1, NEAREST>);
        case 2: return go(k_rows_reg<T, 2, NEAREST>);
        case 3: return go(k_rows_reg<T, 3, NEAREST>);
        case 4: return go(k_rows_reg<T, 4, NEAREST>);
        case 5: return go(k_rows_reg<T, 5, NEAREST>);
        case 6: return go(k_rows_reg<T, 6, NEAREST>);
        case 7: return go(k_rows_reg<T, 7, NEAREST>);
        default: return go(k_rows_reg<T, 8, NEAREST>);
    }
}

static int launch_rows(const Geometry &g, const void *x, int dtype, RowsArgs a, int eg_k, int round_mode, bool rate, bool pen,
                       hipStream_t st) {
    a.eg_add = 1u << eg_k; a.eg_const = 63u - (uint32_t)eg_k;
    const bool extra = a.symbols != nullptr;
    return by_dtype(dtype, [&](auto *tag) {
        using T = std::remove_const_t<std::remove_pointer_t<decltype(tag)>>;
        if (!rate && !pen) return launch_rows_inst<T, GG_FLOOR, false, false, false>(x, a, st);
        if (!rate) return launch_rows_inst<T, GG_FLOOR, false, true, false>(x, a, st);
        const bool exp0 = eg_k == 0 && !extra && !pen;
#ifndef GG_NO_ROWS_REG   // tuning builds
        if (exp0 && a.do_fit && a.cols * (int64_t)sizeof(T) <= kRowRegBytes && (a.cols * (int64_t)sizeof(T)) % 16 == 0) {
            const int rc = round_mode == GG_FLOOR ? launch_rows_reg<T, false>(x, a, st) : launch_rows_reg<T, true>(x, a, st);
            if (rc != -1) return rc;
        }
#endif
        if (round_mode == GG_FLOOR)
            return exp0 ? launch_rows_mode<T, 2>(x, a, rate, pen, extra, st) : launch_rows_mode<T, 0>(x, a, rate, pen, extra, st);
        return exp0 ? launch_rows_mode<T, 3>(x, a, rate, pen, extra, st) : launch_rows_mode<T, 1>(x, a, rate, pen, extra, st);
    });
}

static int check_rate_args(int eg_k, int round_mode, int32_t nbins, const uint64_t *hist, const int32_t *symbols) {
    if (eg_k < 0 || eg_k > GG_MAX_EG_K) return GG_ERR_INVALID_ARG;
    if (round_mode != GG_FLOOR && round_mode != GG_NEAREST_EVEN) return GG_ERR_INVALID_ARG;
    if (nbins != 0 && (nbins < 2 || nbins > GG_MAX_BINS)) return GG_ERR_INVALID_ARG;
    if (nbins != 0 && (!hist || !aligned8(hist))) return GG_ERR_INVALID_ARG;
    if (symbols && !aligned16(symbols)) return GG_ERR_INVALID_ARG;
    return GG_OK;
}

// the second sweep and its finalisation, shared by every rate/penalty entry point
static int run_second_sweep(const Geometry &g, const void *x, int dtype, QuantOpts &o, hipStream_t st) {
    int rc;
    if (o.rate && o.nbins > 0 && !o.hist_cleared && (rc = launch_fill_u64(o.hist, (int64_t)g.S * o.nbins, st)) != GG_OK) return rc;
    if (!o.rate) { o.hist = nullptr; o.symbols = nullptr; o.nbins = 0; }
    if (o.nbins == 0) o.hist = nullptr;
    if (o.rate || o.pen) {
        if ((rc = launch_quant(g, x, dtype, o, st)) != GG_OK) return rc;
    }
    if (o.rate) return launch_rate_finalize(g, o.rate_out, o.hist, o.nbins, o.chunks_per_block_out, o.parts_out, st);
    return GG_OK;
}

static int fused_common(Geometry &g, const void *x, int dtype, float delta_div, const float *delta_dev, int eg_k,
                        int round_mode, int32_t nbins, uint64_t *hist, int32_t *symbols, float lambda, float *grad,
                        int accumulate, gg_fit_t *fit, gg_fit_t *total_fit, gg_rate_t *rate, hipStream_t st) {
    int rc;
    if ((rc = upload_geometry(g, st)) != GG_OK) return rc;
    PrepArgs p{};
    p.fit = nullptr; p.delta_dev = delta_dev; p.delta_div = delta_div; p.delta_scalar = 0.f;
    p.lambda = lambda; p.params = g.params(); p.rate = rate; p.want_pen = grad != nullptr;
    const bool with_hist = rate && nbins > 0 && hist;
    if (with_hist) { p.hist = hist; p.nbins = nbins; }
    if (rate && !grad && !(delta_div > 0.f) && delta_dev) {
        // One-sweep mode: the steps do not depend on this call's fit (e.g. they come from the previous
        // training step), so moments and rate are taken from a single read of x: 4 B/elem instead of 8.
        if ((rc = launch_seg_prepare(g, p, st)) != GG_OK) return rc;
        QuantOpts o;
        o.rate = true; o.eg_k = eg_k; o.round_mode = round_mode; o.nbins = nbins; o.hist = hist; o.symbols = symbols;
        o.rate_out = rate; o.params = g.params(); o.fit_too = true; o.hist_cleared = with_hist;
        if ((rc = run_second_sweep(g, x, dtype, o, st)) != GG_OK) return rc;
        if ((rc = launch_fit_finalize(g, o.chunks_per_block_out, fit, nullptr, st)) != GG_OK) return rc;
        if (total_fit) {
            hipLaunchKernelGGL(k_fit_total, dim3(1), dim3(kTotalThreads), 0, st, fit, (int64_t)g.S, total_fit);
            return check_launch();
        }
        return GG_OK;
    }
    if ((rc = launch_fit(g, x, dtype, fit, &p, st)) != GG_OK) return rc;
    if (total_fit) {
        hipLaunchKernelGGL(k_fit_total, dim3(1), dim3(kTotalThreads), 0, st, fit, (int64_t)g.S, total_fit);
        if ((rc = check_launch()) != GG_OK) return rc;
    }
    QuantOpts o;
    o.rate = rate != nullptr; o.pen = grad != nullptr; o.eg_k = eg_k; o.round_mode = round_mode;
    o.nbins = nbins; o.hist = hist; o.symbols = symbols; o.grad = grad; o.accumulate = accumulate;
    o.rate_out = rate; o.params = g.params();
    o.hist_cleared = with_hist && g.S < kManyUnits;     // the wave-per-unit finalisation clears; the lane-per-unit one does not
    return run_second_sweep(g, x, dtype, o, st);
}

}  // namespace gg

// =============================================================================================
// C ABI
// =============================================================================================
using namespace gg;

extern "C" {

const char *gg_strerror(int code) {
    switch (code) {
        case GG_OK: return "ok";
        case GG_ERR_INVALID_ARG: return "invalid argument";
        case GG_ERR_BAD_DTYPE: return "unsupported dtype";
        case GG_ERR_BAD_SEGMENTS: return "bad segment table";
        case GG_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case GG_ERR_HIP: return "HIP runtime error";
        default: return "unknown error";
    }
}

int gg_workspace_bytes(int64_t n_total, int32_t n_units, int32_t nbins, size_t *bytes_out_host) {
    if (!bytes_out_host || n_total < 0 || n_units < 0 || n_units > kMaxUnits || nbins < 0 || nbins > GG_MAX_BINS)
        return GG_ERR_INVALID_ARG;
    *bytes_out_host = ws_layout(n_total, n_units > 0 ? n_units : 1).total;
    return GG_OK;
}

double gg_init_alpha(int64_t d_in, double shape, double xi) {
    if (d_in <= 0 || !(shape > 0.0) || !(xi > 0.0)) return NAN;
    return sqrt(xi / (double)d_in * exp(lgamma(1.0 / shape) - lgamma(3.0 / shape)));
}

double gg_compression_ratio(double mean_bits, double fl_bits) { return 1.0 - mean_bits / fl_bits; }

static int check_x(const void *x, int dtype, int64_t n) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    if (n < 0) return GG_ERR_INVALID_ARG;
    if (n > 0 && (!x || !aligned16(x))) return GG_ERR_INVALID_ARG;
    return GG_OK;
}

int gg_fit(const void *x_dev, int dtype, int64_t n, gg_fit_t *out_dev, void *ws_dev, size_t ws_bytes, void *stream) {
    int rc = check_x(x_dev, dtype, n);
    if (rc != GG_OK) return rc;
    if (!out_dev || !aligned8(out_dev)) return GG_ERR_INVALID_ARG;
    Geometry g;
    if ((rc = geometry_uniform(1, n, ws_dev, ws_bytes, true, g)) != GG_OK) return rc;
    return launch_fit(g, x_dev, dtype, out_dev, nullptr, (hipStream_t)stream);
}

int gg_fit_segmented(const void *x_dev, int dtype, const int64_t *offsets_host, int32_t S, gg_fit_t *out_dev,
                     void *ws_dev, size_t ws_bytes, void *stream) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    Geometry g;
    int rc = geometry_segmented(offsets_host, S, ws_dev, ws_bytes, g, true);
    if (rc != GG_OK) return rc;
    if ((rc = check_x(x_dev, dtype, g.n_total)) != GG_OK) return rc;
    if (S > 0 && (!out_dev || !aligned8(out_dev))) return GG_ERR_INVALID_ARG;
    if ((rc = upload_geometry(g, (hipStream_t)stream)) != GG_OK) return rc;
    return launch_fit(g, x_dev, dtype, out_dev, nullptr, (hipStream_t)stream);
}

int gg_fit_rows(const void *x_dev, int dtype, int64_t rows, int64_t cols, gg_fit_t *out_dev, gg_fit_t *total_out_dev,
                void *ws_dev, size_t ws_bytes, void *stream) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    Geometry g;
    int rc = geometry_uniform(rows, cols, ws_dev, ws_bytes, true, g);
    if (rc != GG_OK) return rc;
    if ((rc = check_x(x_dev, dtype, g.n_total)) != GG_OK) return rc;
    if (rows > 0 && (!out_dev || !aligned8(out_dev))) return GG_ERR_INVALID_ARG;
    if (total_out_dev && !aligned8(total_out_dev)) return GG_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (rows_take_wave_path(rows, cols)) {
        RowsArgs a{};
        a.rows = rows; a.cols = cols; a.fit = out_dev; a.do_fit = 1;
        a.total_out = total_out_dev; a.wave_sums = g.partials(); a.wave_sums_cap = (int64_t)(g.wl.partials_bytes / sizeof(double2));
        return launch_rows(g, x_dev, dtype, a, 0, GG_FLOOR, false, false, st);
    }
    if ((rc = launch_fit(g, x_dev, dtype, out_dev, nullptr, st)) != GG_OK) return rc;
    if (total_out_dev) {
        hipLaunchKernelGGL(k_fit_total, dim3(1), dim3(kTotalThreads), 0, st, out_dev, rows, total_out_dev);
        return check_launch();
    }
    return GG_OK;
}

int gg_quantize_rate(const void *x_dev, int dtype, int64_t n, float delta, int eg_k, int round_mode, int32_t nbins,
                     uint64_t *hist_dev, int32_t *symbols_dev, gg_rate_t *out_dev, void *ws_dev, size_t ws_bytes,
                     void *stream) {
    int rc = check_x(x_dev, dtype, n);
    if (rc != GG_OK) return rc;
    if (!(delta > 0.f) || !std::isfinite(delta)) return GG_ERR_INVALID_ARG;
    if ((rc = check_rate_args(eg_k, round_mode, nbins, hist_dev, symbols_dev)) != GG_OK) return rc;
    if (!out_dev || !aligned8(out_dev)) return GG_ERR_INVALID_ARG;
    Geometry g;
    if ((rc = geometry_uniform(1, n, ws_dev, ws_bytes, true, g)) != GG_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    PrepArgs p{};
    p.delta_div = 0.f; p.delta_scalar = delta; p.params = g.params(); p.rate = out_dev; p.want_pen = 0;
    if (nbins > 0) { p.hist = hist_dev; p.nbins = nbins; }
    if ((rc = launch_seg_prepare(g, p, st)) != GG_OK) return rc;
    QuantOpts o;
    o.rate = true; o.eg_k = eg_k; o.round_mode = round_mode; o.nbins = nbins; o.hist = hist_dev;
    o.symbols = symbols_dev; o.rate_out = out_dev; o.params = g.params(); o.hist_cleared = nbins > 0;
    return run_second_sweep(g, x_dev, dtype, o, st);
}

int gg_quantize_rate_segmented(const void *x_dev, int dtype, const int64_t *offsets_host, int32_t S,
                               const float *delta_dev, int eg_k, int round_mode, int32_t nbins, uint64_t *hist_dev,
                               int32_t *symbols_dev, gg_rate_t *out_dev, void *ws_dev, size_t ws_bytes, void *stream) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    Geometry g;
    int rc = geometry_segmented(offsets_host, S, ws_dev, ws_bytes, g, true);
    if (rc != GG_OK) return rc;
    if ((rc = check_x(x_dev, dtype, g.n_total)) != GG_OK) return rc;
    if ((rc = check_rate_args(eg_k, round_mode, nbins, hist_dev, symbols_dev)) != GG_OK) return rc;
    if (S > 0 && (!delta_dev || !out_dev || !aligned8(out_dev))) return GG_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if ((rc = upload_geometry(g, st)) != GG_OK) return rc;
    PrepArgs p{};
    p.delta_dev = delta_dev; p.delta_div = 0.f; p.params = g.params(); p.rate = out_dev; p.want_pen = 0;
    if (nbins > 0) { p.hist = hist_dev; p.nbins = nbins; }
    if ((rc = launch_seg_prepare(g, p, st)) != GG_OK) return rc;
    QuantOpts o;
    o.rate = true; o.eg_k = eg_k; o.round_mode = round_mode; o.nbins = nbins; o.hist = hist_dev;
    o.symbols = symbols_dev; o.rate_out = out_dev; o.params = g.params(); o.hist_cleared = nbins > 0 && S > 0;
    return run_second_sweep(g, x_dev, dtype, o, st);
}

int gg_quantize_rate_rows(const void *x_dev, int dtype, int64_t rows, int64_t cols, const float *delta_dev, int eg_k,
                          int round_mode, int32_t *symbols_dev, gg_rate_t *out_dev, void *ws_dev, size_t ws_bytes,
                          void *stream) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    Geometry g;
    int rc = geometry_uniform(rows, cols, ws_dev, ws_bytes, true, g);
    if (rc != GG_OK) return rc;
    if ((rc = check_x(x_dev, dtype, g.n_total)) != GG_OK) return rc;
    if ((rc = check_rate_args(eg_k, round_mode, 0, nullptr, symbols_dev)) != GG_OK) return rc;
    if (rows > 0 && (!delta_dev || !out_dev || !aligned8(out_dev))) return GG_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (rows_take_wave_path(rows, cols)) {
        RowsArgs a{};
        a.rows = rows; a.cols = cols; a.rate = out_dev; a.delta_dev = delta_dev; a.delta_div = 0.f;
        a.symbols = symbols_dev; a.do_fit = 0;
        return launch_rows(g, x_dev, dtype, a, eg_k, round_mode, true, false, st);
    }
    PrepArgs p{};
    p.delta_dev = delta_dev; p.delta_div = 0.f; p.params = g.params(); p.rate = out_dev; p.want_pen = 0;
    if ((rc = launch_seg_prepare(g, p, st)) != GG_OK) return rc;
    QuantOpts o;
    o.rate = true; o.eg_k = eg_k; o.round_mode = round_mode; o.symbols = symbols_dev; o.rate_out = out_dev;
    o.params = g.params();
    return run_second_sweep(g, x_dev, dtype, o, st);
}

int gg_delta_from_fit(const gg_fit_t *fit_dev, int32_t S, float delta_div, float *delta_out_dev, void *stream) {
    if (S < 0 || !(delta_div > 0.f) || !std::isfinite(delta_div)) return GG_ERR_INVALID_ARG;
    if (S == 0) return GG_OK;
    if (!fit_dev || !delta_out_dev) return GG_ERR_INVALID_ARG;
    hipLaunchKernelGGL(k_delta_from_fit, dim3((unsigned)((S + 255) / 256)), dim3(256), 0, (hipStream_t)stream, fit_dev, S,
                       delta_div, delta_out_dev);
    return check_launch();
}

int gg_penalty_grad(const void *w_dev, int dtype, int64_t n, float alpha, float beta, float lambda, float *grad_dev,
                    int accumulate, void *stream) {
    int rc = check_x(w_dev, dtype, n);
    if (rc != GG_OK) return rc;
    if (!(alpha > 0.f) || !std::isfinite(alpha) || !(beta > 0.f) || !std::isfinite(beta) || !std::isfinite(lambda))
        return GG_ERR_INVALID_ARG;
    if (n > 0 && (!grad_dev || !aligned16(grad_dev))) return GG_ERR_INVALID_ARG;
    Geometry g;
    if ((rc = geometry_uniform(1, n, nullptr, 0, false, g)) != GG_OK) return rc;
    QuantOpts o;
    o.pen = true; o.grad = grad_dev; o.accumulate = accumulate ? 1 : 0;
    o.single.inv_alpha = (float)(1.0 / (double)alpha);
    o.single.pen_coef = (float)((double)lambda * (double)beta / (double)alpha);
    o.single.beta_m1 = beta - 1.0f;
    o.single.flags = kSkipRate;
    return run_second_sweep(g, w_dev, dtype, o, (hipStream_t)stream);
}

int gg_penalty_grad_segmented(const void *w_dev, int dtype, const int64_t *offsets_host, int32_t S,
                              const gg_fit_t *fit_dev, float lambda, float *grad_dev, int accumulate, void *ws_dev,
                              size_t ws_bytes, void *stream) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    Geometry g;
    int rc = geometry_segmented(offsets_host, S, ws_dev, ws_bytes, g, true);
    if (rc != GG_OK) return rc;
    if ((rc = check_x(w_dev, dtype, g.n_total)) != GG_OK) return rc;
    if (!std::isfinite(lambda)) return GG_ERR_INVALID_ARG;
    if (S > 0 && !fit_dev) return GG_ERR_INVALID_ARG;
    if (g.n_total > 0 && (!grad_dev || !aligned16(grad_dev))) return GG_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if ((rc = upload_geometry(g, st)) != GG_OK) return rc;
    PrepArgs p{};
    p.fit = fit_dev; p.delta_div = 0.f; p.delta_scalar = 0.f; p.lambda = lambda; p.params = g.params();
    p.rate = nullptr; p.want_pen = 1;
    if ((rc = launch_seg_prepare(g, p, st)) != GG_OK) return rc;
    QuantOpts o;
    o.pen = true; o.grad = grad_dev; o.accumulate = accumulate ? 1 : 0; o.params = g.params();
    return run_second_sweep(g, w_dev, dtype, o, st);
}

int gg_sample(void *out_dev, int dtype, int64_t n, float alpha, float beta, uint64_t seed, uint32_t stream_id,
              uint64_t offset, void *stream) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    if (n < 0 || !(alpha >= 0.f) || !std::isfinite(alpha) || !(beta >= (float)GG_BETA_MIN) || !(beta <= (float)GG_BETA_MAX))
        return GG_ERR_INVALID_ARG;
    if (n == 0) return GG_OK;
    if (!out_dev || !aligned16(out_dev)) return GG_ERR_INVALID_ARG;
    SampleArgs s{};
    const double a = 1.0 / (double)beta;
    s.boost = a < 1.0;
    const double d = (s.boost ? a + 1.0 : a) - 1.0 / 3.0;
    s.alpha = alpha; s.a = (float)a; s.d = (float)d; s.c = (float)(1.0 / sqrt(9.0 * d));
    s.key0 = (uint32_t)seed; s.key1 = (uint32_t)(seed >> 32); s.stream_id = stream_id; s.offset = offset; s.n = n;
    int64_t blocks = (n + (int64_t)kWaves * kSampleSpan - 1) / ((int64_t)kWaves * kSampleSpan);
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipStream_t st = (hipStream_t)stream;
    if (dtype == GG_F32) hipLaunchKernelGGL(k_sample<float>, dim3((unsigned)blocks), dim3(kBlock), 0, st, (float *)out_dev, s);
    else hipLaunchKernelGGL(k_sample<bf16_t>, dim3((unsigned)blocks), dim3(kBlock), 0, st, (bf16_t *)out_dev, s);
    return check_launch();
}

int gg_philox_words(uint32_t *out_dev, int64_t n, uint64_t seed, uint32_t stream_id, uint64_t offset, uint32_t attempt,
                    void *stream) {
    if (n < 0) return GG_ERR_INVALID_ARG;
    if (n == 0) return GG_OK;
    if (!out_dev || !aligned16(out_dev)) return GG_ERR_INVALID_ARG;
    int64_t blocks = (n + kBlock - 1) / kBlock;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(k_philox_words, dim3((unsigned)blocks), dim3(kBlock), 0, (hipStream_t)stream, out_dev, n,
                       (uint32_t)seed, (uint32_t)(seed >> 32), stream_id, offset, attempt);
    return check_launch();
}

static int check_fused(int eg_k, int round_mode, int32_t nbins, uint64_t *hist, int32_t *symbols, float delta_div,
                       const float *delta_dev, float lambda, float *grad, gg_fit_t *fit, gg_rate_t *rate, int32_t S,
                       int64_t n_total) {
    if (S > 0 && (!fit || !aligned8(fit))) return GG_ERR_INVALID_ARG;
    // the order and the rounding mode are checked whether or not a rate is asked for: the launchers shift by eg_k
    if (eg_k < 0 || eg_k > GG_MAX_EG_K) return GG_ERR_INVALID_ARG;
    if (round_mode != GG_FLOOR && round_mode != GG_NEAREST_EVEN) return GG_ERR_INVALID_ARG;
    if (rate) {
        int rc = check_rate_args(eg_k, round_mode, nbins, hist, symbols);
        if (rc != GG_OK) return rc;
        if (!aligned8(rate)) return GG_ERR_INVALID_ARG;
        if (!(delta_div > 0.f) && !delta_dev && S > 0) return GG_ERR_INVALID_ARG;
        if (delta_div > 0.f && !std::isfinite(delta_div)) return GG_ERR_INVALID_ARG;
    }
    if (grad && (!aligned16(grad) || !std::isfinite(lambda))) return GG_ERR_INVALID_ARG;
    (void)n_total;
    return GG_OK;
}

int gg_fused_segmented(const void *x_dev, int dtype, const int64_t *offsets_host, int32_t S, float delta_div,
                       const float *delta_dev, int eg_k, int round_mode, int32_t nbins, uint64_t *hist_dev,
                       int32_t *symbols_dev, float lambda, float *grad_dev, int accumulate, gg_fit_t *fit_dev,
                       gg_rate_t *rate_dev, void *ws_dev, size_t ws_bytes, void *stream) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    Geometry g;
    int rc = geometry_segmented(offsets_host, S, ws_dev, ws_bytes, g, true);
    if (rc != GG_OK) return rc;
    if ((rc = check_x(x_dev, dtype, g.n_total)) != GG_OK) return rc;
    if ((rc = check_fused(eg_k, round_mode, nbins, hist_dev, symbols_dev, delta_div, delta_dev, lambda, grad_dev, fit_dev,
                          rate_dev, S, g.n_total)) != GG_OK)
        return rc;
    return fused_common(g, x_dev, dtype, delta_div, delta_dev, eg_k, round_mode, nbins, hist_dev, symbols_dev, lambda,
                        grad_dev, accumulate ? 1 : 0, fit_dev, nullptr, rate_dev, (hipStream_t)stream);
}

int gg_fused_rows(const void *x_dev, int dtype, int64_t rows, int64_t cols, float delta_div, const float *delta_dev,
                  int eg_k, int round_mode, int32_t *symbols_dev, float lambda, float *grad_dev, int accumulate,
                  gg_fit_t *fit_dev, gg_fit_t *total_fit_dev, gg_rate_t *rate_dev, void *ws_dev, size_t ws_bytes,
                  void *stream) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    Geometry g;
    int rc = geometry_uniform(rows, cols, ws_dev, ws_bytes, true, g);
    if (rc != GG_OK) return rc;
    if ((rc = check_x(x_dev, dtype, g.n_total)) != GG_OK) return rc;
    if ((rc = check_fused(eg_k, round_mode, 0, nullptr, symbols_dev, delta_div, delta_dev, lambda, grad_dev, fit_dev,
                          rate_dev, g.S, g.n_total)) != GG_OK)
        return rc;
    if (total_fit_dev && !aligned8(total_fit_dev)) return GG_ERR_INVALID_ARG;
    if (rows_take_wave_path(rows, cols)) {
        hipStream_t st = (hipStream_t)stream;
        RowsArgs a{};
        a.rows = rows; a.cols = cols; a.fit = fit_dev; a.rate = rate_dev; a.delta_dev = delta_dev; a.delta_div = delta_div;
        a.lambda = lambda; a.symbols = rate_dev ? symbols_dev : nullptr; a.grad = grad_dev; a.accumulate = accumulate ? 1 : 0;
        a.do_fit = 1;
        a.total_out = total_fit_dev; a.wave_sums = g.partials(); a.wave_sums_cap = (int64_t)(g.wl.partials_bytes / sizeof(double2));
        return launch_rows(g, x_dev, dtype, a, eg_k, round_mode, rate_dev != nullptr, grad_dev != nullptr, st);
    }
    return fused_common(g, x_dev, dtype, delta_div, delta_dev, eg_k, round_mode, 0, nullptr, symbols_dev, lambda, grad_dev,
                        accumulate ? 1 : 0, fit_dev, total_fit_dev, rate_dev, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// The pass for callers that cannot allocate and have no workspace to hand over (code under graph
// capture, serving loops, harnesses that forbid hipMalloc): the workspace of gg_fused_segmented lives in a
// file-scope device array.  Every GPU holds its own copy of the array at its own address; host code never
// uses the array's name as an address, only what hipGetSymbolAddress returned for the current device.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[GG_NOALLOC_SCRATCH_BYTES];

static std::atomic<void *> g_scratch_ptr[kMaxDevices];   // per device, set on the first call made with that device current

// device address of `scratch` on the current device, or nullptr when it cannot be had
static void *scratch_for_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    void *q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) { (void)hipGetLastError(); return nullptr; }
    g_scratch_ptr[dev].store(q, std::memory_order_release);   // two threads racing here store the same address
    return q;
}

int gg_fused_segmented_noalloc(const void *x_dev, int dtype, const int64_t *offsets_host, int32_t S, float delta_div,
                               const float *delta_dev, int eg_k, int round_mode, int32_t nbins, uint64_t *hist_dev,
                               int32_t *symbols_dev, float lambda, float *grad_dev, int accumulate, gg_fit_t *fit_dev,
                               gg_rate_t *rate_dev, void *stream) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    // sizes first, against the fixed capacity, before anything touches the device
    Geometry g;
    int rc = geometry_segmented(offsets_host, S, reinterpret_cast<void *>(uintptr_t(256)), GG_NOALLOC_SCRATCH_BYTES, g, true);
    if (rc != GG_OK) return rc;    // GG_ERR_WORKSPACE: the bucket needs more scratch than the library holds
    if ((rc = check_x(x_dev, dtype, g.n_total)) != GG_OK) return rc;
    if ((rc = check_fused(eg_k, round_mode, nbins, hist_dev, symbols_dev, delta_div, delta_dev, lambda, grad_dev, fit_dev,
                          rate_dev, S, g.n_total)) != GG_OK)
        return rc;
    void *ws = scratch_for_current_device();
    if (!ws) return GG_ERR_HIP;
    if ((rc = geometry_segmented(offsets_host, S, ws, GG_NOALLOC_SCRATCH_BYTES, g, true)) != GG_OK) return rc;
    // nothing in the workspace has to start at zero: every slot a kernel reads was written earlier in this call
    return fused_common(g, x_dev, dtype, delta_div, delta_dev, eg_k, round_mode, nbins, hist_dev, symbols_dev, lambda,
                        grad_dev, accumulate ? 1 : 0, fit_dev, nullptr, rate_dev, (hipStream_t)stream);
}

}  // extern "C"
