// gg_train.hip -- the pieces of the paper's training algorithms that sit next to the tensor pass:
//   * gradient of the mean Exp-Golomb length through the straight-through quantiser (ACT backward,
//     Sec. 4.2; the dR/dG of Sec. 4.3),
//   * the element-wise GCT update of Algorithm 2 (secant curvature, equivalent gradient, weight step),
//   * an order-k Exp-Golomb bit-stream encoder / decoder whose stream length is exactly the bit count
//     the rate sweep reports,
//   * the Huffman mean code length (the HM column of the paper's tables) from a histogram (host).

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <algorithm>
#include <cmath>
#include <vector>

#include "../../include/gg.h"
#include "gg_device.h"
#include "gg_geometry.h"

namespace gg {

constexpr int32_t kQLimT = 1 << 30;

// u = Map(floor(x * inv_delta)) with the quantiser's conventions (NaN -> 0, clamp to +-2^30)
__device__ __forceinline__ uint32_t map_floor(float x, float inv_delta) {
    const float t = x * inv_delta;
    int32_t m;
    asm("v_cvt_i32_f32 %0, %1" : "=v"(m) : "v"(ceilf(-t)));   // hardware conversion: NaN -> 0, saturating
    m = m < -kQLimT ? -kQLimT : (m > kQLimT ? kQLimT : m);
    return ((uint32_t)m << 1) ^ (uint32_t)(m >> 31);
}

// dR/dx = coef * sign(x) / (u + 2^k), coef = scale * 4 inv_delta / (N ln 2)
__device__ __forceinline__ float rate_slope(float x, float inv_delta, float coef, uint32_t eg_add) {
    const uint32_t u = map_floor(x, inv_delta);
    const float d = coef / (float)(u + eg_add);
    return x > 0.f ? d : (x < 0.f ? -d : 0.f);
}

struct UnitCoef { float inv_delta, coef; };   // per unit: 1/Delta and 4 (1/Delta) / (N ln 2) (times a scale)

struct SlopeArgs {
    const UnitCoef *units;   // device per-unit parameters or nullptr -> `single`
    UnitCoef single;
    uint32_t eg_add;
    int64_t n_chunks;
    int32_t chunks_per_block;
};

// ---------------------------------------------------------------------------------------------
// rate gradient
// ---------------------------------------------------------------------------------------------
struct RateGradBody {
    float inv_delta, coef; uint32_t eg_add;
    float *grad; int accumulate;
    template <int W>
    __device__ __forceinline__ void vec(const float (&v)[W], int64_t idx) {
        static_assert(W == 4, "four elements per lane");
        gg_f4 g = {rate_slope(v[0], inv_delta, coef, eg_add), rate_slope(v[1], inv_delta, coef, eg_add),
                   rate_slope(v[2], inv_delta, coef, eg_add), rate_slope(v[3], inv_delta, coef, eg_add)};
        gg_f4 *dst = reinterpret_cast<gg_f4 *>(grad + idx);
        if (accumulate) g += __builtin_nontemporal_load(dst);
        __builtin_nontemporal_store(g, dst);
    }
    __device__ __forceinline__ void one(float v, int64_t idx) {
        const float g = rate_slope(v, inv_delta, coef, eg_add);
        grad[idx] = accumulate ? grad[idx] + g : g;
    }
};

template <typename E>
__global__ __launch_bounds__(kBlock) void k_rate_grad(SegView sv, const typename E::type *__restrict__ x, SlopeArgs a,
                                                      float *__restrict__ grad, int accumulate) {
    const int64_t first = (int64_t)blockIdx.x * a.chunks_per_block;
    int64_t last = first + a.chunks_per_block;
    if (last > a.n_chunks) last = a.n_chunks;
    if (first >= last) return;
    RateGradBody body;
    body.eg_add = a.eg_add; body.grad = grad; body.accumulate = accumulate;
    int seg = -1;
    RunCursor cur;
    for (cur.init(sv, first, last); cur.valid(); cur.next(sv)) {
        if (cur.L.seg != seg) {
            seg = cur.L.seg;
            const UnitCoef uc = a.units ? a.units[seg] : a.single;
            body.inv_delta = uc.inv_delta; body.coef = uc.coef;
        }
        process_chunk<E, 8>(x, cur.L.start, cur.L.len, body);
    }
}

// ---------------------------------------------------------------------------------------------
// GCT update (Algorithm 2): per parameter
//   h    = (1/eta) (1 - g / (ghat_prev + eps)) * 1[t >= 2]
//   ghat = g + lambda * dR/dg * h          (stored over ghat_prev)
//   w   <- w - eta * ghat
// ---------------------------------------------------------------------------------------------
struct GctBody {
    float inv_delta, coef; uint32_t eg_add;
    float eta, inv_eta, lambda, eps; int first_step;
    float *w, *ghat_prev;

    __device__ __forceinline__ float step(float g, float gp, float &wv) const {
        const float dr = rate_slope(g, inv_delta, coef, eg_add);
        const float h = first_step ? 0.f : inv_eta * (1.0f - g / (gp + eps));
        const float ghat = __builtin_fmaf(lambda * dr, h, g);
        wv = __builtin_fmaf(-eta, ghat, wv);
        return ghat;
    }
    template <int W>
    __device__ __forceinline__ void vec(const float (&v)[W], int64_t idx) {
        static_assert(W == 4, "four elements per lane");
        gg_f4 *pw = reinterpret_cast<gg_f4 *>(w + idx), *pg = reinterpret_cast<gg_f4 *>(ghat_prev + idx);
        const gg_f4 wv = __builtin_nontemporal_load(pw);
        const gg_f4 gp = __builtin_nontemporal_load(pg);
        float w0 = wv.x, w1 = wv.y, w2 = wv.z, w3 = wv.w;
        const gg_f4 gh = {step(v[0], gp.x, w0), step(v[1], gp.y, w1), step(v[2], gp.z, w2), step(v[3], gp.w, w3)};
        const gg_f4 wn = {w0, w1, w2, w3};
        __builtin_nontemporal_store(gh, pg);
        __builtin_nontemporal_store(wn, pw);
    }
    __device__ __forceinline__ void one(float v, int64_t idx) {
        float wv = w[idx];
        ghat_prev[idx] = step(v, ghat_prev[idx], wv);
        w[idx] = wv;
    }
};

struct GctScalars { float eta, inv_eta, lambda, eps; int first_step; };

__global__ __launch_bounds__(kBlock) void k_gct_update(SegView sv, const float *__restrict__ g, SlopeArgs a, GctScalars sc,
                                                       float *__restrict__ w, float *__restrict__ ghat_prev) {
    const int64_t first = (int64_t)blockIdx.x * a.chunks_per_block;
    int64_t last = first + a.chunks_per_block;
    if (last > a.n_chunks) last = a.n_chunks;
    if (first >= last) return;
    GctBody body;
    body.eg_add = a.eg_add; body.eta = sc.eta; body.inv_eta = sc.inv_eta; body.lambda = sc.lambda; body.eps = sc.eps;
    body.first_step = sc.first_step; body.w = w; body.ghat_prev = ghat_prev;
    int seg = -1;
    RunCursor cur;
    for (cur.init(sv, first, last); cur.valid(); cur.next(sv)) {
        if (cur.L.seg != seg) {
            seg = cur.L.seg;
            const UnitCoef uc = a.units ? a.units[seg] : a.single;
            body.inv_delta = uc.inv_delta; body.coef = uc.coef;
        }
        process_chunk<Elem<float>, 4>(g, cur.L.start, cur.L.len, body);
    }
}

// per-unit 1/Delta and slope coefficient from device steps; a unit without a usable step gets 0 (no rate term)
__global__ void k_unit_coef(SegView sv, const float *__restrict__ delta_dev, float scale, UnitCoef *__restrict__ out) {
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= sv.S) return;
    const float d = delta_dev[s];
    const int64_t n = unit_len(sv, s);
    UnitCoef uc{0.f, 0.f};
    if (d > 0.f && isfinite(d) && n > 0) {
        uc.inv_delta = (float)(1.0 / (double)d);
        uc.coef = (float)((double)scale * 4.0 * (double)uc.inv_delta / ((double)n * 0.69314718055994530942));
    }
    out[s] = uc;
}

// ---------------------------------------------------------------------------------------------
// Exp-Golomb-k bit stream.  Symbol i contributes (L_i - 1 - k) zero bits and then the L_i bits of
// v_i = u_i + 2^k, most significant bit first; bytes are filled from their most significant bit.
// Blocks of kEgBlock symbols: (1) bits per block, (2) exclusive scan, (3) each block assembles its
// span in LDS with bit-wise ORs and copies whole 32-bit words out; the two words a span shares with
// its neighbours are OR-ed into the (pre-cleared) stream atomically.
// ---------------------------------------------------------------------------------------------
constexpr int kEgBlock = 2048;                      // symbols per block (8 per lane)
constexpr int kEgPerLane = kEgBlock / kBlock;
constexpr int kEgLdsWords = kEgBlock * 2 + 2;       // <= 63 bits per symbol, plus the alignment slack

__device__ __forceinline__ uint32_t map_q(int32_t q) {
    const int32_t m = -q;
    return ((uint32_t)m << 1) ^ (uint32_t)(m >> 31);
}

__global__ __launch_bounds__(kBlock) void k_eg_block_bits(const int32_t *__restrict__ q, int64_t n, int eg_k,
                                                          uint64_t *__restrict__ block_bits) {
    __shared__ uint32_t red[kWaves];
    const int64_t base = (int64_t)blockIdx.x * kEgBlock;
    uint32_t bits = 0;
#pragma unroll
    for (int j = 0; j < kEgPerLane; ++j) {
        const int64_t i = base + j * kBlock + threadIdx.x;
        if (i < n) {
            const uint32_t v = map_q(q[i]) + (1u << eg_k);
            bits += 63u - (uint32_t)eg_k - 2u * (uint32_t)__builtin_clz(v);
        }
    }
    const uint32_t total = block_reduce(bits, OpAdd(), red);
    if (threadIdx.x == 0) block_bits[blockIdx.x] = total;
}

// exclusive scan of block_bits[0..nb) in place, total to block_bits[nb] and *total_out; one workgroup
__global__ __launch_bounds__(1024) void k_eg_scan(uint64_t *__restrict__ block_bits, int64_t nb, uint64_t *__restrict__ total_out) {
    __shared__ uint64_t part[1024];
    const int tid = threadIdx.x;
    const int64_t per = (nb + 1023) / 1024;
    const int64_t lo = tid * per, hi = lo + per < nb ? lo + per : nb;
    uint64_t s = 0;
    for (int64_t i = lo; i < hi; ++i) s += block_bits[i];
    part[tid] = s;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {      // Hillis-Steele inclusive scan over the 1024 partials
        const uint64_t add = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    uint64_t run = tid ? part[tid - 1] : 0;
    for (int64_t i = lo; i < hi; ++i) { const uint64_t b = block_bits[i]; block_bits[i] = run; run += b; }
    if (tid == 1023) { block_bits[nb] = part[1023]; if (total_out) *total_out = part[1023]; }
}

__global__ __launch_bounds__(kBlock) void k_eg_encode(const int32_t *__restrict__ q, int64_t n, int eg_k,
                                                      const uint64_t *__restrict__ block_off, uint32_t *__restrict__ stream,
                                                      uint64_t capacity_bits) {
    __shared__ uint32_t buf[kEgLdsWords];
    __shared__ uint32_t wave_tot[kWaves];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t base = (int64_t)blockIdx.x * kEgBlock;
    const uint64_t off0 = block_off[blockIdx.x], off1 = block_off[blockIdx.x + 1];
    if (off1 > capacity_bits) return;               // stream too small: nothing of this block is written
    for (int i = tid; i < kEgLdsWords; i += kBlock) buf[i] = 0;

    // lane owns kEgPerLane consecutive symbols, so positions follow from one scan of lane totals
    uint32_t v[kEgPerLane], len[kEgPerLane], mine = 0;
#pragma unroll
    for (int j = 0; j < kEgPerLane; ++j) {
        const int64_t i = base + (int64_t)tid * kEgPerLane + j;
        v[j] = 0; len[j] = 0;
        if (i < n) {
            v[j] = map_q(q[i]) + (1u << eg_k);
            len[j] = 63u - (uint32_t)eg_k - 2u * (uint32_t)__builtin_clz(v[j]);
        }
        mine += len[j];
    }
    uint32_t incl = mine;                           // inclusive scan across the wave
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(incl, d, 64);
        if (lane >= d) incl += t;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t pos = incl - mine;
    for (int w = 0; w < wave; ++w) pos += wave_tot[w];
    pos += (uint32_t)(off0 & 31u);                  // LDS bit 0 is the stream's word boundary below off0
#pragma unroll
    for (int j = 0; j < kEgPerLane; ++j) {
        if (len[j]) {
            const uint32_t nb = 32u - (uint32_t)__builtin_clz(v[j]);   // significant bits of v
            const uint32_t p = pos + (len[j] - nb);                     // after the zero prefix
            // place nb bits so that the first lands at stream bit p (bit 31 of a word is the earliest)
            const uint64_t window = (uint64_t)v[j] << (64u - nb - (p & 31u));
            atomicOr(&buf[p >> 5], (uint32_t)(window >> 32));
            const uint32_t lo = (uint32_t)window;
            if (lo) atomicOr(&buf[(p >> 5) + 1], lo);
            pos += len[j];
        }
    }
    __syncthreads();
    const uint64_t w0 = off0 >> 5;
    const uint32_t span_bits = (uint32_t)(off0 & 31u) + (uint32_t)(off1 - off0);
    const uint32_t nwords = (span_bits + 31u) >> 5;
    for (uint32_t i = tid; i < nwords; i += kBlock) {
        const uint32_t word = __builtin_bswap32(buf[i]);     // most significant byte first in memory
        if (word == 0 && (i == 0 || i == nwords - 1)) continue;
        if (i == 0 || i == nwords - 1) atomicOr(&stream[w0 + i], word);
        else stream[w0 + i] = word;
    }
}

__global__ void k_fill_u32(uint32_t *p, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// one lane decodes one block of kEgBlock symbols from its indexed bit offset
__global__ __launch_bounds__(64) void k_eg_decode(const uint8_t *__restrict__ stream, const uint64_t *__restrict__ block_off,
                                                  int64_t n, int64_t nb, int eg_k, int32_t *__restrict__ q) {
    const int64_t b = (int64_t)blockIdx.x * 64 + threadIdx.x;
    if (b >= nb) return;
    uint64_t pos = block_off[b];
    const uint64_t end = block_off[b + 1];
    const int64_t first = b * kEgBlock;
    const int64_t cnt = n - first < kEgBlock ? n - first : kEgBlock;
    auto bit = [&](uint64_t p) -> uint32_t { return (stream[p >> 3] >> (7u - (uint32_t)(p & 7u))) & 1u; };
    for (int64_t i = 0; i < cnt; ++i) {
        int zeros = 0;
        while (pos < end && !bit(pos)) { ++zeros; ++pos; }
        const int L = zeros + eg_k + 1;
        uint64_t v = 0;
        for (int j = 0; j < L && pos < end; ++j) { v = (v << 1) | bit(pos); ++pos; }
        const uint32_t u = (uint32_t)(v - (1ull << eg_k));
        // inverse Map: odd -> positive (u+1)/2, even -> negative -u/2
        q[first + i] = (u & 1u) ? (int32_t)((u + 1u) >> 1) : -(int32_t)(u >> 1);
    }
}

// ---------------------------------------------------------------------------------------------
// host
// ---------------------------------------------------------------------------------------------
static SlopeArgs slope_args(const Geometry &g, int eg_k, int blocks_per_cu, unsigned &blocks_out) {
    SlopeArgs a{};
    a.eg_add = 1u << eg_k;
    a.n_chunks = g.n_chunks;
    const RunSplit rs = split_runs(g.n_chunks, blocks_per_cu);
    a.chunks_per_block = rs.chunks_per_block;
    blocks_out = (unsigned)rs.blocks;
    return a;
}

static UnitCoef host_coef(float delta, int64_t n_rate, float scale) {
    UnitCoef uc;
    uc.inv_delta = (float)(1.0 / (double)delta);
    uc.coef = (float)((double)scale * 4.0 * (double)uc.inv_delta / ((double)n_rate * 0.69314718055994530942));
    return uc;
}

}  // namespace gg

using namespace gg;

extern "C" {

int gg_rate_grad(const void *x_dev, int dtype, int64_t n, float delta, int eg_k, int64_t n_rate, float scale,
                 float *grad_dev, int accumulate, void *stream) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    if (n < 0 || n_rate <= 0 || !(delta > 0.f) || !std::isfinite(delta) || !std::isfinite(scale) || eg_k < 0 ||
        eg_k > GG_MAX_EG_K)
        return GG_ERR_INVALID_ARG;
    if (n == 0) return GG_OK;
    if (!x_dev || !aligned16(x_dev) || !grad_dev || !aligned16(grad_dev)) return GG_ERR_INVALID_ARG;
    Geometry g;
    int rc = geometry_uniform(1, n, nullptr, 0, false, g);
    if (rc != GG_OK) return rc;
    unsigned blocks;
    SlopeArgs a = slope_args(g, eg_k, 8, blocks);
    a.single = host_coef(delta, n_rate, scale);
    hipStream_t st = (hipStream_t)stream;
    if (dtype == GG_F32)
        hipLaunchKernelGGL(k_rate_grad<Elem<float>>, dim3(blocks), dim3(kBlock), 0, st, g.sv, (const float *)x_dev, a, grad_dev,
                           accumulate ? 1 : 0);
    else
        hipLaunchKernelGGL(k_rate_grad<ElemBf16x4>, dim3(blocks), dim3(kBlock), 0, st, g.sv, (const bf16_t *)x_dev, a, grad_dev,
                           accumulate ? 1 : 0);
    return check_launch();
}

static int check_gct(float *w, const float *g, float *gp, int64_t n, float eta, float lambda, float eps, int eg_k) {
    if (n < 0 || !(eta > 0.f) || !std::isfinite(eta) || !std::isfinite(lambda) || !std::isfinite(eps) || eg_k < 0 ||
        eg_k > GG_MAX_EG_K)
        return GG_ERR_INVALID_ARG;
    if (n > 0 && (!w || !g || !gp || !aligned16(w) || !aligned16(g) || !aligned16(gp))) return GG_ERR_INVALID_ARG;
    return GG_OK;
}

int gg_gct_update(float *w_dev, const float *g_dev, float *ghat_prev_dev, int64_t n, float eta, float lambda, float eps,
                  float delta, int eg_k, int64_t n_rate, int first_step, void *stream) {
    int rc = check_gct(w_dev, g_dev, ghat_prev_dev, n, eta, lambda, eps, eg_k);
    if (rc != GG_OK) return rc;
    if (n_rate <= 0 || !(delta > 0.f) || !std::isfinite(delta)) return GG_ERR_INVALID_ARG;
    if (n == 0) return GG_OK;
    Geometry g;
    if ((rc = geometry_uniform(1, n, nullptr, 0, false, g)) != GG_OK) return rc;
    unsigned blocks;
    SlopeArgs a = slope_args(g, eg_k, 8, blocks);
    a.single = host_coef(delta, n_rate, 1.0f);
    GctScalars sc{eta, (float)(1.0 / (double)eta), lambda, eps, first_step ? 1 : 0};
    hipLaunchKernelGGL(k_gct_update, dim3(blocks), dim3(kBlock), 0, (hipStream_t)stream, g.sv, g_dev, a, sc, w_dev,
                       ghat_prev_dev);
    return check_launch();
}

int gg_gct_update_segmented(float *w_dev, const float *g_dev, float *ghat_prev_dev, const int64_t *offsets_host, int32_t S,
                            const float *delta_dev, float eta, float lambda, float eps, int eg_k, int first_step,
                            void *ws_dev, size_t ws_bytes, void *stream) {
    Geometry g;
    int rc = geometry_segmented(offsets_host, S, ws_dev, ws_bytes, g);
    if (rc != GG_OK) return rc;
    if ((rc = check_gct(w_dev, g_dev, ghat_prev_dev, g.n_total, eta, lambda, eps, eg_k)) != GG_OK) return rc;
    if (S > 0 && !delta_dev) return GG_ERR_INVALID_ARG;
    if (g.n_chunks == 0) return GG_OK;
    hipStream_t st = (hipStream_t)stream;
    if ((rc = upload_geometry(g, st)) != GG_OK) return rc;
    UnitCoef *units = reinterpret_cast<UnitCoef *>(g.params());   // the per-unit parameter area of the workspace
    hipLaunchKernelGGL(k_unit_coef, dim3((unsigned)((S + 255) / 256)), dim3(256), 0, st, g.sv, delta_dev, 1.0f, units);
    if ((rc = check_launch()) != GG_OK) return rc;
    unsigned blocks;
    SlopeArgs a = slope_args(g, eg_k, 8, blocks);
    a.units = units;
    GctScalars sc{eta, (float)(1.0 / (double)eta), lambda, eps, first_step ? 1 : 0};
    hipLaunchKernelGGL(k_gct_update, dim3(blocks), dim3(kBlock), 0, st, g.sv, g_dev, a, sc, w_dev, ghat_prev_dev);
    return check_launch();
}

int gg_eg_workspace_bytes(int64_t n, size_t *bytes_out_host) {
    if (!bytes_out_host || n < 0) return GG_ERR_INVALID_ARG;
    *bytes_out_host = (size_t)((n + kEgBlock - 1) / kEgBlock + 1) * sizeof(uint64_t);
    return GG_OK;
}

int gg_eg_encode(const int32_t *symbols_dev, int64_t n, int eg_k, uint8_t *stream_dev, uint64_t stream_bytes,
                 uint64_t *block_offsets_dev, uint64_t *total_bits_dev, void *stream) {
    if (n < 0 || eg_k < 0 || eg_k > GG_MAX_EG_K || (stream_bytes & 3u)) return GG_ERR_INVALID_ARG;
    if (!block_offsets_dev || !aligned8(block_offsets_dev)) return GG_ERR_WORKSPACE;
    if (total_bits_dev && !aligned8(total_bits_dev)) return GG_ERR_INVALID_ARG;
    if (stream_bytes && (!stream_dev || (reinterpret_cast<uintptr_t>(stream_dev) & 3u))) return GG_ERR_INVALID_ARG;
    if (n > 0 && !symbols_dev) return GG_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int64_t nb = (n + kEgBlock - 1) / kEgBlock;
    if (nb > 2147483647LL) return GG_ERR_INVALID_ARG;
    int rc;
    if (stream_bytes) {
        const int64_t words = (int64_t)(stream_bytes / 4);
        int64_t fb = (words + 255) / 256;
        if (fb > 8192) fb = 8192;
        hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)fb), dim3(256), 0, st, reinterpret_cast<uint32_t *>(stream_dev), words);
        if ((rc = check_launch()) != GG_OK) return rc;
    }
    if (nb > 0) {
        hipLaunchKernelGGL(k_eg_block_bits, dim3((unsigned)nb), dim3(kBlock), 0, st, symbols_dev, n, eg_k, block_offsets_dev);
        if ((rc = check_launch()) != GG_OK) return rc;
    }
    hipLaunchKernelGGL(k_eg_scan, dim3(1), dim3(1024), 0, st, block_offsets_dev, nb, total_bits_dev);
    if ((rc = check_launch()) != GG_OK) return rc;
    if (nb > 0) {
        hipLaunchKernelGGL(k_eg_encode, dim3((unsigned)nb), dim3(kBlock), 0, st, symbols_dev, n, eg_k, block_offsets_dev,
                           reinterpret_cast<uint32_t *>(stream_dev), stream_bytes * 8ull);
        if ((rc = check_launch()) != GG_OK) return rc;
    }
    return GG_OK;
}

int gg_eg_decode(const uint8_t *stream_dev, const uint64_t *block_offsets_dev, int64_t n, int eg_k, int32_t *symbols_dev,
                 void *stream) {
    if (n < 0 || eg_k < 0 || eg_k > GG_MAX_EG_K) return GG_ERR_INVALID_ARG;
    if (n == 0) return GG_OK;
    if (!stream_dev || !block_offsets_dev || !symbols_dev) return GG_ERR_INVALID_ARG;
    const int64_t nb = (n + kEgBlock - 1) / kEgBlock;
    hipLaunchKernelGGL(k_eg_decode, dim3((unsigned)((nb + 63) / 64)), dim3(64), 0, (hipStream_t)stream, stream_dev,
                       block_offsets_dev, n, nb, eg_k, symbols_dev);
    return check_launch();
}

int gg_huffman_mean_bits(const uint64_t *hist_host, int32_t nbins, double *mean_bits_out_host) {
    if (!hist_host || nbins <= 0 || !mean_bits_out_host) return GG_ERR_INVALID_ARG;
    std::vector<uint64_t> leaves;
    uint64_t total = 0;
    for (int32_t b = 0; b < nbins; ++b)
        if (hist_host[b]) { leaves.push_back(hist_host[b]); total += hist_host[b]; }
    if (leaves.empty()) { *mean_bits_out_host = 0.0; return GG_OK; }
    if (leaves.size() == 1) { *mean_bits_out_host = 1.0; return GG_OK; }
    // two-queue construction: sorted leaves and a FIFO of merged nodes (whose weights come out sorted);
    // the mean length is the sum of all merged weights over the symbol count
    std::sort(leaves.begin(), leaves.end());
    std::vector<uint64_t> merged;
    merged.reserve(leaves.size());
    size_t li = 0, mi = 0;
    long double coded = 0.0L;
    auto take = [&]() {
        if (li < leaves.size() && (mi >= merged.size() || leaves[li] <= merged[mi])) return leaves[li++];
        return merged[mi++];
    };
    for (size_t step = 0; step + 1 < leaves.size(); ++step) {
        const uint64_t a = take(), b = take();
        merged.push_back(a + b);
        coded += (long double)(a + b);
    }
    *mean_bits_out_host = (double)(coded / (long double)total);
    return GG_OK;
}

}  // extern "C"
