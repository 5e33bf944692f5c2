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
    int32_t parts;           // blocks that share one chunk (the grid has n_chunks * parts blocks)
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
    const int64_t chunk = blockIdx.x / a.parts;
    if (chunk >= a.n_chunks) return;
    const ChunkLoc L = locate(sv, chunk);
    int64_t start; int len;
    if (!chunk_part(L.start, L.len, (int)(blockIdx.x - chunk * a.parts), a.parts, start, len)) return;
    RateGradBody body;
    body.eg_add = a.eg_add; body.grad = grad; body.accumulate = accumulate;
    const UnitCoef uc = a.units ? a.units[L.seg] : a.single;
    body.inv_delta = uc.inv_delta; body.coef = uc.coef;
    process_chunk<E, 4>(x, start, len, body);
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
    const int64_t chunk = blockIdx.x / a.parts;
    if (chunk >= a.n_chunks) return;
    const ChunkLoc L = locate(sv, chunk);
    int64_t start; int len;
    if (!chunk_part(L.start, L.len, (int)(blockIdx.x - chunk * a.parts), a.parts, start, len)) return;
    GctBody body;
    body.eg_add = a.eg_add; body.eta = sc.eta; body.inv_eta = sc.inv_eta; body.lambda = sc.lambda; body.eps = sc.eps;
    body.first_step = sc.first_step; body.w = w; body.ghat_prev = ghat_prev;
    const UnitCoef uc = a.units ? a.units[L.seg] : a.single;
    body.inv_delta = uc.inv_delta; body.coef = uc.coef;
    process_chunk<Elem<float>, 4>(g, start, len, body);
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
// Packing tiles of kEgBlock symbols; the decoding index has one entry per GG_EG_TILE symbols:
//   (1) bits per tile (one wave per tile),
//   (2) exclusive scan of the tile sizes,
//   (3) each tile's span is assembled in LDS with bit-wise ORs and copied out as whole 32-bit words.  Every
//       stream word has one writer: a word shared by two tiles of one workgroup is carried from the first
//       to the second in LDS; a word shared by two workgroups is written by the earlier one, which packs
//       the first symbols of the later one's tile into it as well.
// ---------------------------------------------------------------------------------------------
constexpr int kEgBlock = 2048;                      // symbols per packing tile (8 per lane in the packing kernel)
constexpr int kEgPerLane = kEgBlock / kBlock;
constexpr int kEgSubTiles = kEgBlock / GG_EG_TILE;  // index entries per packing tile
constexpr int kEgSubLanes = kBlock / kEgSubTiles;   // lanes of the packing kernel per index entry
static_assert(kEgSubTiles * GG_EG_TILE == kEgBlock && kEgSubLanes * kEgPerLane == GG_EG_TILE, "index entries fall on lane boundaries");
constexpr int kEgLdsWords = kEgBlock * 2 + 2;       // <= 63 bits per symbol, plus the alignment slack
constexpr int kEgTilesPerBlock = 4;                 // consecutive tiles one workgroup packs, loads of the next in flight
static_assert(kEgPerLane == 8, "two 16-byte loads per lane and tile");

__device__ __forceinline__ uint32_t map_q(int32_t q) {
    const int32_t m = -q;
    return ((uint32_t)m << 1) ^ (uint32_t)(m >> 31);
}

__device__ __forceinline__ uint32_t eg_len(uint32_t v, int eg_k) {   // v = u + 2^k
    return 63u - (uint32_t)eg_k - 2u * (uint32_t)__builtin_clz(v);
}

// Where the coder's symbols come from: an int32 array (as written by the rate sweep), or a tensor quantised
// on the fly with the rate sweep's arithmetic (one fp32 product, NaN -> 0, clamp to +-2^30, floor or
// nearest-even), so that a tensor goes to its bit stream without a symbol array in between.
// A source also says which elements share one set of parameters: `begin(i)` gives the context of element
// i, `covers(ctx, end)` tells whether it holds unchanged up to element `end`, `seek(ctx, i)` and `one(i, ctx)`
// move it on as needed (i must not decrease).  Only the bucket source has more than one context.
struct NoCtx {};

struct SymbolArray {
    const int32_t *q;
    using raw4 = gg_i4;
    using Ctx = NoCtx;
    __device__ __forceinline__ Ctx begin(int64_t) const { return {}; }
    __device__ __forceinline__ bool covers(const Ctx &, int64_t) const { return true; }
    __device__ __forceinline__ void seek(Ctx &, int64_t) const {}
    __device__ __forceinline__ raw4 load4(int64_t i) const { return load_vec<gg_i4, true>(reinterpret_cast<const gg_i4 *>(q + i)); }
    __device__ __forceinline__ void conv4(const raw4 &r, int32_t *o, const Ctx &) const { o[0] = r.x; o[1] = r.y; o[2] = r.z; o[3] = r.w; }
    __device__ __forceinline__ int32_t one(int64_t i, Ctx &) const { return q[i]; }
};

template <bool NEAREST>
__device__ __forceinline__ int32_t quantise(float x, float inv_delta) {
    const float t = x * inv_delta;
    int32_t m;
    asm("v_cvt_i32_f32 %0, %1" : "=v"(m) : "v"(NEAREST ? rintf(-t) : ceilf(-t)));   // m = -q; NaN -> 0, saturating
    m = m < -kQLimT ? -kQLimT : (m > kQLimT ? kQLimT : m);
    return -m;
}

// four consecutive elements of a tensor as raw bits, and their values
template <typename T> struct Quad;
template <> struct Quad<float> {
    using raw4 = gg_f4;
    static __device__ __forceinline__ raw4 load(const float *p) { return load_vec<gg_f4, true>(reinterpret_cast<const gg_f4 *>(p)); }
    static __device__ __forceinline__ void values(const raw4 &r, float (&v)[4]) { v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w; }
    static __device__ __forceinline__ float value(const float *p) { return *p; }
};
template <> struct Quad<bf16_t> {
    using raw4 = gg_u2;
    static __device__ __forceinline__ raw4 load(const bf16_t *p) { return load_vec<gg_u2, true>(reinterpret_cast<const gg_u2 *>(p)); }
    static __device__ __forceinline__ void values(const raw4 &r, float (&v)[4]) {
        v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
        v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
    }
    static __device__ __forceinline__ float value(const bf16_t *p) { return __uint_as_float((uint32_t)p->bits << 16); }
};

template <typename T, bool NEAREST> struct QuantisedTensor {
    const T *x; float inv_delta;
    using raw4 = typename Quad<T>::raw4;
    using Ctx = NoCtx;
    __device__ __forceinline__ Ctx begin(int64_t) const { return {}; }
    __device__ __forceinline__ bool covers(const Ctx &, int64_t) const { return true; }
    __device__ __forceinline__ void seek(Ctx &, int64_t) const {}
    __device__ __forceinline__ raw4 load4(int64_t i) const { return Quad<T>::load(x + i); }
    __device__ __forceinline__ void conv4(const raw4 &r, int32_t *o, const Ctx &) const {
        float v[4];
        Quad<T>::values(r, v);
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = quantise<NEAREST>(v[j], inv_delta);
    }
    __device__ __forceinline__ int32_t one(int64_t i, Ctx &) const { return quantise<NEAREST>(Quad<T>::value(x + i), inv_delta); }
};

// a flat bucket with one step per unit (off: S + 1 element offsets, units: 1/Delta per unit, 0 = no usable step)
template <typename T, bool NEAREST> struct QuantisedBucket {
    const T *x; const int64_t *off; const UnitCoef *units; int32_t S;
    using raw4 = typename Quad<T>::raw4;
    struct Ctx { int32_t unit; int64_t end; float inv_delta; };
    __device__ __forceinline__ Ctx begin(int64_t i) const {     // i < off[S]
        int lo = 0, hi = S;        // the largest u with off[u] <= i: its unit is not empty and holds i
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (off[mid] <= i) lo = mid; else hi = mid;
        }
        return Ctx{lo, off[lo + 1], units[lo].inv_delta};
    }
    __device__ __forceinline__ bool covers(const Ctx &c, int64_t end) const { return end <= c.end; }
    // move a context forward to element i >= its unit's start: a few steps of walking, else a fresh search
    __device__ __forceinline__ void seek(Ctx &c, int64_t i) const {
        for (int step = 0; step < 8 && i >= c.end; ++step) { ++c.unit; c.end = off[c.unit + 1]; c.inv_delta = units[c.unit].inv_delta; }
        if (i >= c.end) c = begin(i);
    }
    __device__ __forceinline__ raw4 load4(int64_t i) const { return Quad<T>::load(x + i); }
    __device__ __forceinline__ void conv4(const raw4 &r, int32_t *o, const Ctx &c) const {
        float v[4];
        Quad<T>::values(r, v);
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = quantise<NEAREST>(v[j], c.inv_delta);
    }
    __device__ __forceinline__ int32_t one(int64_t i, Ctx &c) const {
        while (i >= c.end) { ++c.unit; c.end = off[c.unit + 1]; c.inv_delta = units[c.unit].inv_delta; }
        return quantise<NEAREST>(Quad<T>::value(x + i), c.inv_delta);
    }
};

// one wave per tile: 8 x 16 bytes per lane in flight
template <typename Src>
__global__ __launch_bounds__(kBlock) void k_eg_tile_bits(Src src, int64_t n, int64_t nb, int eg_k, uint64_t *__restrict__ tile_bits) {
    const int lane = threadIdx.x & 63;
    const int64_t tile = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (tile >= nb) return;
    const int64_t base = tile * kEgBlock;
    const int64_t stop = base + kEgBlock < n ? base + kEgBlock : n;
    const uint32_t add = 1u << eg_k;
    uint32_t bits = 0;
    typename Src::Ctx ctx = src.begin(base);
    if (base + kEgBlock <= n && src.covers(ctx, base + kEgBlock)) {
        typename Src::raw4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = src.load4(base + (int64_t)(j * 64 + lane) * 4);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            int32_t q[4];
            src.conv4(v[j], q, ctx);
            bits += eg_len(map_q(q[0]) + add, eg_k) + eg_len(map_q(q[1]) + add, eg_k) + eg_len(map_q(q[2]) + add, eg_k) +
                    eg_len(map_q(q[3]) + add, eg_k);
        }
    } else {
        for (int64_t i = base + lane; i < stop; i += 64) bits += eg_len(map_q(src.one(i, ctx)) + add, eg_k);
    }
    bits = wave_reduce(bits, OpAdd());
    if (lane == 0) tile_bits[tile] = bits;
}

// Exclusive scan of the tile sizes: tile_off[i] = sizes[0] + ... + sizes[i-1], the total to tile_off[nb] and
// *total_out.  A workgroup owns kEgScanSeg consecutive tiles; what lies before its segment it adds up from
// the per-group sums a first small kernel leaves (one group: nothing to add), so the groups need not wait
// for each other and the work stays linear in the number of tiles.
constexpr int kEgScanSeg = 8192;                    // 1024 lanes x 8 tiles

__global__ __launch_bounds__(1024) void k_eg_group_sums(const uint64_t *__restrict__ sizes, int64_t nb, uint64_t *__restrict__ group_sums) {
    __shared__ uint64_t wsum[16];
    const int tid = threadIdx.x;
    const int64_t i0 = (int64_t)blockIdx.x * kEgScanSeg + (int64_t)tid * 8;
    uint64_t mine = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) mine += i0 + j < nb ? sizes[i0 + j] : 0;
    mine = wave_reduce(mine, OpAdd());
    if ((tid & 63) == 0) wsum[tid >> 6] = mine;
    __syncthreads();
    if (tid == 0) {
        uint64_t all = 0;
        for (int w = 0; w < 16; ++w) all += wsum[w];
        group_sums[blockIdx.x] = all;
    }
}

__global__ __launch_bounds__(1024) void k_eg_scan(const uint64_t *__restrict__ sizes, const uint64_t *__restrict__ group_sums,
                                                  uint64_t *__restrict__ tile_off, int64_t nb,
                                                  uint64_t *__restrict__ index_end, uint64_t *__restrict__ total_out) {
    __shared__ uint64_t wsum[2][16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t seg0 = (int64_t)blockIdx.x * kEgScanSeg;
    uint64_t before = 0;
    for (int64_t g = tid; g < (int64_t)blockIdx.x; g += 1024) before += group_sums[g];
    const uint64_t before_w = wave_reduce(before, OpAdd());
    if (lane == 0) wsum[0][wave] = before_w;

    const int64_t i0 = seg0 + (int64_t)tid * 8;
    uint64_t e[8];
    if (i0 + 8 <= nb) {
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = sizes[i0 + j];
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = i0 + j < nb ? sizes[i0 + j] : 0;
    }
    uint64_t mine = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) mine += e[j];
    uint64_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t t = __shfl_up(incl, d, 64);
        if (lane >= d) incl += t;
    }
    if (lane == 63) wsum[1][wave] = incl;
    __syncthreads();
    uint64_t carry = 0, below = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) { carry += wsum[0][w]; below += w < wave ? wsum[1][w] : 0; all += wsum[1][w]; }
    uint64_t run = carry + below + (incl - mine);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (i0 + j < nb) {
            tile_off[i0 + j] = run;
            run += e[j];
        }
    }
    if (tid == 0 && seg0 + kEgScanSeg >= nb) {          // the group that owns the last tile (or the only group when nb = 0)
        const uint64_t total = carry + all;
        tile_off[nb] = total;
        *index_end = total;                             // the last entry of the decoding index
        if (total_out) *total_out = total;
    }
}

struct EgSymbols { int32_t q[kEgPerLane]; };

// the eight consecutive symbols of a lane; positions at and beyond n read as 0.  `tile_ctx` is the context of
// the tile's first element (if the tile has any).
template <typename Src>
__device__ __forceinline__ EgSymbols eg_load(const Src &src, const typename Src::Ctx &tile_ctx, int64_t i0, int64_t n) {
    EgSymbols s;
    if (i0 + kEgPerLane <= n && src.covers(tile_ctx, i0 + kEgPerLane)) {
        const typename Src::raw4 a = src.load4(i0), b = src.load4(i0 + 4);
        src.conv4(a, s.q, tile_ctx);
        src.conv4(b, s.q + 4, tile_ctx);
    } else if (i0 < n) {
        typename Src::Ctx c = src.begin(i0);
#pragma unroll
        for (int j = 0; j < kEgPerLane; ++j) s.q[j] = i0 + j < n ? src.one(i0 + j, c) : 0;
    } else {
#pragma unroll
        for (int j = 0; j < kEgPerLane; ++j) s.q[j] = 0;
    }
    return s;
}

// A workgroup packs kEgTilesPerBlock consecutive tiles.  All its symbol loads and tile offsets are issued up
// front, so the only wait for global memory comes once; the words it stores are never waited for.
template <typename Src>
__global__ __launch_bounds__(kBlock) void k_eg_encode(Src src, int64_t n, int64_t nb, int eg_k,
                                                      const uint64_t *__restrict__ tile_off, uint64_t *__restrict__ index,
                                                      uint32_t *__restrict__ stream, uint64_t capacity_bits) {
    __shared__ uint32_t buf[kEgLdsWords];
    __shared__ uint32_t wave_tot[kWaves];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t tile_first = (int64_t)blockIdx.x * kEgTilesPerBlock;
    if (tile_first >= nb) return;
    const int tiles = (int)(nb - tile_first < kEgTilesPerBlock ? nb - tile_first : kEgTilesPerBlock);
    const uint32_t add = 1u << eg_k;

    EgSymbols sym[kEgTilesPerBlock];
    uint64_t off[kEgTilesPerBlock + 1];
    typename Src::Ctx tile_ctx = src.begin(tile_first * kEgBlock);      // one search per workgroup; the rest moves on from it
#pragma unroll
    for (int t = 0; t < kEgTilesPerBlock; ++t) {
        const int64_t tile_base = (tile_first + t) * kEgBlock;
        if (tile_base < n) src.seek(tile_ctx, tile_base);
        sym[t] = eg_load(src, tile_ctx, tile_base + (int64_t)tid * kEgPerLane, n);   // all zero past n
    }
#pragma unroll
    for (int t = 0; t <= kEgTilesPerBlock; ++t) off[t] = tile_off[t <= tiles ? tile_first + t : tile_first + tiles];
    // the symbols that follow this group's tiles: at most 31 of them reach into the group's last word
    const int64_t peek_i = (tile_first + tiles) * kEgBlock + tid;
    const bool peek_live = tid < 32 && peek_i < n;
    int32_t peek_q = 0;
    if (peek_live) { typename Src::Ctx c = tile_ctx; src.seek(c, peek_i); peek_q = src.one(peek_i, c); }
    for (int i = tid; i < kEgLdsWords; i += kBlock) buf[i] = 0;
    uint32_t carry = 0;       // held by the lane that copied out a tile's last word: bits to start the next tile with
    bool carried = false;     // uniform: the previous tile left its last word to this one

#pragma unroll
    for (int t = 0; t < kEgTilesPerBlock; ++t) {
        if (t >= tiles) break;
        const int64_t i0 = (tile_first + t) * kEgBlock + (int64_t)tid * kEgPerLane;
        const uint64_t off0 = off[t], off1 = off[t + 1];
        const bool fits = off1 <= capacity_bits;        // stream too small: nothing of this tile is written

        // a lane owns kEgPerLane consecutive symbols, so positions follow from one scan of lane totals
        const int64_t left = n - i0;
        const int nvalid = left >= kEgPerLane ? kEgPerLane : (left > 0 ? (int)left : 0);   // < 8 only at the very end
        uint32_t v[kEgPerLane], len[kEgPerLane], mine = 0;
#pragma unroll
        for (int j = 0; j < kEgPerLane; ++j) {
            v[j] = map_q(sym[t].q[j]) + add;            // absent symbols were loaded as 0: v >= 1 always
            len[j] = eg_len(v[j], eg_k);
        }
        if (nvalid < kEgPerLane) {
#pragma unroll
            for (int j = 0; j < kEgPerLane; ++j) len[j] = j < nvalid ? len[j] : 0u;
        }
#pragma unroll
        for (int j = 0; j < kEgPerLane; ++j) mine += len[j];
        uint32_t incl = mine;                           // inclusive scan across the wave
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t x = __shfl_up(incl, d, 64);
            if (lane >= d) incl += x;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();                                // also: buf is all zero (initial clear / previous copy-out)
        uint32_t pos = incl - mine;
        for (int w = 0; w < wave; ++w) pos += wave_tot[w];
        if ((tid & (kEgSubLanes - 1)) == 0 && i0 < n) index[i0 / GG_EG_TILE] = off0 + pos;   // bit offset of symbol i0
        pos += (uint32_t)(off0 & 31u);                  // LDS bit 0 is the stream's word boundary below off0
        if (fits) {
            if (carry) { atomicOr(&buf[0], carry); carry = 0; }   // the previous tile's last, partial word
            // the zero prefix is already there (buf is clear); OR the significant bits of v in, first bit at
            // stream bit p (bit 31 of a word is the earliest).  The second word is OR-ed even when nothing
            // spills into it: cheaper than a divergent branch.
            auto place = [&](int j) {
                const uint32_t nbit = 32u - (uint32_t)__builtin_clz(v[j]);   // significant bits of v
                const uint32_t p = pos + (len[j] - nbit);
                const uint64_t window = (uint64_t)v[j] << (64u - nbit - (p & 31u));
                atomicOr(&buf[p >> 5], (uint32_t)(window >> 32));
                atomicOr(&buf[(p >> 5) + 1], (uint32_t)window);
                pos += len[j];
            };
            if (nvalid == kEgPerLane) {
#pragma unroll
                for (int j = 0; j < kEgPerLane; ++j) place(j);
            } else {
#pragma unroll
                for (int j = 0; j < kEgPerLane; ++j) if (j < nvalid) place(j);
            }
            const uint32_t span_end = (uint32_t)(off0 & 31u) + (uint32_t)(off1 - off0);   // LDS bit after the tile
            if (t + 1 == tiles && wave == 0 && (span_end & 31u)) {
                // complete the group's last word with the first bits of the next group's tile
                const uint32_t pv = map_q(peek_q) + add;
                const uint32_t plen = peek_live ? eg_len(pv, eg_k) : 0u;
                uint32_t pincl = plen;
#pragma unroll
                for (int d = 1; d < 32; d <<= 1) {
                    const uint32_t x = __shfl_up(pincl, d, 64);
                    if (lane >= d) pincl += x;
                }
                const uint32_t pstart = span_end + (pincl - plen);
                if (plen && pstart < ((span_end + 31u) & ~31u)) {       // starts inside that word
                    const uint32_t nbit = 32u - (uint32_t)__builtin_clz(pv);
                    const uint32_t p = pstart + (plen - nbit);
                    const uint64_t window = (uint64_t)pv << (64u - nbit - (p & 31u));
                    atomicOr(&buf[p >> 5], (uint32_t)(window >> 32));
                    atomicOr(&buf[(p >> 5) + 1], (uint32_t)window);
                }
            }
        }
        __syncthreads();
        if (fits) {
            const uint64_t w0 = off0 >> 5;
            const uint32_t span_bits = (uint32_t)(off0 & 31u) + (uint32_t)(off1 - off0);
            const uint32_t nwords = (span_bits + 31u) >> 5;
            const bool tail_shared = (off1 & 31u) != 0;     // the last word also holds the next tile's first bits
            // The word shared with the next tile stays in the workgroup when that tile is packed here too: its
            // bits are carried into the next tile's first LDS word.  The group's very last word was completed
            // above and is stored whole; the first word of the group's first tile, when it starts inside a
            // word, belongs to the group before.
            const bool keep_tail = tail_shared && t + 1 < tiles && off[t + 2 <= kEgTilesPerBlock ? t + 2 : t + 1] <= capacity_bits;
            const bool head_foreign = !carried && (off0 & 31u) != 0;
            for (uint32_t i = tid; i < nwords; i += kBlock) {
                const uint32_t raw = buf[i];
                buf[i] = 0;
                if (i == nwords - 1 && keep_tail) carry = raw;
                else if (i == 0 && head_foreign) {}
                else stream[w0 + i] = __builtin_bswap32(raw);       // most significant byte first in memory
            }
            carried = keep_tail;
        } else {
            carried = false;
        }
        // the barrier after the next tile's lane scan separates this copy-out from the next tile's ORs
    }
}

// Decoder: one lane per index tile (GG_EG_TILE symbols), a wave decodes 64 tiles side by side.  Each lane
// keeps the next words of its tile in an LDS ring that is topped up four words at a time by a load issued
// before four symbols are decoded and stored after them, so decoding does not wait for global memory.
// ROW symbols per lane are collected in LDS and written as one piece per tile (a whole 128-byte line for
// ROW = 32).  Reads stay within the words that hold bits of the indexed tiles, whatever the stream contains.
constexpr int kEgDecStep = 4;      // symbols between top-ups
// Symbols a lane decodes between writes (ROW of k_eg_decode).  32 symbols of a tile are one 128-byte line per
// store round, written with streaming stores: 16 is 15-20 % slower, 8 and 4 25-80 % (partial lines), 64 15 % (LDS
// leaves room for fewer waves).  The per-unit variant takes the same (its own constant for tuning builds).
#ifndef GG_EG_DEC_ROW
#define GG_EG_DEC_ROW 32
#endif
#ifndef GG_EG_DEC_ROW_UNITS
#define GG_EG_DEC_ROW_UNITS 32
#endif
constexpr int kEgRing = 16;        // ring words per lane
constexpr int kEgTopUp = 4;        // words a lane loads per top-up
constexpr int kEgStepWords = 10;   // a step takes at most 4 x 63 bits < 8 words, plus the look-ahead word and slack
static_assert(kEgStepWords + kEgTopUp <= kEgRing && GG_EG_TILE % GG_EG_DEC_ROW == 0 && GG_EG_DEC_ROW % kEgDecStep == 0 &&
              GG_EG_TILE % GG_EG_DEC_ROW_UNITS == 0 && GG_EG_DEC_ROW_UNITS % kEgDecStep == 0,
              "ring holds a step and a top-up");
typedef unsigned int EgWords4 __attribute__((ext_vector_type(4), aligned(4)));   // four stream words at any word address

// OUT 0: the symbols.  OUT 1, 2: what they stand for instead, q * delta in fp32, written or added to what is
// there (the receiving side of a sum of coded tensors needs no symbol array in memory) -- 1 with one step for
// the whole stream, 2 with the step of the unit an element lies in (a flat bucket as gg_eg_encode_segmented
// codes it; a unit without a positive finite step was coded as zeros and decodes to zeros).
struct EgUnits { const int64_t *off; const float *delta; int32_t S; };

// the unit that holds element i (the largest u with off[u] <= i; unit 0 for anything before the first)
__device__ __forceinline__ int eg_unit_of(const EgUnits &un, int64_t i) {
    int lo = 0, hi = un.S;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (un.off[mid] <= i) lo = mid; else hi = mid;
    }
    return lo;
}
// move u forward to the unit of element i >= the start of u: a few steps of walking, else a fresh search
__device__ __forceinline__ void eg_unit_seek(const EgUnits &un, int &u, int64_t i) {
    for (int step = 0; step < 8 && u + 1 < un.S && un.off[u + 1] <= i; ++step) ++u;
    if (u + 1 < un.S && un.off[u + 1] <= i) u = eg_unit_of(un, i);
}
__device__ __forceinline__ float eg_unit_step(const EgUnits &un, int u) {
    const float d = un.delta[u];
    return d > 0.f && isfinite(d) ? d : 0.f;
}

// -m without signed overflow (a stream that is not a code stream may decode to any 32 bits)
__device__ __forceinline__ int32_t eg_turn(int32_t m) { return (int32_t)(0u - (uint32_t)m); }

template <int OUT, int ROW>
__global__ __launch_bounds__(64) void k_eg_decode(const uint32_t *__restrict__ stream, const uint64_t *__restrict__ index,
                                                  int64_t n, int64_t tiles, int eg_k, int32_t *__restrict__ q,
                                                  float *__restrict__ xhat, float delta, int accumulate, EgUnits un) {
    __shared__ int tile_unit[64];
    __shared__ uint32_t ring[kEgRing + 1][64];        // see commit4
    constexpr int kEgLanesPerTile = ROW / 4;          // lanes that write one tile's symbols of a round, 16 bytes each
    constexpr int kEgTilesPerPass = 64 / kEgLanesPerTile;   // tiles one store instruction of the wave covers
#ifdef GG_EG_DEC_PLAIN_STORES   // tuning builds
    constexpr bool kStreamOut = false;
#else
    constexpr bool kStreamOut = ROW >= 32;
#endif
    __shared__ int32_t stage[64][ROW + 1];
    const int lane = threadIdx.x;
    const int64_t tile0 = (int64_t)blockIdx.x * 64;
    const int64_t tile = tile0 + lane;
    const bool live = tile < tiles;
    if constexpr (OUT == 2) {            // read after the first barrier below
        const int64_t e = tile * GG_EG_TILE;
        tile_unit[lane] = live && e < n ? eg_unit_of(un, e) : 0;
    }
    // OUT 2: the unit each row this lane writes has reached, where that unit ends and its step -- kept in registers,
    // so that only a group of four elements that reaches the end of its unit goes back to the unit table
    int row_unit[kEgLanesPerTile];
    int64_t row_end[kEgLanesPerTile];
    float row_step[kEgLanesPerTile];
#pragma unroll
    for (int r = 0; r < kEgLanesPerTile; ++r) { row_unit[r] = -1; row_end[r] = 0; row_step[r] = 0.f; }
    const uint64_t pos0 = live ? index[tile] : 0;
    const uint32_t *src = stream + (pos0 >> 5);                             // the lane's words, counted from its first
    // Words from `end_rel` on read as zero: the stream's words end there (those that hold bits of the indexed tiles).
    // A lane may load words of the tiles behind its own -- it decodes GG_EG_TILE symbols and no more -- so that only
    // the loads at the very end of the stream take the word-by-word path below.
    const uint64_t stream_words = (index[tiles] + 31u) >> 5, first_word = pos0 >> 5;
    const uint64_t left = live && stream_words > first_word ? stream_words - first_word : 0u;
    const uint32_t end_rel = left < 0x7fffffffu ? (uint32_t)left : 0x7fffffffu;
    uint32_t ld = 0;                  // words loaded into the ring so far (a multiple of kEgTopUp)
    // four words from the lane's position `ld` on (a 16-byte load from a 4-byte-aligned address)
    auto fetch4 = [&]() -> EgWords4 {
        EgWords4 w = {0u, 0u, 0u, 0u};
        if (ld + kEgTopUp <= end_rel) {
            w = *reinterpret_cast<const EgWords4 *>(src + ld);
        } else {
            if (ld < end_rel) w.x = src[ld];
            if (ld + 1 < end_rel) w.y = src[ld + 1];
            if (ld + 2 < end_rel) w.z = src[ld + 2];
        }
        return w;
    };
    // word i of the lane lives in slot kEgRing - (i mod kEgRing), so that a word and its successor are read as one
    // 64-bit value with the earlier word on top; words 0, kEgRing, ... are kept in slot 0 as well (no wrap in a window)
    auto commit4 = [&](EgWords4 w) {
        const uint32_t slot = kEgRing - (ld & (kEgRing - 1)), first = __builtin_bswap32(w.x);
        ring[slot][lane] = first;
        ring[slot - 1][lane] = __builtin_bswap32(w.y);
        ring[slot - 2][lane] = __builtin_bswap32(w.z);
        ring[slot - 3][lane] = __builtin_bswap32(w.w);
        if (slot == kEgRing) ring[0][lane] = first;
        ld += kEgTopUp;
    };
#pragma unroll 1
    for (int r = 0; r < kEgRing / kEgTopUp; ++r) commit4(fetch4());       // fill the ring

    // The lane's position in its part of the stream is one number, `pos` (bits from the start of its first word); the
    // 32 bits from any position on are two neighbouring ring words shifted together, so a symbol costs no window
    // upkeep: count the zeros, cut the value out of the same 32 bits, move on.  Words below pos / 32 are spent.
    uint32_t pos = (uint32_t)(pos0 & 31u);
    auto bits32 = [&](uint32_t at) -> uint32_t {
        const uint32_t *p = &ring[(kEgRing - 1) - ((at >> 5) & (uint32_t)(kEgRing - 1))][lane];   // the successor's slot
        const uint64_t two = ((uint64_t)p[64] << 32) | (uint64_t)p[0];
        return (uint32_t)((two << (at & 31u)) >> 32);
    };

    const uint32_t add = 1u << eg_k, k1 = (uint32_t)eg_k + 1u;
    const bool adding = OUT != 0 && accumulate && n >= 4;
    for (int s0 = 0; s0 < GG_EG_TILE; s0 += ROW) {
        // adding to what is there: the values this round's writers will add to start travelling now, while the
        // round's symbols are decoded (a writer past the end of the data asks for elements 0..3 and drops them)
        gg_f4 was[kEgLanesPerTile];
        if constexpr (OUT != 0) {
            if (adding) {
#pragma unroll
                for (int r = 0; r < kEgLanesPerTile; ++r) {
                    const int row = r * kEgTilesPerPass + lane / kEgLanesPerTile, c = (lane % kEgLanesPerTile) * 4;
                    const int64_t g = (tile0 + row) * GG_EG_TILE + s0 + c;
                    const gg_f4 *from = reinterpret_cast<const gg_f4 *>(xhat + (g + 4 <= n ? g : 0));
                    if constexpr (kStreamOut) was[r] = __builtin_nontemporal_load(from);
                    else was[r] = *from;
                }
            }
        }
#pragma unroll
        for (int s1 = 0; s1 < ROW; s1 += kEgDecStep) {
            while (__any(ld - (pos >> 5) < (uint32_t)kEgStepWords)) {          // rare: only streams with very long codes
                if (ld - (pos >> 5) < (uint32_t)kEgStepWords) commit4(fetch4());
            }
            const bool more = ld - (pos >> 5) <= (uint32_t)(kEgRing - kEgTopUp);   // room for four more whatever this step takes
            EgWords4 pre = {0u, 0u, 0u, 0u};
            if (more) pre = fetch4();
            // lanes past the end of the data decode zeros or stale bits; nothing of that is written
#pragma unroll
            for (int j = 0; j < kEgDecStep; ++j) {
                const uint32_t top = bits32(pos);
                uint32_t zeros = (uint32_t)__clz((int)top);         // 32 for no bit at all
                zeros = zeros > 31u ? 31u : zeros;                  // a valid stream has at most 31
                uint32_t L = zeros + k1;
                L = L > 32u ? 32u : L;
                const uint32_t total = zeros + L;
                uint32_t v;
                if (__any(total > 32u)) v = bits32(pos + zeros) >> (32u - L);   // some lane's code does not end within these 32 bits
                else v = (top << zeros) >> (32u - L);
                pos += total;
                const uint32_t u = v - add;
                // inverse Map, negated: -q is the zig-zag decoding of u (the writers below turn the sign)
                stage[lane][s1 + j] = (int32_t)(u >> 1) ^ -(int32_t)(u & 1u);
            }
            if (more) commit4(pre);
        }
        __syncthreads();
        // kEgLanesPerTile lanes cover one tile's symbols of this round (ROW 32: eight lanes write its 128 bytes, a
        // store instruction of the wave covers 8 tiles, 8 instructions)
#pragma unroll
        for (int r = 0; r < kEgLanesPerTile; ++r) {
            const int row = r * kEgTilesPerPass + lane / kEgLanesPerTile, c = (lane % kEgLanesPerTile) * 4;
            const int64_t g = (tile0 + row) * GG_EG_TILE + s0 + c;
            if constexpr (OUT != 0) {
                float d[4] = {delta, delta, delta, delta};
                if constexpr (OUT == 2) {
                    if (g < n) {
                        if (g + 4 <= row_end[r]) {                          // the four elements lie in the row's unit
                            d[0] = row_step[r]; d[1] = d[0]; d[2] = d[0]; d[3] = d[0];
                        } else {
                            int u = row_unit[r] < 0 ? tile_unit[row] : row_unit[r];
                            for (int x = 0; x < 4; ++x) { eg_unit_seek(un, u, g + x); d[x] = eg_unit_step(un, u); }
                            row_unit[r] = u;                                // the unit of element g + 3: later groups start behind it
                            row_end[r] = u + 1 < un.S ? un.off[u + 1] : 0x7fffffffffffffffLL;
                            row_step[r] = d[3];
                        }
                    }
                }
                if (g + 4 <= n) {
                    gg_f4 val = {(float)eg_turn(stage[row][c]) * d[0], (float)eg_turn(stage[row][c + 1]) * d[1], (float)eg_turn(stage[row][c + 2]) * d[2],
                                 (float)eg_turn(stage[row][c + 3]) * d[3]};
                    gg_f4 *dst = reinterpret_cast<gg_f4 *>(xhat + g);
                    // streaming accesses where a round writes whole 128-byte lines: what is written here is not read
                    // again by this kernel, and the cache is better spent on the stream lines, which every lane comes
                    // back to eight times
                    if (adding) val += was[r];
                    if constexpr (kStreamOut) __builtin_nontemporal_store(val, dst);
                    else *dst = val;
                } else {
                    for (int x = 0; x < 4; ++x)
                        if (g + x < n) {
                            const float val = (float)eg_turn(stage[row][c + x]) * d[x];
                            xhat[g + x] = accumulate ? xhat[g + x] + val : val;
                        }
                }
            } else if (g + 4 <= n) {
                const gg_i4 val = {eg_turn(stage[row][c]), eg_turn(stage[row][c + 1]), eg_turn(stage[row][c + 2]), eg_turn(stage[row][c + 3])};
                if constexpr (kStreamOut) __builtin_nontemporal_store(val, reinterpret_cast<gg_i4 *>(q + g));
                else *reinterpret_cast<gg_i4 *>(q + g) = val;
            } else {
                for (int x = 0; x < 4; ++x) if (g + x < n) q[g + x] = eg_turn(stage[row][c + x]);
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// host
// ---------------------------------------------------------------------------------------------
// Element-wise kernels run as many short blocks (one read + write stream each): `parts` blocks per chunk,
// so that a block issues all its loads at once.
#ifndef GG_TRAIN_PARTS_F32
#define GG_TRAIN_PARTS_F32 4      // 4096 elements per block = 256 lanes x 4 loads x 4 elements
#endif
static int slope_args(const Geometry &g, int eg_k, int parts, SlopeArgs &a, unsigned &blocks_out) {
    a = SlopeArgs{};
    a.eg_add = 1u << eg_k;
    a.n_chunks = g.n_chunks;
    a.parts = parts;
    if (g.n_chunks > 2147483647LL / parts) return GG_ERR_INVALID_ARG;
    blocks_out = (unsigned)(g.n_chunks * parts);
    return GG_OK;
}

static UnitCoef host_coef(float delta, int64_t n_rate, float scale) {
    UnitCoef uc;
    uc.inv_delta = (float)(1.0 / (double)delta);
    uc.coef = (float)((double)scale * 4.0 * (double)uc.inv_delta / ((double)n_rate * 0.69314718055994530942));
    return uc;
}

// workspace: decoding index (T + 1 entries, T = ceil(n / GG_EG_TILE)) | packing-tile offsets (P + 1) | tile sizes (P) |
// sums of the scan groups (ceil(P / kEgScanSeg))
static int64_t eg_index_tiles(int64_t n) { return (n + GG_EG_TILE - 1) / GG_EG_TILE; }
static int64_t eg_pack_tiles(int64_t n) { return (n + kEgBlock - 1) / kEgBlock; }

// the three launches of the coder for any symbol source
template <typename Src>
static int eg_encode_launch(const Src &src, int64_t n, int eg_k, uint8_t *stream_dev, uint64_t stream_bytes,
                            uint64_t *block_offsets_dev, uint64_t *total_bits_dev, hipStream_t st) {
    const int64_t nb = eg_pack_tiles(n), T = eg_index_tiles(n);
    if (nb > 2147483647LL * kWaves) return GG_ERR_INVALID_ARG;
    uint64_t *tile_off = block_offsets_dev + T + 1;
    uint64_t *sizes = tile_off + nb + 1;
    int rc;
    if (nb > 0) {
        hipLaunchKernelGGL(k_eg_tile_bits<Src>, dim3((unsigned)((nb + kWaves - 1) / kWaves)), dim3(kBlock), 0, st, src, n, nb,
                           eg_k, sizes);
        if ((rc = check_launch()) != GG_OK) return rc;
    }
    const int64_t groups = nb > 0 ? (nb + kEgScanSeg - 1) / kEgScanSeg : 1;
    uint64_t *group_sums = sizes + nb;
    if (groups > 1) {
        hipLaunchKernelGGL(k_eg_group_sums, dim3((unsigned)groups), dim3(1024), 0, st, sizes, nb, group_sums);
        if ((rc = check_launch()) != GG_OK) return rc;
    }
    hipLaunchKernelGGL(k_eg_scan, dim3((unsigned)groups), dim3(1024), 0, st, sizes, group_sums, tile_off, nb,
                       block_offsets_dev + T, total_bits_dev);
    if ((rc = check_launch()) != GG_OK) return rc;
    if (nb > 0) {   // also without room for any stream: this kernel writes the index
        hipLaunchKernelGGL(k_eg_encode<Src>, dim3((unsigned)((nb + kEgTilesPerBlock - 1) / kEgTilesPerBlock)), dim3(kBlock), 0,
                           st, src, n, nb, eg_k, tile_off, block_offsets_dev, reinterpret_cast<uint32_t *>(stream_dev),
                           stream_bytes * 8ull);
        if ((rc = check_launch()) != GG_OK) return rc;
    }
    return GG_OK;
}

static int check_eg_buffers(int64_t n, int eg_k, const uint8_t *stream_dev, uint64_t stream_bytes,
                            const uint64_t *block_offsets_dev, const uint64_t *total_bits_dev) {
    if (n < 0 || eg_k < 0 || eg_k > GG_MAX_EG_K || (stream_bytes & 3u)) return GG_ERR_INVALID_ARG;
    if (!block_offsets_dev || !aligned8(block_offsets_dev)) return GG_ERR_WORKSPACE;
    if (total_bits_dev && !aligned8(total_bits_dev)) return GG_ERR_INVALID_ARG;
    if (stream_bytes && (!stream_dev || (reinterpret_cast<uintptr_t>(stream_dev) & 3u))) return GG_ERR_INVALID_ARG;
    return GG_OK;
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
    SlopeArgs a;
    if ((rc = slope_args(g, eg_k, GG_TRAIN_PARTS_F32, a, blocks)) != GG_OK) return rc;
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
    SlopeArgs a;
    if ((rc = slope_args(g, eg_k, GG_TRAIN_PARTS_F32, a, blocks)) != GG_OK) return rc;
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
    int rc = geometry_segmented(offsets_host, S, ws_dev, ws_bytes, g, true);
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
    SlopeArgs a;
    if ((rc = slope_args(g, eg_k, GG_TRAIN_PARTS_F32, a, blocks)) != GG_OK) return rc;
    a.units = units;
    GctScalars sc{eta, (float)(1.0 / (double)eta), lambda, eps, first_step ? 1 : 0};
    hipLaunchKernelGGL(k_gct_update, dim3(blocks), dim3(kBlock), 0, st, g.sv, g_dev, a, sc, w_dev, ghat_prev_dev);
    return check_launch();
}

int gg_eg_workspace_bytes(int64_t n, size_t *bytes_out_host) {
    if (!bytes_out_host || n < 0) return GG_ERR_INVALID_ARG;
    const int64_t P = eg_pack_tiles(n);
    *bytes_out_host = (size_t)(eg_index_tiles(n) + 2 * P + 2 + (P + kEgScanSeg - 1) / kEgScanSeg) * sizeof(uint64_t);
    return GG_OK;
}

int gg_eg_encode(const int32_t *symbols_dev, int64_t n, int eg_k, uint8_t *stream_dev, uint64_t stream_bytes,
                 uint64_t *block_offsets_dev, uint64_t *total_bits_dev, void *stream) {
    int rc = check_eg_buffers(n, eg_k, stream_dev, stream_bytes, block_offsets_dev, total_bits_dev);
    if (rc != GG_OK) return rc;
    if (n > 0 && (!symbols_dev || !aligned16(symbols_dev))) return GG_ERR_INVALID_ARG;
    return eg_encode_launch(SymbolArray{symbols_dev}, n, eg_k, stream_dev, stream_bytes, block_offsets_dev, total_bits_dev,
                            (hipStream_t)stream);
}

int gg_eg_encode_tensor(const void *x_dev, int dtype, int64_t n, float delta, int round_mode, int eg_k, uint8_t *stream_dev,
                        uint64_t stream_bytes, uint64_t *block_offsets_dev, uint64_t *total_bits_dev, void *stream) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    int rc = check_eg_buffers(n, eg_k, stream_dev, stream_bytes, block_offsets_dev, total_bits_dev);
    if (rc != GG_OK) return rc;
    if (!(delta > 0.f) || !std::isfinite(delta)) return GG_ERR_INVALID_ARG;
    if (round_mode != GG_FLOOR && round_mode != GG_NEAREST_EVEN) return GG_ERR_INVALID_ARG;
    if (n > 0 && (!x_dev || !aligned16(x_dev))) return GG_ERR_INVALID_ARG;
    const float inv_delta = (float)(1.0 / (double)delta);
    hipStream_t st = (hipStream_t)stream;
    const bool nearest = round_mode == GG_NEAREST_EVEN;
    if (dtype == GG_F32) {
        const float *x = static_cast<const float *>(x_dev);
        return nearest ? eg_encode_launch(QuantisedTensor<float, true>{x, inv_delta}, n, eg_k, stream_dev, stream_bytes,
                                          block_offsets_dev, total_bits_dev, st)
                       : eg_encode_launch(QuantisedTensor<float, false>{x, inv_delta}, n, eg_k, stream_dev, stream_bytes,
                                          block_offsets_dev, total_bits_dev, st);
    }
    const bf16_t *x = static_cast<const bf16_t *>(x_dev);
    return nearest ? eg_encode_launch(QuantisedTensor<bf16_t, true>{x, inv_delta}, n, eg_k, stream_dev, stream_bytes,
                                      block_offsets_dev, total_bits_dev, st)
                   : eg_encode_launch(QuantisedTensor<bf16_t, false>{x, inv_delta}, n, eg_k, stream_dev, stream_bytes,
                                      block_offsets_dev, total_bits_dev, st);
}

int gg_eg_encode_segmented(const void *x_dev, int dtype, const int64_t *offsets_host, int32_t S, const float *delta_dev,
                           int round_mode, int eg_k, uint8_t *stream_dev, uint64_t stream_bytes, uint64_t *block_offsets_dev,
                           uint64_t *total_bits_dev, void *ws_dev, size_t ws_bytes, void *stream) {
    if (dtype != GG_F32 && dtype != GG_BF16) return GG_ERR_BAD_DTYPE;
    Geometry g;
    int rc = geometry_segmented(offsets_host, S, ws_dev, ws_bytes, g);
    if (rc != GG_OK) return rc;
    if (S > 0 && offsets_host[0] != 0) return GG_ERR_BAD_SEGMENTS;   // the stream codes elements 0 .. offsets[S): no gap in front
    const int64_t n = g.n_total;
    if ((rc = check_eg_buffers(n, eg_k, stream_dev, stream_bytes, block_offsets_dev, total_bits_dev)) != GG_OK) return rc;
    if (round_mode != GG_FLOOR && round_mode != GG_NEAREST_EVEN) return GG_ERR_INVALID_ARG;
    if (n > 0 && (!x_dev || !aligned16(x_dev) || !delta_dev)) return GG_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const UnitCoef *units = nullptr;
    if (S > 0) {
        if ((rc = upload_geometry(g, st)) != GG_OK) return rc;
        UnitCoef *u = reinterpret_cast<UnitCoef *>(g.params());   // the per-unit parameter area of the workspace
        hipLaunchKernelGGL(k_unit_coef, dim3((unsigned)((S + 255) / 256)), dim3(256), 0, st, g.sv, delta_dev, 1.0f, u);
        if ((rc = check_launch()) != GG_OK) return rc;
        units = u;
    }
    const bool nearest = round_mode == GG_NEAREST_EVEN;
    if (dtype == GG_F32) {
        const float *x = static_cast<const float *>(x_dev);
        return nearest ? eg_encode_launch(QuantisedBucket<float, true>{x, g.sv.off, units, S}, n, eg_k, stream_dev, stream_bytes,
                                          block_offsets_dev, total_bits_dev, st)
                       : eg_encode_launch(QuantisedBucket<float, false>{x, g.sv.off, units, S}, n, eg_k, stream_dev, stream_bytes,
                                          block_offsets_dev, total_bits_dev, st);
    }
    const bf16_t *x = static_cast<const bf16_t *>(x_dev);
    return nearest ? eg_encode_launch(QuantisedBucket<bf16_t, true>{x, g.sv.off, units, S}, n, eg_k, stream_dev, stream_bytes,
                                      block_offsets_dev, total_bits_dev, st)
                   : eg_encode_launch(QuantisedBucket<bf16_t, false>{x, g.sv.off, units, S}, n, eg_k, stream_dev, stream_bytes,
                                      block_offsets_dev, total_bits_dev, st);
}

int gg_eg_decode(const uint8_t *stream_dev, const uint64_t *block_offsets_dev, int64_t n, int eg_k, int32_t *symbols_dev,
                 void *stream) {
    if (n < 0 || eg_k < 0 || eg_k > GG_MAX_EG_K) return GG_ERR_INVALID_ARG;
    if (n == 0) return GG_OK;
    if (!stream_dev || (reinterpret_cast<uintptr_t>(stream_dev) & 3u) || !block_offsets_dev || !aligned8(block_offsets_dev) ||
        !symbols_dev || !aligned16(symbols_dev))
        return GG_ERR_INVALID_ARG;
    const int64_t T = eg_index_tiles(n);
    if ((T + 63) / 64 > 2147483647LL) return GG_ERR_INVALID_ARG;
    hipLaunchKernelGGL((k_eg_decode<0, GG_EG_DEC_ROW>), dim3((unsigned)((T + 63) / 64)), dim3(64), 0, (hipStream_t)stream,
                       reinterpret_cast<const uint32_t *>(stream_dev), block_offsets_dev, n, T, eg_k, symbols_dev,
                       (float *)nullptr, 0.f, 0, EgUnits{nullptr, nullptr, 0});
    return check_launch();
}

int gg_eg_decode_dequant(const uint8_t *stream_dev, const uint64_t *block_offsets_dev, int64_t n, int eg_k, float delta,
                         float *out_dev, int accumulate, void *stream) {
    if (n < 0 || eg_k < 0 || eg_k > GG_MAX_EG_K) return GG_ERR_INVALID_ARG;
    if (!(delta > 0.f) || !std::isfinite(delta)) return GG_ERR_INVALID_ARG;
    if (n == 0) return GG_OK;
    if (!stream_dev || (reinterpret_cast<uintptr_t>(stream_dev) & 3u) || !block_offsets_dev || !aligned8(block_offsets_dev) ||
        !out_dev || !aligned16(out_dev))
        return GG_ERR_INVALID_ARG;
    const int64_t T = eg_index_tiles(n);
    if ((T + 63) / 64 > 2147483647LL) return GG_ERR_INVALID_ARG;
    hipLaunchKernelGGL((k_eg_decode<1, GG_EG_DEC_ROW>), dim3((unsigned)((T + 63) / 64)), dim3(64), 0, (hipStream_t)stream,
                       reinterpret_cast<const uint32_t *>(stream_dev), block_offsets_dev, n, T, eg_k, (int32_t *)nullptr,
                       out_dev, delta, accumulate ? 1 : 0, EgUnits{nullptr, nullptr, 0});
    return check_launch();
}

int gg_eg_decode_dequant_segmented(const uint8_t *stream_dev, const uint64_t *block_offsets_dev, const int64_t *offsets_host,
                                   int32_t S, int eg_k, const float *delta_dev, float *out_dev, int accumulate, void *ws_dev,
                                   size_t ws_bytes, void *stream) {
    if (eg_k < 0 || eg_k > GG_MAX_EG_K) return GG_ERR_INVALID_ARG;
    Geometry g;
    int rc = geometry_segmented(offsets_host, S, ws_dev, ws_bytes, g);
    if (rc != GG_OK) return rc;
    if (S > 0 && offsets_host[0] != 0) return GG_ERR_BAD_SEGMENTS;   // as in gg_eg_encode_segmented
    const int64_t n = g.n_total;
    if (n == 0) return GG_OK;
    if (!stream_dev || (reinterpret_cast<uintptr_t>(stream_dev) & 3u) || !block_offsets_dev || !aligned8(block_offsets_dev) ||
        !delta_dev || !out_dev || !aligned16(out_dev))
        return GG_ERR_INVALID_ARG;
    const int64_t T = eg_index_tiles(n);
    if ((T + 63) / 64 > 2147483647LL) return GG_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if ((rc = upload_geometry(g, st)) != GG_OK) return rc;
    hipLaunchKernelGGL((k_eg_decode<2, GG_EG_DEC_ROW_UNITS>), dim3((unsigned)((T + 63) / 64)), dim3(64), 0, st,
                       reinterpret_cast<const uint32_t *>(stream_dev), block_offsets_dev, n, T, eg_k, (int32_t *)nullptr,
                       out_dev, 0.f, accumulate ? 1 : 0, EgUnits{g.sv.off, delta_dev, S});
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
