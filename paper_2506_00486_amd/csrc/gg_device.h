// gg_device.h -- device-side building blocks of libgg (gfx950 / CDNA4, wave64).
//
// Lane exchange by DPP inside a 16-lane row and by ds_bpermute across rows, wave and
// block reductions with a fixed combination order (so every result is reproducible),
// 128-bit element loads for fp32 / bf16, the chunk walker all streaming kernels share,
// and the Philox4x32-10 block function.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gg {

constexpr int kBlock = 256;          // threads per workgroup: 4 wave64
constexpr int kWaves = kBlock / 64;
#ifndef GG_CHUNK
#define GG_CHUNK 16384
#endif
constexpr int kChunk = GG_CHUNK;     // elements per work item (64 KiB of fp32, 32 KiB of bf16)

// ---------------------------------------------------------------------------------------------
// lane exchange
// ---------------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
}

// DPP controls: quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror.
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

template <int CTRL, typename V>
__device__ __forceinline__ V dpp_xchg(V v) {
    static_assert(sizeof(V) == 4 || sizeof(V) == 8, "32- or 64-bit values only");
    if constexpr (sizeof(V) == 4) {
        uint32_t w = dpp_u32<CTRL>(__builtin_bit_cast(uint32_t, v));
        return __builtin_bit_cast(V, w);
    } else {
        uint64_t b = __builtin_bit_cast(uint64_t, v);
        uint32_t lo = dpp_u32<CTRL>((uint32_t)b), hi = dpp_u32<CTRL>((uint32_t)(b >> 32));
        return __builtin_bit_cast(V, ((uint64_t)hi << 32) | lo);
    }
}

// All-lanes reduction of a wave64 with a commutative op.  After each step both partners hold
// op(a, b) computed from the same two operands, so every lane ends with the same bits.
template <typename V, typename Op>
__device__ __forceinline__ V wave_reduce(V v, Op op) {
    v = op(v, dpp_xchg<kDppXor1>(v));        // pairs
    v = op(v, dpp_xchg<kDppXor2>(v));        // quads
    v = op(v, dpp_xchg<kDppHalfMirror>(v));  // groups of 8
    v = op(v, dpp_xchg<kDppMirror>(v));      // rows of 16
    v = op(v, __shfl_xor(v, 16, 64));
    v = op(v, __shfl_xor(v, 32, 64));
    return v;
}

struct OpAdd { template <typename V> __device__ V operator()(V a, V b) const { return a + b; } };
struct OpMax { template <typename V> __device__ V operator()(V a, V b) const { return a > b ? a : b; } };
struct OpOr  { template <typename V> __device__ V operator()(V a, V b) const { return a | b; } };

// Block reduction: wave results go through LDS and every thread combines them in wave order.
// `slot` must have kWaves entries; consecutive calls must use different slots or be separated
// by the barrier this function ends with.
template <typename V, typename Op>
__device__ __forceinline__ V block_reduce(V v, Op op, V *slot) {
    v = wave_reduce(v, op);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) slot[wave] = v;
    __syncthreads();
    V r = slot[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) r = op(r, slot[w]);
    __syncthreads();
    return r;
}

// ---------------------------------------------------------------------------------------------
// element access: 16 bytes per lane per load
// ---------------------------------------------------------------------------------------------
struct bf16_t { uint16_t bits; };

// The inputs are streamed exactly once per sweep, so their loads are marked non-temporal: on
// gfx950 that keeps the stream from displacing L2 contents and measurably raises read bandwidth.
#ifndef GG_STREAM_LOADS
#define GG_STREAM_LOADS 1
#endif
typedef float gg_f4 __attribute__((ext_vector_type(4)));
typedef unsigned int gg_u4 __attribute__((ext_vector_type(4)));
typedef int gg_i4 __attribute__((ext_vector_type(4)));

typedef unsigned int gg_u2 __attribute__((ext_vector_type(2)));

// NT = true: streaming load (data read once per sweep); NT = false: ordinary cached load (data that
// the same compute unit re-reads shortly, as in the wave-per-row kernels).
template <typename V, bool NT>
__device__ __forceinline__ V load_vec(const V *p) {
#if GG_STREAM_LOADS
    if constexpr (NT) return __builtin_nontemporal_load(p);
#endif
    return *p;
}

template <typename T, bool NT = true> struct Elem;

template <bool NT> struct Elem<float, NT> {
    static constexpr int W = 4;
    using type = float;
    using raw = gg_f4;
    static __device__ __forceinline__ raw loadv(const float *p) {
        return load_vec<gg_f4, NT>(reinterpret_cast<const gg_f4 *>(p));
    }
    static __device__ __forceinline__ void unpack(const raw &r, float (&v)[W]) {
        v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
    }
    static __device__ __forceinline__ float load1(const float *p) { return *p; }
};

template <bool NT> struct Elem<bf16_t, NT> {
    static constexpr int W = 8;
    using type = bf16_t;
    using raw = gg_u4;
    static __device__ __forceinline__ raw loadv(const bf16_t *p) {
        return load_vec<gg_u4, NT>(reinterpret_cast<const gg_u4 *>(p));
    }
    static __device__ __forceinline__ void unpack(const raw &r, float (&v)[W]) {
        // bf16 is the high half of an fp32: widening is a shift (even element) or a mask (odd)
        v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
        v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
        v[4] = __uint_as_float(r.z << 16); v[5] = __uint_as_float(r.z & 0xffff0000u);
        v[6] = __uint_as_float(r.w << 16); v[7] = __uint_as_float(r.w & 0xffff0000u);
    }
    static __device__ __forceinline__ float load1(const bf16_t *p) {
        return __uint_as_float((uint32_t)p->bits << 16);
    }
};

// bf16 with four elements (8 bytes) per lane: used where every element produces a 4-byte output,
// so that a lane's outputs are one 16-byte store and a wave's store instruction covers whole lines.
template <bool NT = true> struct ElemBf16x4T {
    static constexpr int W = 4;
    using type = bf16_t;
    using raw = gg_u2;
    static __device__ __forceinline__ raw loadv(const bf16_t *p) {
        return load_vec<gg_u2, NT>(reinterpret_cast<const gg_u2 *>(p));
    }
    static __device__ __forceinline__ void unpack(const raw &r, float (&v)[W]) {
        v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
        v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
    }
    static __device__ __forceinline__ float load1(const bf16_t *p) {
        return __uint_as_float((uint32_t)p->bits << 16);
    }
};

using ElemBf16x4 = ElemBf16x4T<true>;

// fp32 -> bf16, round to nearest even, NaN kept quiet
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t b = __float_as_uint(f);
    if ((b & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((b >> 16) | 0x0040u);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}

// ---------------------------------------------------------------------------------------------
// chunk walker.  Elements [start, start+len) of x are visited once each by the block:
// a scalar head up to the first vector boundary, W-element vectors (U loads in flight per
// lane), and a scalar tail.  `x` itself must be 16-byte aligned, so the boundary is a
// property of the element index.  body.vec(v, idx) gets W consecutive elements starting at
// element index idx (a multiple of W); body.one(v, idx) gets one.  E is the element policy
// (Elem<float>, Elem<bf16_t>, ElemBf16x4).
// ---------------------------------------------------------------------------------------------
// GROUP threads cooperate (the whole block, or one wave with GROUP = 64).
template <typename E, int U, typename Body, int GROUP = kBlock>
__device__ __forceinline__ void process_chunk(const typename E::type *__restrict__ x, int64_t start, int len,
                                              Body &body) {
    using T = typename E::type;
    constexpr int W = E::W;
    const int tid = threadIdx.x & (GROUP - 1);
    int head = (int)((W - (int)(start % W)) % W);
    if (head > len) head = len;
    if (tid < head) body.one(E::load1(x + start + tid), start + tid);

    const int64_t vstart = start + head;
    const int nvec = (len - head) / W;
    const T *__restrict__ p = x + vstart;
    int i = tid;
    for (; i + (U - 1) * GROUP < nvec; i += U * GROUP) {
        typename E::raw r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = E::loadv(p + (int64_t)(i + u * GROUP) * W);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float v[W];
            E::unpack(r[u], v);
            body.vec(v, vstart + (int64_t)(i + u * GROUP) * W);
        }
    }
    for (; i < nvec; i += GROUP) {
        typename E::raw r = E::loadv(p + (int64_t)i * W);
        float v[W];
        E::unpack(r, v);
        body.vec(v, vstart + (int64_t)i * W);
    }
    const int done = head + nvec * W;
    if (tid < len - done) body.one(E::load1(x + start + done + tid), start + done + tid);
}

// The same walk in two steps, with the loads of the next group of U vectors issued before the current group is
// worked on (two register sets taking turns): for bodies whose work per element is long compared with what the
// resident waves can hide -- a kernel limited to few waves per compute unit by its LDS -- so that a lane always
// has loads in flight.  begin() issues the first group's loads and returns at once, so that the caller can do
// other work (clear LDS, ...) while they travel; peek() hands the first group's elements to a functor without
// consuming them (a look at the data before the body is chosen); run() visits every element exactly once.
template <typename E, int U, int GROUP = kBlock>
struct AheadWalk {
    using T = typename E::type;
    static constexpr int W = E::W;
    const T *x;
    const T *p;
    int64_t start, vstart;
    int len, head, nvec, tid;
    typename E::raw cur[U];
    bool have;

    __device__ __forceinline__ void begin(const T *__restrict__ x_, int64_t start_, int len_) {
        x = x_; start = start_; len = len_;
        tid = threadIdx.x & (GROUP - 1);
        head = (int)((W - (int)(start % W)) % W);
        if (head > len) head = len;
        vstart = start + head;
        nvec = (len - head) / W;
        p = x + vstart;
        have = tid + (U - 1) * GROUP < nvec;
        if (have) {
#pragma unroll
            for (int u = 0; u < U; ++u) cur[u] = E::loadv(p + (int64_t)(tid + u * GROUP) * W);
        }
    }

    // f(v) for the W elements of the first loaded vector of this lane, if it has one
    template <typename F>
    __device__ __forceinline__ void peek(F &&f) const {
        if (have) {
            float v[W];
            E::unpack(cur[0], v);
            f(v);
        }
    }

    template <typename Body>
    __device__ __forceinline__ void run(Body &body) {
        if (tid < head) body.one(E::load1(x + start + tid), start + tid);
        int i = tid;
        typename E::raw nxt[U];
        while (have) {
            const int j = i + U * GROUP;
            const bool more = j + (U - 1) * GROUP < nvec;
            if (more) {
#pragma unroll
                for (int u = 0; u < U; ++u) nxt[u] = E::loadv(p + (int64_t)(j + u * GROUP) * W);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float v[W];
                E::unpack(cur[u], v);
                body.vec(v, vstart + (int64_t)(i + u * GROUP) * W);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) cur[u] = nxt[u];
            i = j;
            have = more;
        }
        for (; i < nvec; i += GROUP) {
            typename E::raw r = E::loadv(p + (int64_t)i * W);
            float v[W];
            E::unpack(r, v);
            body.vec(v, vstart + (int64_t)i * W);
        }
        const int done = head + nvec * W;
        if (tid < len - done) body.one(E::load1(x + start + done + tid), start + done + tid);
    }
};

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): ten rounds of multiply-hi/lo mixing, key bumped by the
// Weyl constants after each round.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // one 32x32->64 multiply per product (v_mad_u64_u32) instead of separate high and low halves
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// top 23 bits of a word -> uniform in (0,1), exact in fp32
__device__ __forceinline__ float unit_open(uint32_t w) {
    return ((float)(w >> 9) + 0.5f) * 0x1p-23f;
}

}  // namespace gg
