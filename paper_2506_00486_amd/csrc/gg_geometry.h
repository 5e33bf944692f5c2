// gg_geometry.h -- how a buffer is cut into units, chunks and runs, on the device (SegView,
// locate, RunCursor) and on the host (argument validation, workspace layout, table upload,
// occupancy-aware run split).  Shared by the translation units of libgg.
#pragma once

#include <hip/hip_runtime.h>
#include <mutex>
#include <stdint.h>
#include <string.h>

#include <type_traits>

#include "../../include/gg.h"
#include "gg_device.h"

namespace gg {

// ---------------------------------------------------------------------------------------------
// unit geometry
// ---------------------------------------------------------------------------------------------
struct SegView {
    const int64_t *off;    // device: S+1 element offsets, or nullptr for uniform rows
    const int32_t *cpre;   // device: S+1 chunk prefix sums (with off)
    int64_t cols;          // uniform: elements per row
    int64_t cpr;           // uniform: chunks per row
    int32_t S;
};

struct ChunkLoc {
    int64_t start;   // first element
    int64_t c;       // chunk index inside the unit
    int32_t seg;
    int32_t len;
};

__device__ __forceinline__ ChunkLoc locate(const SegView &sv, int64_t chunk) {
    ChunkLoc L;
    if (sv.off == nullptr) {
        const int64_t seg = chunk / sv.cpr;
        L.c = chunk - seg * sv.cpr;
        L.seg = (int32_t)seg;
        L.start = seg * sv.cols + L.c * kChunk;
        const int64_t rest = sv.cols - L.c * kChunk;
        L.len = (int32_t)(rest < kChunk ? rest : kChunk);
    } else {
        // Largest s with cpre[s] <= chunk (skips empty units).  Every lane of the wave asks for the same chunk
        // (the callers are uniform over the block), so the wave probes 64 places at once: two dependent loads
        // for a few thousand units instead of a dozen -- a block's first load waits for this.
        const int lane = threadIdx.x & 63;
        int lo = 0, hi = sv.S;
        while (hi - lo > 1) {
            const int step = (hi - lo + 63) >> 6;
            const int idx = lo + (lane + 1) * step;
            const bool le = idx < hi && sv.cpre[idx] <= chunk;
            const int cnt = (int)__popcll(__ballot(le));     // the probes not above the chunk are a prefix of the lanes
            lo += cnt * step;
            hi = lo + step < hi ? lo + step : hi;
        }
        L.seg = lo;
        L.c = chunk - sv.cpre[lo];
        L.start = sv.off[lo] + L.c * kChunk;
        const int64_t rest = sv.off[lo + 1] - L.start;
        L.len = (int32_t)(rest < kChunk ? rest : kChunk);
    }
    return L;
}

__device__ __forceinline__ int64_t unit_len(const SegView &sv, int seg) {
    return sv.off ? sv.off[seg + 1] - sv.off[seg] : sv.cols;
}
__device__ __forceinline__ int64_t unit_chunk0(const SegView &sv, int seg) {
    return sv.off ? sv.cpre[seg] : (int64_t)seg * sv.cpr;
}
__device__ __forceinline__ int64_t unit_chunk1(const SegView &sv, int seg) {
    return sv.off ? sv.cpre[seg + 1] : (int64_t)(seg + 1) * sv.cpr;
}

__device__ __forceinline__ int64_t unit_end(const SegView &sv, int seg) {
    return sv.off ? sv.off[seg + 1] : (int64_t)(seg + 1) * sv.cols;
}

// Walks the consecutive chunks [first, last) a block owns; the unit table is searched only when
// the walk crosses into another unit.
// Element-wise sweeps let `parts` blocks share a chunk: part p takes elements [p, p+1) * kChunk/parts of it.
__device__ __forceinline__ bool chunk_part(int64_t start, int len, int part, int parts, int64_t &pstart, int &plen) {
    const int piece = kChunk / parts, lo = part * piece;
    if (lo >= len) return false;
    pstart = start + lo;
    plen = len - lo < piece ? len - lo : piece;
    return true;
}

struct RunCursor {
    ChunkLoc L;
    int64_t chunk, last, seg_chunks;
    __device__ __forceinline__ void init(const SegView &sv, int64_t first, int64_t last_) {
        chunk = first; last = last_;
        L = locate(sv, first);
        seg_chunks = unit_chunk1(sv, L.seg) - unit_chunk0(sv, L.seg);
    }
    __device__ __forceinline__ bool valid() const { return chunk < last; }
    __device__ __forceinline__ void next(const SegView &sv) {
        if (++chunk >= last) return;
        if (L.c + 1 < seg_chunks) {
            L.c += 1;
            L.start += kChunk;
            const int64_t rest = unit_end(sv, L.seg) - L.start;
            L.len = (int32_t)(rest < kChunk ? rest : kChunk);
        } else {
            L = locate(sv, chunk);
            seg_chunks = unit_chunk1(sv, L.seg) - unit_chunk0(sv, L.seg);
        }
    }
};

// per-unit parameters of the second sweep
constexpr uint32_t kSkipRate = 1u;   // no usable step: symbols 0, nothing accumulated
constexpr uint32_t kPenZero = 2u;    // alpha == 0: penalty contributes 0
struct SegParam {
    float inv_delta;
    float delta;
    float pen_coef;    // lambda * beta / alpha
    float inv_alpha;
    float beta_m1;
    uint32_t flags;
    uint32_t ticket;   // how many workgroups of the unit's finalisation have delivered their part (starts at 0)
    uint32_t _pad;
};

// ---------------------------------------------------------------------------------------------
// small utility kernels
// ---------------------------------------------------------------------------------------------
constexpr int kPackI64 = 448;  // 3584 bytes of kernel arguments per launch
struct PackI64 { int64_t v[kPackI64]; };
constexpr int kTableThreads = 1024;

// Chunk prefix of a unit table, by one workgroup of kTableThreads: cpre[s] = chunks of the units before s,
// cpre[S] = all of them.  A thread takes a contiguous range of units; the range totals are scanned across
// the block (wave scan, wave totals through LDS) and every thread then writes its own range.
__device__ __forceinline__ int32_t unit_chunks(const int64_t *off, int s) {
    return (int32_t)((off[s + 1] - off[s] + kChunk - 1) / kChunk);
}
__device__ __forceinline__ void chunk_prefix_block(const int64_t *off, int32_t S, int32_t *cpre) {
    __shared__ int32_t wave_tot[kTableThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = (S + kTableThreads - 1) / kTableThreads;
    const int s0 = tid * per < S ? tid * per : S, s1 = s0 + per < S ? s0 + per : S;
    int32_t mine = 0;
    for (int s = s0; s < s1; ++s) mine += unit_chunks(off, s);
    int32_t incl = mine;                       // inclusive scan over the wave
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int32_t up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int32_t before = 0;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    int32_t run = before + incl - mine;
    for (int s = s0; s < s1; ++s) { cpre[s] = run; run += unit_chunks(off, s); }
    if (tid == kTableThreads - 1) cpre[S] = run;   // the last thread's range ends the table (possibly empty)
}

// `count` table words out of the kernel arguments to dst; the launch that carries the last words of a unit
// table (cpre != nullptr) also derives the chunk prefix from the complete table `off`.
static __global__ __launch_bounds__(kTableThreads) void k_upload_i64(PackI64 pack, int count, int64_t *dst,
                                                                     const int64_t *off, int32_t S, int32_t *cpre) {
    for (int i = threadIdx.x; i < count; i += kTableThreads) dst[i] = pack.v[i];
    if (cpre) {
        __syncthreads();                       // this block's own stores; earlier words came from earlier launches
        chunk_prefix_block(off, S, cpre);
    }
}

static __global__ void k_fill_u64(uint64_t *p, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = 0;
}


// =============================================================================================
// host side
// =============================================================================================
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

constexpr int kSolveTable = 4096;   // intervals of the tabulated moment-ratio curve (gen_solve_curve.py reads this line)

// What one run contributes to the rate record of a unit that several runs share; a later kernel folds the
// slots into the record, so the sweep needs no atomics on a record that hundreds of blocks finish on at the
// same time.  A run shares at most two units with other runs: the one it starts in (slot 2 run) and the one
// it ends in (slot 2 run + 1); a piece that starts with the run takes the first.
struct RatePiece {
    uint64_t bits;           // sum of code lengths
    uint64_t n_clamped;      // a run of a very large unit can hold more than 2^32 clamped elements
    uint32_t u_max, flags, _pad[2];
};
static_assert(sizeof(RatePiece) == 32, "two 16-byte stores");
constexpr int64_t kMaxRuns = 256 * 512;  // most blocks a reducing sweep is split into

// A rate sweep that also writes a stream (penalty gradient, symbols) runs as short blocks, kStreamParts per
// chunk, like the element-wise sweeps; every such block leaves its sums in a slot of its own (block index =
// chunk * kStreamParts + part), and one workgroup per unit folds the unit's slots, which are consecutive.
struct PartSlot { uint32_t bits, u_max, flags, n_clamped; };   // n_clamped: symbols past the last bin (with a histogram)
static_assert(sizeof(PartSlot) == 16, "one 16-byte store");
#ifndef GG_STREAM_PARTS
#define GG_STREAM_PARTS 4                // 4096 elements per block = 256 lanes x 4 loads x 4 elements
#endif
constexpr int kStreamParts = GG_STREAM_PARTS;
static_assert(kStreamParts * sizeof(PartSlot) <= 2 * sizeof(RatePiece), "the slot area is sized as two run slots per chunk");

struct WsLayout {
    size_t off_bytes, params_bytes, partials_bytes, pieces_bytes, total;   // off_bytes: offsets + chunk prefix
    size_t off_at, params_at, partials_at, pieces_at;
};

static WsLayout ws_layout(int64_t n_total, int64_t n_units) {
    WsLayout w;
    const size_t S = (size_t)n_units;
    const size_t max_chunks = (size_t)(n_total / kChunk) + S + 1;
    w.off_bytes = align_up((S + 1) * sizeof(int64_t) + ((S + 2) / 2) * sizeof(int64_t), 256);
    w.params_bytes = align_up(S * sizeof(SegParam), 256);
    w.partials_bytes = align_up(max_chunks * sizeof(double2), 256);
    w.off_at = 256;
    w.params_at = w.off_at + w.off_bytes;
    w.partials_at = w.params_at + w.params_bytes;
    w.pieces_bytes = align_up(max_chunks * 2 * sizeof(RatePiece), 256);   // runs <= chunks; or kStreamParts part slots per chunk
    w.pieces_at = w.partials_at + w.partials_bytes;
    w.total = w.pieces_at + w.pieces_bytes;
    return w;
}

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline bool aligned8(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 7u) == 0; }

constexpr int64_t kMaxUnits = 1 << 24;      // rows of a matrix
constexpr int64_t kMaxSegments = 1 << 17;   // units of a flat bucket (293 table launches)
constexpr int64_t kMaxChunks = 2147483647LL;

// A validated description of how a buffer is cut into units, plus where its tables live.
struct Geometry {
    SegView sv{};
    int64_t n_total = 0, n_chunks = 0;
    int32_t S = 0;
    WsLayout wl{};
    char *ws = nullptr;
    const int64_t *host_off = nullptr;   // the caller's S+1 element offsets (segmented only); the chunk prefix sums
                                         // that follow them in the workspace are derived on the device
    SegParam *params() const { return reinterpret_cast<SegParam *>(ws + wl.params_at); }
    double2 *partials() const { return reinterpret_cast<double2 *>(ws + wl.partials_at); }
    RatePiece *rate_pieces() const { return reinterpret_cast<RatePiece *>(ws + wl.pieces_at); }
    PartSlot *part_slots() const { return reinterpret_cast<PartSlot *>(ws + wl.pieces_at); }
};

static int geometry_uniform(int64_t rows, int64_t cols, void *ws, size_t ws_bytes, bool need_ws, Geometry &g) {
    if (rows < 0 || cols < 0 || rows > kMaxUnits) return GG_ERR_INVALID_ARG;
    if (rows > 0 && cols > INT64_MAX / rows) return GG_ERR_INVALID_ARG;
    g.S = (int32_t)rows;
    g.n_total = rows * cols;
    const int64_t cpr = (cols + kChunk - 1) / kChunk;
    if (cpr > 0 && rows > kMaxChunks / cpr) return GG_ERR_INVALID_ARG;
    g.n_chunks = rows * cpr;
    g.sv.off = nullptr; g.sv.cpre = nullptr; g.sv.cols = cols; g.sv.cpr = cpr; g.sv.S = g.S;
    g.wl = ws_layout(g.n_total, rows > 0 ? rows : 1);
    if (need_ws) {
        if (!ws || ws_bytes < g.wl.total || !aligned16(ws)) return GG_ERR_WORKSPACE;
        g.ws = static_cast<char *>(ws);
    }
    return GG_OK;
}

// `single_as_uniform`: a bucket of one unit that starts at element 0 is a plain tensor; described as one (no
// unit table to upload, no search in the kernels) when the caller's kernels need no table on the device.
static int geometry_segmented(const int64_t *offsets, int32_t S, void *ws, size_t ws_bytes, Geometry &g,
                              bool single_as_uniform = false) {
    // the unit table travels through kernel arguments (448 offsets per launch): keep it to a few hundred launches
    if (!offsets || S < 0 || S > kMaxSegments) return S < 0 || !offsets ? GG_ERR_INVALID_ARG : GG_ERR_BAD_SEGMENTS;
    if (offsets[0] < 0) return GG_ERR_BAD_SEGMENTS;
    if (single_as_uniform && S == 1 && offsets[0] == 0) {
        if (offsets[1] < 0) return GG_ERR_BAD_SEGMENTS;
        const int rc = geometry_uniform(1, offsets[1], ws, ws_bytes, true, g);
        return rc == GG_ERR_INVALID_ARG ? GG_ERR_BAD_SEGMENTS : rc;
    }
    g.S = S;
    g.host_off = offsets;
    const size_t n_off = (size_t)S + 1;
    int64_t chunks = 0;
    for (int32_t s = 0; s < S; ++s) {
        if (offsets[s + 1] < offsets[s]) return GG_ERR_BAD_SEGMENTS;
        chunks += (offsets[s + 1] - offsets[s] + kChunk - 1) / kChunk;
        if (chunks > kMaxChunks) return GG_ERR_BAD_SEGMENTS;
    }
    g.n_chunks = chunks;
    g.n_total = S > 0 ? offsets[S] : 0;   // elements of the buffer the units index into (none without units)
    g.wl = ws_layout(g.n_total, S > 0 ? S : 1);
    if (!ws || ws_bytes < g.wl.total || !aligned16(ws)) return GG_ERR_WORKSPACE;
    g.ws = static_cast<char *>(ws);
    g.sv.off = reinterpret_cast<const int64_t *>(g.ws + g.wl.off_at);
    g.sv.cpre = reinterpret_cast<const int32_t *>(g.ws + g.wl.off_at + n_off * sizeof(int64_t));
    g.sv.cols = 0; g.sv.cpr = 1; g.sv.S = S;
    return GG_OK;
}

static int check_launch() { return hipGetLastError() == hipSuccess ? GG_OK : GG_ERR_HIP; }

// The unit table travels as kernel arguments, straight from the caller's array: asynchronous, no staging
// buffer, no allocation on either side.  The last launch also writes the chunk prefix sums behind the offsets.
static int upload_geometry(const Geometry &g, hipStream_t st) {
    if (g.sv.off == nullptr) return GG_OK;
    int64_t *dst = const_cast<int64_t *>(g.sv.off);
    const size_t words = (size_t)g.S + 1;
    for (size_t base = 0; base < words; base += kPackI64) {
        PackI64 pack;
        const int count = (int)((words - base) < (size_t)kPackI64 ? words - base : kPackI64);
        memcpy(pack.v, g.host_off + base, (size_t)count * sizeof(int64_t));
        const bool last = base + kPackI64 >= words;
        hipLaunchKernelGGL(k_upload_i64, dim3(1), dim3(kTableThreads), 0, st, pack, count, dst + base, g.sv.off, g.S,
                           last ? const_cast<int32_t *>(g.sv.cpre) : (int32_t *)nullptr);
    }
    return check_launch();
}

template <typename F>
static int by_dtype(int dtype, F &&f) {
    if (dtype == GG_F32) return f(static_cast<const float *>(nullptr));
    if (dtype == GG_BF16) return f(static_cast<const bf16_t *>(nullptr));
    return GG_ERR_BAD_DTYPE;
}

// Static split of the chunk list into one run per block: `blocks_per_cu` resident blocks on each
// of the 256 compute units, every block a contiguous range of chunks.
constexpr int kComputeUnits = 256;
constexpr int kManyUnits = 2048;   // from here on the finalisation uses one lane per unit instead of one wave
struct RunSplit { int64_t blocks; int32_t chunks_per_block; };
static RunSplit split_runs(int64_t n_chunks, int blocks_per_cu) {
    const int64_t target = (int64_t)kComputeUnits * blocks_per_cu;
    int64_t cpb = (n_chunks + target - 1) / target;
    if (cpb < 1) cpb = 1;
    return RunSplit{(n_chunks + cpb - 1) / cpb, (int32_t)cpb};
}

// Workgroups of `threads` threads and `dyn_lds` bytes of dynamic LDS of `kernel` that fit a compute unit: a pure
// function of the code object and the device, but a question to the runtime that costs microseconds, so the answers
// are kept (a small table under a lock; a full table forgets its oldest entry).  The value only sizes grids.
static int workgroups_per_cu(const void *kernel, int threads, size_t dyn_lds) {
    struct Entry { const void *kernel; size_t lds; int threads, dev, n; };
    static Entry table[64];
    static int used = 0, next = 0;
    static std::mutex lock;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); dev = -1; }
    {
        std::lock_guard<std::mutex> hold(lock);
        for (int i = 0; i < used; ++i)
            if (table[i].kernel == kernel && table[i].lds == dyn_lds && table[i].threads == threads && table[i].dev == dev) return table[i].n;
    }
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, threads, dyn_lds) != hipSuccess || n < 1) { (void)hipGetLastError(); n = 1; }
    std::lock_guard<std::mutex> hold(lock);
    const int at = used < 64 ? used++ : (next = (next + 1) % 64);
    table[at] = Entry{kernel, dyn_lds, threads, dev, n};
    return n;
}

// resident blocks of `kernel` per compute unit, capped at `cap`
template <typename K>
static int resident_blocks(K kernel, size_t dyn_lds, int cap) {
    const int n = workgroups_per_cu(reinterpret_cast<const void *>(kernel), kBlock, dyn_lds);
    return n < cap ? n : cap;
}

static int launch_fill_u64(uint64_t *p, int64_t n, hipStream_t st) {
    if (n <= 0) return GG_OK;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_fill_u64, dim3((unsigned)blocks), dim3(256), 0, st, p, n);
    return check_launch();
}

}  // namespace gg
