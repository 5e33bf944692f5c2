// probe_bandwidth.hip -- stand-alone bandwidth probe for MI355X (not part of libgg).
//
// Gives the practical ceilings the library's streaming kernels are judged against:
//   read   : sum a 6.17 GB fp32 buffer with 128-bit loads -- one 64 KiB chunk per block, resident
//            blocks with contiguous runs, resident blocks pulling items through an atomic ticket;
//            plain and non-temporal loads
//   reread : the same reader over a 64 / 128 / 256 MiB window, eight times (Infinity-Cache sized)
//   widen  : bf16 -> fp32 widening copy (2 B read + 4 B written per element)
//   copy   : fp32 y = c x (4 B read + 4 B written) as resident runs, one 64 / 16 KiB piece per block,
//            grid-strided 256 KiB tiles; write-only fill; the runtime's own device copy
//   publish: the same reader with Σ|x| and Σx² combined per block and stored (one barrier pair), or stored
//            per wave (no barrier), at 8 .. 368 runs per compute unit
//   spread : finish-time spread of resident blocks with equal contiguous shares
// Usage: probe_bandwidth [elements]   (default 1543655424).  Prints one line per experiment.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

typedef float vf4 __attribute__((ext_vector_type(4)));
typedef unsigned vu2 __attribute__((ext_vector_type(2)));
constexpr int kBlock = 256, kChunkVec = 4096;   // 64 KiB chunks

template <int U, bool NT>
__device__ __forceinline__ float chunk_sum(const vf4 *__restrict__ p, int nvec) {
    float s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    int i = threadIdx.x;
    for (; i + (U - 1) * kBlock < nvec; i += U * kBlock) {
        vf4 r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = NT ? __builtin_nontemporal_load(p + i + u * kBlock) : p[i + u * kBlock];
#pragma unroll
        for (int u = 0; u < U; ++u) { s0 += fabsf(r[u].x); s1 += fabsf(r[u].y); s2 += fabsf(r[u].z); s3 += fabsf(r[u].w); }
    }
    for (; i < nvec; i += kBlock) { const vf4 r = p[i]; s0 += r.x; s1 += r.y; s2 += r.z; s3 += r.w; }
    return (s0 + s1) + (s2 + s3);
}

__device__ __forceinline__ int chunk_len(long c, long nvec) {
    const long rest = nvec - c * kChunkVec;
    return (int)(rest < kChunkVec ? rest : kChunkVec);
}

// contiguous run of `cpb` chunks per block (cpb = 1 with one block per chunk: the many-blocks shape)
template <bool NT>
__global__ __launch_bounds__(kBlock) void k_runs(const vf4 *__restrict__ x, long nchunks, long nvec, int cpb, double *out,
                                                 long long *stamps) {
    const long long t0 = wall_clock64();
    double acc = 0;
    const long first = (long)blockIdx.x * cpb;
    long last = first + cpb;
    if (last > nchunks) last = nchunks;
    for (long c = first; c < last; ++c) acc += chunk_sum<8, NT>(x + c * kChunkVec, chunk_len(c, nvec));
    if (acc == 123.456) out[blockIdx.x] = acc;
    if (stamps) {
        __syncthreads();
        if (threadIdx.x == 0) { stamps[2 * blockIdx.x] = t0; stamps[2 * blockIdx.x + 1] = wall_clock64(); }
    }
}

// The same reader with the block -> run map made XCD-aware: workgroups are dealt to the 8 XCDs round-robin
// (workgroup b runs on XCD b mod 8), so run = (b mod 8) * (runs / 8) + b / 8 gives every XCD one contiguous
// eighth of the buffer; the plain map (run = b) interleaves the XCDs run by run.
__global__ __launch_bounds__(kBlock) void k_runs_xcd(const vf4 *__restrict__ x, long nchunks, long nvec, int cpb, long runs,
                                                     double *out) {
    const long per = (runs + 7) / 8;
    const long run = (long)(blockIdx.x & 7) * per + (blockIdx.x >> 3);
    double acc = 0;
    const long first = run * cpb;
    long last = first + cpb;
    if (last > nchunks) last = nchunks;
    if ((long)(blockIdx.x >> 3) < per)
        for (long c = first; c < last; ++c) acc += chunk_sum<8, true>(x + c * kChunkVec, chunk_len(c, nvec));
    if (acc == 123.456) out[blockIdx.x] = acc;
}

// the reader with a result per block: EPI 0 nothing stored, 1 block reduction + one store, 2 one store per wave
template <int EPI>
__global__ __launch_bounds__(kBlock) void k_publish(const vf4 *__restrict__ x, long nchunks, long nvec, int cpb, double *out) {
    __shared__ double red[4];
    const long first = (long)blockIdx.x * cpb;
    long last = first + cpb;
    if (last > nchunks) last = nchunks;
    double acc = 0;
    for (long c = first; c < last; ++c) acc += chunk_sum<8, true>(x + c * kChunkVec, chunk_len(c, nvec));
    if (EPI == 0) { if (acc == 123.456) out[blockIdx.x] = acc; return; }
    for (int d = 32; d; d >>= 1) acc += __shfl_xor(acc, d, 64);
    if (EPI == 2) { if ((threadIdx.x & 63) == 0) out[4 * first + (threadIdx.x >> 6)] = acc; return; }
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) out[first] = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
}

// resident blocks pulling items of `item_chunks` chunks through an atomic ticket
__global__ __launch_bounds__(kBlock) void k_ticket(const vf4 *__restrict__ x, long nchunks, long nvec, int item_chunks,
                                                   unsigned *counter, double *out) {
    __shared__ unsigned s_next;
    double acc = 0;
    const long nitems = (nchunks + item_chunks - 1) / item_chunks;
    for (;;) {
        if (threadIdx.x == 0) s_next = atomicAdd(counter, 1u);
        __syncthreads();
        const unsigned item = s_next;
        __syncthreads();
        if (item >= nitems) break;   // the counter only grows: every block leaves after at most nitems+1 pulls
        const long c0 = (long)item * item_chunks;
        long c1 = c0 + item_chunks;
        if (c1 > nchunks) c1 = nchunks;
        for (long c = c0; c < c1; ++c) acc += chunk_sum<8, true>(x + c * kChunkVec, chunk_len(c, nvec));
    }
    if (acc == 123.456) out[blockIdx.x] = acc;
}

// bf16 -> fp32 widening copy: 8-byte loads, one 16-byte streaming store per lane
__global__ __launch_bounds__(kBlock) void k_widen(const vu2 *__restrict__ x, vf4 *__restrict__ y, long nvec, long vec_per_block) {
    const long base = (long)blockIdx.x * vec_per_block;
    long end = vec_per_block;
    if (base + end > nvec) end = nvec - base;
    const vu2 *p = x + base;
    vf4 *q = y + base;
    constexpr int U = 8;
    long i = threadIdx.x;
    for (; i + (U - 1) * kBlock < end; i += U * kBlock) {
        vu2 r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = __builtin_nontemporal_load(p + i + u * kBlock);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const vf4 o = {__uint_as_float(r[u].x << 16), __uint_as_float(r[u].x & 0xffff0000u), __uint_as_float(r[u].y << 16),
                           __uint_as_float(r[u].y & 0xffff0000u)};
            __builtin_nontemporal_store(o, q + i + u * kBlock);
        }
    }
    for (; i < end; i += kBlock) {
        const vu2 r = __builtin_nontemporal_load(p + i);
        const vf4 o = {__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u), __uint_as_float(r.y << 16),
                       __uint_as_float(r.y & 0xffff0000u)};
        __builtin_nontemporal_store(o, q + i);
    }
}

// y = c x over [0, nvec) vectors: block b takes `vpb` consecutive vectors, or (stride > 0) tiles b, b + grid, ...
template <bool NTS>
__global__ __launch_bounds__(kBlock) void k_copy(const vf4 *__restrict__ x, vf4 *__restrict__ y, long nvec, long vpb, int strided, float c) {
    constexpr int U = 4;
    const long ntiles = (nvec + vpb - 1) / vpb;
    for (long t = blockIdx.x; t < ntiles; t += strided ? gridDim.x : ntiles) {
        const long base = t * vpb;
        long end = vpb;
        if (base + end > nvec) end = nvec - base;
        const vf4 *p = x + base;
        vf4 *q = y + base;
        long i = threadIdx.x;
        for (; i + (U - 1) * kBlock < end; i += U * kBlock) {
            vf4 r[U];
#pragma unroll
            for (int u = 0; u < U; ++u) r[u] = __builtin_nontemporal_load(p + i + u * kBlock);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const vf4 o = r[u] * c;
                if (NTS) __builtin_nontemporal_store(o, q + i + u * kBlock); else q[i + u * kBlock] = o;
            }
        }
        for (; i < end; i += kBlock) q[i] = p[i] * c;
    }
}

__global__ __launch_bounds__(kBlock) void k_fill(vf4 *__restrict__ y, long nvec, long vpb, float c) {
    const long base = (long)blockIdx.x * vpb;
    if (base >= nvec) return;
    long end = vpb;
    if (base + end > nvec) end = nvec - base;
    const vf4 o = {c, c, c, c};
    for (long i = threadIdx.x; i < end; i += kBlock) __builtin_nontemporal_store(o, y + base + i);
}

__global__ void k_init(float *x, long n) {
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) x[i] = (float)(i & 1023) * 1e-3f;
}

template <typename F>
static float timeit(F f, int reps) {
    hipEvent_t a, b;
    CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    f(); CK(hipDeviceSynchronize());
    CK(hipEventRecord(a));
    for (int i = 0; i < reps; ++i) f();
    CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
    float ms;
    CK(hipEventElapsedTime(&ms, a, b));
    return ms / reps;
}

int main(int argc, char **argv) {
    const long n = argc > 1 ? atol(argv[1]) : 1543655424L;
    float *x, *y; double *out; unsigned *ctr; long long *stamps;
    CK(hipMalloc(&x, n * 4)); CK(hipMalloc(&y, n * 4)); CK(hipMalloc(&out, (size_t)(n / 4 / kChunkVec + 8) * 4 * sizeof(double))); CK(hipMalloc(&ctr, 256));
    CK(hipMalloc(&stamps, 1 << 20));
    k_init<<<4096, 256>>>(x, n);
    CK(hipDeviceSynchronize());
    const long nvec = n / 4, nchunks = (nvec + kChunkVec - 1) / kChunkVec;
    const double gb = n * 4.0 / 1e9;
    const int reps = 10;
    float ms;
    ms = timeit([&] { k_runs<false><<<nchunks, kBlock>>>((const vf4 *)x, nchunks, nvec, 1, out, nullptr); }, reps);
    printf("read  one chunk per block (%ld blocks), plain loads        %.3f ms %7.1f GB/s\n", nchunks, ms, gb / ms * 1e3);
    ms = timeit([&] { k_runs<true><<<nchunks, kBlock>>>((const vf4 *)x, nchunks, nvec, 1, out, nullptr); }, reps);
    printf("read  one chunk per block (%ld blocks), non-temporal       %.3f ms %7.1f GB/s\n", nchunks, ms, gb / ms * 1e3);
    for (int G : {1536, 2048}) {
        const int cpb = (int)((nchunks + G - 1) / G);
        ms = timeit([&] { k_runs<true><<<G, kBlock>>>((const vf4 *)x, nchunks, nvec, cpb, out, nullptr); }, reps);
        printf("read  %4d resident blocks, contiguous runs, non-temporal   %.3f ms %7.1f GB/s\n", G, ms, gb / ms * 1e3);
        ms = timeit([&] { k_runs<false><<<G, kBlock>>>((const vf4 *)x, nchunks, nvec, cpb, out, nullptr); }, reps);
        printf("read  %4d resident blocks, contiguous runs, plain loads    %.3f ms %7.1f GB/s\n", G, ms, gb / ms * 1e3);
    }
    for (int rpc : {8, 32, 128}) {
        const long G = 256L * rpc;
        const int cpb = (int)((nchunks + G - 1) / G);
        const long runs = (nchunks + cpb - 1) / cpb, grid = (runs + 7) / 8 * 8;
        const float plain = timeit([&] { k_runs<true><<<runs, kBlock>>>((const vf4 *)x, nchunks, nvec, cpb, out, nullptr); }, reps);
        const float xcd = timeit([&] { k_runs_xcd<<<grid, kBlock>>>((const vf4 *)x, nchunks, nvec, cpb, runs, out); }, reps);
        printf("read  %3d runs/CU, run = block: %.3f ms %7.1f GB/s | one contiguous eighth per XCD: %.3f ms %7.1f GB/s\n", rpc, plain,
               gb / plain * 1e3, xcd, gb / xcd * 1e3);
    }
    for (int item : {1, 4, 16}) {
        float tot = 0;
        for (int r = 0; r <= reps; ++r) {   // the ticket counter is cleared outside the timed region; run 0 is a warm-up
            CK(hipMemset(ctr, 0, 4));
            hipEvent_t a, b;
            CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
            CK(hipEventRecord(a));
            k_ticket<<<2048, kBlock>>>((const vf4 *)x, nchunks, nvec, item, ctr, out);
            CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
            float t;
            CK(hipEventElapsedTime(&t, a, b));
            if (r) tot += t;
            CK(hipEventDestroy(a)); CK(hipEventDestroy(b));
        }
        printf("read  2048 resident blocks, ticketed items of %4d KiB        %.3f ms %7.1f GB/s\n", item * 64, tot / reps, gb / (tot / reps) * 1e3);
    }
    for (long mb : {64L, 128L, 256L}) {
        const long nv = mb * 1024 * 1024 / 16, nc = nv / kChunkVec;
        ms = timeit([&] { for (int r = 0; r < 8; ++r) k_runs<true><<<nc, kBlock>>>((const vf4 *)x, nc, nv, 1, out, nullptr); }, 5);
        printf("reread %3ld MiB window x8, non-temporal                       %.4f ms %7.1f GB/s\n", mb, ms, 8 * mb * 1.048576 / ms);
    }
    {
        const long ne = n / 2 * 2, nv = ne / 4;   // ne bf16 elements in x (2 B each), ne fp32 out
        const long G = 2048, vpb = (nv + G - 1) / G;
        ms = timeit([&] { k_widen<<<G, kBlock>>>((const vu2 *)x, (vf4 *)y, nv, vpb); }, 5);
        printf("widen bf16->fp32, 2048 resident blocks (2 B in + 4 B out)     %.3f ms %7.1f GB/s\n", ms, ne * 6.0 / 1e9 / ms * 1e3);
        const long G2 = 131072, vpb2 = (nv + G2 - 1) / G2;
        ms = timeit([&] { k_widen<<<G2, kBlock>>>((const vu2 *)x, (vf4 *)y, nv, vpb2); }, 5);
        printf("widen bf16->fp32, 131072 short blocks                         %.3f ms %7.1f GB/s\n", ms, ne * 6.0 / 1e9 / ms * 1e3);
    }
    {
        const double gb2 = n * 8.0 / 1e9;
        const long G = 2048, vpb = ((nvec + G - 1) / G + 255) / 256 * 256;
        ms = timeit([&] { k_copy<true><<<G, kBlock>>>((const vf4 *)x, (vf4 *)y, nvec, vpb, 0, 1.5f); }, 5);
        printf("copy  fp32, 2048 resident blocks, contiguous runs             %.3f ms %7.1f GB/s\n", ms, gb2 / ms * 1e3);
        ms = timeit([&] { k_copy<false><<<G, kBlock>>>((const vf4 *)x, (vf4 *)y, nvec, vpb, 0, 1.5f); }, 5);
        printf("copy  fp32, 2048 resident blocks, plain stores                %.3f ms %7.1f GB/s\n", ms, gb2 / ms * 1e3);
        ms = timeit([&] { k_copy<true><<<G, kBlock>>>((const vf4 *)x, (vf4 *)y, nvec, 16384, 1, 1.5f); }, 5);
        printf("copy  fp32, 2048 blocks grid-strided over 256 KiB tiles       %.3f ms %7.1f GB/s\n", ms, gb2 / ms * 1e3);
        for (long piece : {4096L, 1024L}) {
            const long nb = (nvec + piece - 1) / piece;
            ms = timeit([&] { k_copy<true><<<nb, kBlock>>>((const vf4 *)x, (vf4 *)y, nvec, piece, 0, 1.5f); }, 5);
            printf("copy  fp32, one %2ld KiB piece per block (%ld blocks)        %.3f ms %7.1f GB/s\n", piece * 16 / 1024, nb, ms, gb2 / ms * 1e3);
        }
        ms = timeit([&] { CK(hipMemcpyAsync(y, x, n * 4, hipMemcpyDeviceToDevice, 0)); }, 5);
        printf("copy  the runtime's device-to-device copy                     %.3f ms %7.1f GB/s\n", ms, gb2 / ms * 1e3);
        ms = timeit([&] { k_fill<<<G, kBlock>>>((vf4 *)y, nvec, vpb, 2.f); }, 5);
        printf("fill  fp32, 2048 resident blocks (write only)                 %.3f ms %7.1f GB/s\n", ms, gb / ms * 1e3);
    }
    for (int rpc : {8, 32, 64, 128, 368}) {
        const long G = 256L * rpc;
        const int cpb = (int)((nchunks + G - 1) / G);
        const long blocks = (nchunks + cpb - 1) / cpb;
        const float t0 = timeit([&] { k_publish<0><<<blocks, kBlock>>>((const vf4 *)x, nchunks, nvec, cpb, out); }, reps);
        const float t1 = timeit([&] { k_publish<1><<<blocks, kBlock>>>((const vf4 *)x, nchunks, nvec, cpb, out); }, reps);
        const float t2 = timeit([&] { k_publish<2><<<blocks, kBlock>>>((const vf4 *)x, nchunks, nvec, cpb, out); }, reps);
        printf("publish %3d runs/CU (%6ld blocks x %2d chunks): nothing stored %.3f ms | per block %.3f ms | per wave %.3f ms\n", rpc,
               blocks, cpb, t0, t1, t2);
    }
    {
        const int G = 2048, cpb = (int)((nchunks + G - 1) / G);
        k_runs<true><<<G, kBlock>>>((const vf4 *)x, nchunks, nvec, cpb, out, stamps);
        CK(hipDeviceSynchronize());
        std::vector<long long> h(2 * G);
        CK(hipMemcpy(h.data(), stamps, 2 * G * sizeof(long long), hipMemcpyDeviceToHost));
        long long s0 = h[0];
        for (int b = 0; b < G; ++b) s0 = std::min(s0, h[2 * b]);
        std::vector<double> en;
        for (int b = 0; b < G; ++b) en.push_back((h[2 * b + 1] - s0) / 100.0);   // 100 MHz clock -> us
        std::sort(en.begin(), en.end());
        printf("spread of block finish times, 2048 equal contiguous runs: min %.0f p10 %.0f p50 %.0f p90 %.0f max %.0f us\n",
               en[0], en[G / 10], en[G / 2], en[G * 9 / 10], en.back());
    }
    return 0;
}
