// libpf_probe: latency-floor probes for the measurement harness (bench.py --mode floors).
// Not part of the product path: tiny kernels whose replayed-graph node time and event-stamped
// eager time show what a launch, a dependent memory round trip, a small stream and a
// grid-wide barrier cost on this part, so that the kernels of libpf can be priced against
// floors instead of against bytes alone.  gfx950 only.
#include "../../include/pf_probe.h"

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <vector>

namespace {

typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

__global__ void k_empty(int *sink)
{
    if (sink == nullptr && threadIdx.x == 12345) __builtin_trap();
}

// one memory round trip, then a store
__global__ void k_one_load(const int *__restrict__ a, int *__restrict__ b, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) b[i] = a[i] + 1;
}

// two dependent round trips, then a store
__global__ void k_two_loads(const int *__restrict__ a, const int *__restrict__ c, int *__restrict__ b, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) b[i] = c[a[i]] + 1;
}

// a chain of `hops` dependent loads by one lane: time / hops = one round trip
__global__ void k_chase(const int *__restrict__ next, int hops, int *__restrict__ out)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    int p = 0;
    for (int h = 0; h < hops; ++h) p = next[p];
    *out = p;
}

// the same over a region far larger than the caches: entry i lives in its own 128-byte line,
// and the entries form one cycle through all lines (full-period linear congruence)
__global__ void k_chase_init(int *__restrict__ region, uint32_t nlines)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nlines) region[(size_t)i * 32] = (int)((i * 1664525u + 1013904223u) & (nlines - 1));
}
__global__ void k_chase_cold(const int *__restrict__ region, int hops, int start, int *__restrict__ out)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    int p = start;
    for (int h = 0; h < hops; ++h) p = region[(size_t)p * 32];
    *out = p;
}

// plain stream: every thread keeps 8 16-byte non-temporal loads in flight
__global__ __launch_bounds__(256) void k_stream(const void *__restrict__ src, uint32_t bytes, int *__restrict__ sink)
{
    const rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(src), 0, (int)bytes, 0x00020000);
    const uint32_t nthreads = gridDim.x * blockDim.x;
    const uint32_t tid = blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t acc = 0;
    for (uint32_t base = 0; base < bytes; base += nthreads * 16u * 8u) {
        u32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = __builtin_amdgcn_raw_buffer_load_b128(r, (int)(base + ((uint32_t)u * nthreads + tid) * 16u), 0, 2);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9e3779b9u) *sink = 1;
}

// shader clock: cycle counter against the constant 100 MHz wall clock over a fixed spin
__global__ void k_clock(unsigned long long *out)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    const unsigned long long w0 = wall_clock64(), c0 = clock64();
    unsigned long long w1 = w0;
    while (w1 - w0 < 20000ull) w1 = wall_clock64();  // 200 us; ends whatever the clocks do
    out[0] = clock64() - c0;
    out[1] = w1 - w0;
}

__global__ void k_fill(uint32_t *p, int n, uint32_t v)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// ---- grid-wide barrier without device-scope fences ---------------------------------------
// Device-scope relaxed atomics only (they are performed at the memory side, so the per-XCD
// L2s need no write-back or invalidate), two levels: workgroups of a group of 16 count up
// the group's counter, the last arriver of a group counts up the top counter, everybody
// polls the top counter.  Every spin is bounded; a timed-out barrier raises a flag that makes
// all later barriers fall through, so the kernel always ends.
struct BarrierMem {
    uint32_t top;          // +0
    uint32_t pad0[63];
    uint32_t error;        // +256
    uint32_t pad1[63];
    uint32_t group[64 * 64];  // one 256-byte line per group
};

__device__ __forceinline__ uint32_t ld_dev(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(uint32_t *p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t add_dev(uint32_t *p, uint32_t v)
{
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int kGroupSize = 16;
constexpr uint32_t kSpinLimit = 1u << 20;

// gen = 1, 2, 3, ...: the number of this barrier since the counters were zeroed.
__device__ __forceinline__ void grid_barrier(BarrierMem *bm, uint32_t gen)
{
    // every thread's earlier stores have been acknowledged before the workgroup arrives
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t nwg = gridDim.x;
        const uint32_t grp = blockIdx.x / kGroupSize;
        const uint32_t ngrp = (nwg + kGroupSize - 1) / kGroupSize;
        const uint32_t in_grp = min((uint32_t)kGroupSize, nwg - grp * kGroupSize);
        if (ld_dev(&bm->error) == 0) {
            const uint32_t old = add_dev(&bm->group[grp * 64], 1u);
            if (old + 1 == gen * in_grp) add_dev(&bm->top, 1u);
            uint32_t spins = 0;
            while (ld_dev(&bm->top) < gen * ngrp) {
                if (++spins > kSpinLimit) {
                    st_dev(&bm->error, gen);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
        }
    }
    __syncthreads();
}

// nb barriers back to back; thread 0 of block 0 leaves the cycle count per barrier.
__global__ __launch_bounds__(256) void k_barriers(BarrierMem *bm, int nb, unsigned long long *ticks)
{
    const unsigned long long t0 = wall_clock64();
    for (int g = 1; g <= nb; ++g) grid_barrier(bm, (uint32_t)g);
    if (blockIdx.x == 0 && threadIdx.x == 0) ticks[0] = wall_clock64() - t0;
}

// Visibility of plain data across workgroups through the barrier: in round g every workgroup
// writes `words` values derived from (g, block) with device-scope stores, passes the barrier,
// and then reads the piece of another workgroup with device-scope loads; mismatches are counted.
__global__ __launch_bounds__(256) void k_exchange(BarrierMem *bm, uint32_t *data, int words, int rounds,
                                                  uint32_t *mismatches)
{
    uint32_t bad = 0;
    for (int g = 1; g <= rounds; ++g) {
        uint32_t *mine = data + (size_t)blockIdx.x * words;
        for (int i = threadIdx.x; i < words; i += blockDim.x)
            st_dev(&mine[i], (uint32_t)g * 0x9E3779B1u + blockIdx.x * 131u + (uint32_t)i);
        grid_barrier(bm, (uint32_t)(2 * g - 1));
        const uint32_t other = (blockIdx.x + 97u * (uint32_t)g) % gridDim.x;
        const uint32_t *theirs = data + (size_t)other * words;
        for (int i = threadIdx.x; i < words; i += blockDim.x)
            bad += ld_dev(&theirs[i]) != (uint32_t)g * 0x9E3779B1u + other * 131u + (uint32_t)i;
        grid_barrier(bm, (uint32_t)(2 * g));  // nobody overwrites before everybody has read
    }
    if (bad) atomicAdd(mismatches, bad);
}

#define PFP_HIP(call)                                                              \
    do {                                                                           \
        hipError_t e_ = (call);                                                    \
        if (e_ != hipSuccess) {                                                    \
            snprintf(g_err, sizeof(g_err), "%s: %s", #call, hipGetErrorString(e_)); \
            return 1;                                                              \
        }                                                                          \
    } while (0)

char g_err[256] = {0};

struct Buffers {
    int *a = nullptr, *b = nullptr, *c = nullptr;
    void *big = nullptr;
    BarrierMem *bm = nullptr;
    unsigned long long *ticks = nullptr;
    uint32_t *xdata = nullptr, *mism = nullptr;
    size_t big_bytes = 0;
    int n = 0;
};

}  // namespace

extern "C" {

const char *pfp_last_error(void) { return g_err; }

int pfp_measure(int kind, size_t bytes, int grid, int nodes, int reps, double *graph_us_per_node,
                double *eager_event_us, double *extra)
{
    if (!graph_us_per_node || !eager_event_us || nodes < 1 || reps < 1 || grid < 1) return 1;
    *graph_us_per_node = *eager_event_us = 0.0;
    if (extra) *extra = 0.0;
    Buffers B;
    B.n = grid * 256;
    hipStream_t st;
    PFP_HIP(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
    PFP_HIP(hipMalloc(&B.a, (size_t)B.n * 4));
    PFP_HIP(hipMalloc(&B.b, (size_t)B.n * 4));
    PFP_HIP(hipMalloc(&B.c, (size_t)B.n * 4));
    PFP_HIP(hipMalloc(&B.bm, sizeof(BarrierMem)));
    PFP_HIP(hipMalloc(&B.ticks, 64));
    PFP_HIP(hipMalloc(&B.mism, 64));
    PFP_HIP(hipMemset(B.mism, 0, 64));
    PFP_HIP(hipMemset(B.ticks, 0, 64));
    const int xwords = 1024;
    PFP_HIP(hipMalloc(&B.xdata, (size_t)grid * xwords * 4));
    {
        std::vector<int> h(B.n);
        for (int i = 0; i < B.n; ++i) h[i] = (int)(((long long)i * 7919 + 13) % B.n);
        PFP_HIP(hipMemcpy(B.a, h.data(), (size_t)B.n * 4, hipMemcpyHostToDevice));
        PFP_HIP(hipMemcpy(B.c, h.data(), (size_t)B.n * 4, hipMemcpyHostToDevice));
    }
    if (kind == PFP_STREAM) {
        if (bytes < 4096 || bytes >= (1ull << 31)) {
            snprintf(g_err, sizeof(g_err), "stream size out of range");
            return 1;
        }
        B.big_bytes = bytes;
        PFP_HIP(hipMalloc(&B.big, bytes));
        PFP_HIP(hipMemset(B.big, 1, bytes));
    }
    const int nb = (int)bytes;  // barrier / exchange probes: number of barriers or rounds
    if ((kind == PFP_BARRIERS || kind == PFP_EXCHANGE) && (nb < 0 || nb > 4096 || grid > 64 * kGroupSize)) {
        snprintf(g_err, sizeof(g_err), "barrier count or grid out of range");
        return 1;
    }
    const size_t region_bytes = 1ull << 30;  // cold probes: four times the last-level cache
    if (kind == PFP_STREAM_COLD || kind == PFP_CHASE_COLD) {
        if (kind == PFP_STREAM_COLD && (bytes < 4096 || bytes > region_bytes / 8)) {
            snprintf(g_err, sizeof(g_err), "stream size out of range");
            return 1;
        }
        B.big_bytes = bytes;
        PFP_HIP(hipMalloc(&B.big, region_bytes));
        if (kind == PFP_STREAM_COLD) {
            PFP_HIP(hipMemset(B.big, 1, region_bytes));
        } else {
            const uint32_t nlines = (uint32_t)(region_bytes / 128);
            hipLaunchKernelGGL(k_chase_init, dim3(nlines / 256), dim3(256), 0, st, static_cast<int *>(B.big), nlines);
            PFP_HIP(hipStreamSynchronize(st));
        }
    }
    int launch_no = 0;
    auto launch = [&](hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
        const dim3 g(grid), b(256);
        const int i = launch_no++;
#define PFP_L(kernel, ...)                                                         \
        do {                                                                       \
            if (e0) hipExtLaunchKernelGGL(kernel, g, b, 0, s, e0, e1, 0, __VA_ARGS__); \
            else hipLaunchKernelGGL(kernel, g, b, 0, s, __VA_ARGS__);              \
        } while (0)
        switch (kind) {
            case PFP_EMPTY: PFP_L(k_empty, B.b); break;
            case PFP_ONE_LOAD: PFP_L(k_one_load, (const int *)B.a, B.b, B.n); break;
            case PFP_TWO_LOADS: PFP_L(k_two_loads, (const int *)B.a, (const int *)B.c, B.b, B.n); break;
            case PFP_CHASE: PFP_L(k_chase, (const int *)B.a, (int)(bytes ? bytes : 64), B.b); break;
            case PFP_STREAM: PFP_L(k_stream, (const void *)B.big, (uint32_t)B.big_bytes, B.b); break;
            case PFP_BARRIERS:
                hipLaunchKernelGGL(k_fill, dim3((sizeof(BarrierMem) / 4 + 255) / 256), dim3(256), 0, s,
                                   reinterpret_cast<uint32_t *>(B.bm), (int)(sizeof(BarrierMem) / 4), 0u);
                PFP_L(k_barriers, B.bm, nb, B.ticks);
                break;
            case PFP_EXCHANGE:
                hipLaunchKernelGGL(k_fill, dim3((sizeof(BarrierMem) / 4 + 255) / 256), dim3(256), 0, s,
                                   reinterpret_cast<uint32_t *>(B.bm), (int)(sizeof(BarrierMem) / 4), 0u);
                PFP_L(k_exchange, B.bm, B.xdata, xwords, nb, B.mism);
                break;
            case PFP_STREAM_COLD: {  // every launch reads another window of the region
                const size_t nwin = region_bytes / B.big_bytes;
                const char *win = static_cast<const char *>(B.big) + ((size_t)i * 37 % nwin) * B.big_bytes;
                PFP_L(k_stream, (const void *)win, (uint32_t)B.big_bytes, B.b);
                break;
            }
            case PFP_CLOCK: PFP_L(k_clock, B.ticks); break;
            case PFP_CHASE_COLD:
                PFP_L(k_chase_cold, (const int *)B.big, (int)(bytes ? bytes : 64), (i * 7919) & 0xfffff, B.b);
                break;
            default: break;
        }
#undef PFP_L
    };
    if (kind < 0 || kind > PFP_CLOCK) {
        snprintf(g_err, sizeof(g_err), "unknown probe %d", kind);
        return 1;
    }
    // eager, event-stamped
    hipEvent_t e0, e1;
    PFP_HIP(hipEventCreate(&e0));
    PFP_HIP(hipEventCreate(&e1));
    double sum = 0.0;
    for (int i = 0; i < 8 + reps; ++i) {
        launch(st, e0, e1);
        PFP_HIP(hipGetLastError());
        PFP_HIP(hipEventSynchronize(e1));
        float ms = 0.f;
        PFP_HIP(hipEventElapsedTime(&ms, e0, e1));
        if (i >= 8) sum += ms;
    }
    *eager_event_us = 1e3 * sum / reps;
    // a graph of `nodes` launches in a row, replayed
    hipGraph_t graph;
    hipGraphExec_t exec;
    PFP_HIP(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
    for (int i = 0; i < nodes; ++i) launch(st, nullptr, nullptr);
    PFP_HIP(hipStreamEndCapture(st, &graph));
    PFP_HIP(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));
    for (int i = 0; i < 3; ++i) PFP_HIP(hipGraphLaunch(exec, st));
    PFP_HIP(hipStreamSynchronize(st));
    PFP_HIP(hipEventRecord(e0, st));
    for (int i = 0; i < reps; ++i) PFP_HIP(hipGraphLaunch(exec, st));
    PFP_HIP(hipEventRecord(e1, st));
    PFP_HIP(hipEventSynchronize(e1));
    float ms = 0.f;
    PFP_HIP(hipEventElapsedTime(&ms, e0, e1));
    *graph_us_per_node = 1e3 * ms / ((double)reps * nodes);
    if (extra) {
        if (kind == PFP_BARRIERS) {
            unsigned long long t = 0;
            PFP_HIP(hipMemcpy(&t, B.ticks, 8, hipMemcpyDeviceToHost));
            *extra = nb > 0 ? (double)t / 100.0 / nb : 0.0;  // 100 MHz clock -> us per barrier
        }
        if (kind == PFP_CLOCK) {
            unsigned long long t[2] = {0, 0};
            PFP_HIP(hipMemcpy(t, B.ticks, 16, hipMemcpyDeviceToHost));
            *extra = t[1] ? (double)t[0] / ((double)t[1] / 100.0) : 0.0;  // cycles per us = MHz
        }
        if (kind == PFP_EXCHANGE) {
            uint32_t m = 0, err = 0;
            PFP_HIP(hipMemcpy(&m, B.mism, 4, hipMemcpyDeviceToHost));
            PFP_HIP(hipMemcpy(&err, &B.bm->error, 4, hipMemcpyDeviceToHost));
            *extra = (double)m + (err ? 1e9 : 0.0);
        }
        if (kind == PFP_BARRIERS) {
            uint32_t err = 0;
            PFP_HIP(hipMemcpy(&err, &B.bm->error, 4, hipMemcpyDeviceToHost));
            if (err) *extra = -1.0;  // a barrier timed out
        }
    }
    (void)hipGraphExecDestroy(exec);
    (void)hipGraphDestroy(graph);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipFree(B.a);
    (void)hipFree(B.b);
    (void)hipFree(B.c);
    (void)hipFree(B.big);
    (void)hipFree(B.bm);
    (void)hipFree(B.ticks);
    (void)hipFree(B.xdata);
    (void)hipFree(B.mism);
    (void)hipStreamDestroy(st);
    return 0;
}

}  // extern "C"
