/*
 * pf_probe.h -- C ABI of libpf_probe: latency-floor probes for the measurement harness.
 *
 * Not part of the sparse-FFN path and not cited from the paper: tiny kernels whose time as a
 * node of a replayed HIP graph, and as an eager launch stamped with HIP events, shows what a
 * kernel launch, one or two dependent memory round trips, a small plain stream and a
 * grid-wide barrier cost on the device, so that bench.py can price libpf's kernels against
 * those floors.  Allocates its own small device buffers per call and frees them.
 */
#ifndef PF_PROBE_H
#define PF_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PFP_EMPTY = 0,     /* a kernel that does nothing                                         */
    PFP_ONE_LOAD = 1,  /* b[i] = a[i] + 1: one round trip to memory, then a store            */
    PFP_TWO_LOADS = 2, /* b[i] = c[a[i]] + 1: two dependent round trips                      */
    PFP_CHASE = 3,     /* one lane follows `bytes` dependent loads (time / hops = round trip) */
    PFP_STREAM = 4,    /* reads `bytes` once with 16-byte loads, 8 in flight per thread      */
    PFP_BARRIERS = 5,  /* `bytes` grid-wide barriers (device-scope relaxed atomics, bounded
                          spins) in one launch of `grid` <= 1024 workgroups; *extra = us per
                          barrier by the device clock, -1 if a barrier timed out            */
    PFP_EXCHANGE = 6,  /* `bytes` rounds of: every workgroup stores 4 KB with device-scope
                          stores, barrier, reads another workgroup's 4 KB with device-scope
                          loads, barrier; *extra = number of mismatching words (>= 1e9: a
                          barrier timed out)                                                */
    PFP_STREAM_COLD = 7, /* PFP_STREAM, but every launch reads another window of a 1 GiB region
                            (four times the last-level cache), so the bytes come from HBM    */
    PFP_CHASE_COLD = 8,  /* PFP_CHASE through a 1 GiB region, one entry per 128-byte line     */
    PFP_CLOCK = 9        /* one lane spins 200 us; *extra = shader clock in MHz (cycle counter
                            against the constant 100 MHz wall clock)                         */
} pfp_kind;

/* Runs probe `kind` with `grid` workgroups of 256 threads on the current device.
 * graph_us_per_node: wall time of a replayed graph of `nodes` launches in a row, per launch,
 * averaged over `reps` replays (PFP_BARRIERS / PFP_EXCHANGE: a launch is preceded by a small
 * fill kernel that zeroes the counters).  eager_event_us: mean start-to-end time of one eager
 * launch from the events the launch itself stamps.  Returns 0, or 1 with pfp_last_error set. */
int pfp_measure(int kind, size_t bytes, int grid, int nodes, int reps, double *graph_us_per_node,
                double *eager_event_us, double *extra);

const char *pfp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PF_PROBE_H */
