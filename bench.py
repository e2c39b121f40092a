#!/usr/bin/env python3
"""Decode FFN-stack benchmark for the neuron-aware sparse FFN library (one MI355X).

One "step" is one decode token pushed through the whole FFN stack of the configured model
shape: per layer predictor -> compaction -> row-sparse FC1 -> column-sparse FC2 -> glue
(residual + scale-only RMS norm).  Weights and all token inputs are resident in HBM before
the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config opt-6.7b] [--batch B]

Three legs:
  value         K tokens through the recorded HIP graph of the stack (timed with host clocks
                between device synchronisations);
  roofline      a second, eager pass in which the library has every kernel launch stamp a
                pair of HIP events with its start and end on its stream; the dominant
                kernel's algorithmic bytes per launch over its mean duration against the
                8 TB/s HBM peak;
  cpu_baseline  the CPU oracle timed on the host cores on a bounded sample of the same
                workload (a few layers x a few tokens, scaled by the layer count).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="decode tokens timed (default: config)")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", default="opt-6.7b")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--layers", type=int, default=None, help="override the layer count")
    ap.add_argument("--mode", choices=["graph", "eager", "copycal", "m0", "floors", "crossover"],
                    default="graph",
                    help="copycal: only run plain device copies of a known size, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters by; m0: operator "
                         "micro-benchmark, one 4096 x 4096 layer, active fraction swept; "
                         "floors: latency-floor probes (empty kernel, dependent loads, plain "
                         "streams from cache and from HBM, grid barrier) as graph nodes; "
                         "crossover: one layer of --config at --batch, sparse path against the "
                         "dense path over the listed fraction (Sec. 8.2 dense fallback)")
    ap.add_argument("--sort-neurons", type=int, default=0, metavar="N",
                    help="profile activation counts over N tokens first and lay every layer's "
                         "neurons out hot-first (frequency-sorted layout)")
    ap.add_argument("--lookahead", type=int, default=0, choices=[0, 1],
                    help="1: look-ahead prediction at distance 1 (predictors overlap the sparse "
                         "kernels of the layer before; lists differ from the default path)")
    ap.add_argument("--rank", type=int, default=None,
                    help="override the predictor rank r of every layer (a multiple of 8)")
    ap.add_argument("--rate", type=float, default=None,
                    help="override the configuration's mean activation rate (scaling runs)")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "pmc_traffic.json"),
                    help="HBM bytes per launch per kernel from the rocprofv3 --pmc runs (optional)")
    ap.add_argument("--profile-steps", type=int, default=16)
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--cpu-layers", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-pred-bias", action="store_true",
                    help="bias-free random predictor (about half of the neurons marked)")
    ap.add_argument("--opt", action="append", default=[], metavar="NAME=VALUE",
                    help="set a library option (pf_ctx_set_option) by its name without the PF_OPT_ "
                         "prefix, e.g. --opt fused=0 --opt down_split=2 --opt lookahead_form=3")
    ap.add_argument("--seed", type=int, default=2312)
    return ap.parse_args()


def operator_microbench(args, torch, np, pf, wl):
    """The paper's operator test (Sec. 8.3.3 'Neuron-aware Operator Performance', Fig.
    "operator"): one FFN layer with
    4096 x 4096 matrices, batch 1, a uniformly random set of active rows of swept size; time
    of FC1 and FC2 against the active fraction (slope = 1 / bandwidth, intercept = latency)."""
    cfg = wl.scaled(wl.CONFIGS["opt-6.7b"], name="m0-4096x4096", layers=1, ffn=4096, r=128)
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=1)
    lay = wl.make_layer(cfg, 0, args.seed, device="cuda")
    L = pf.Layer.from_workload(ctx, cfg, lay)
    x = wl.make_inputs(cfg, 0, args.seed, batch=1, device="cuda")
    y = torch.empty_like(x)
    rng = np.random.Generator(np.random.PCG64(args.seed))
    rows = []
    for frac in (0.01, 0.02, 0.05, 0.1, 0.2, 0.5, 1.0):
        k = max(1, int(round(frac * cfg.ffn)))
        sel = np.sort(rng.choice(cfg.ffn, size=k, replace=False)).astype(np.int32)
        idx = torch.zeros(cfg.ffn, dtype=torch.int32, device="cuda")
        idx[:k] = torch.from_numpy(sel).cuda()
        cnt = torch.tensor([k], dtype=torch.int32, device="cuda")
        for _ in range(8):
            ctx.sparse_ffn(L, x, idx, cnt, y)
        torch.cuda.synchronize()
        ctx.profile_begin()
        for _ in range(64):
            ctx.sparse_ffn(L, x, idx, cnt, y)
        st = ctx.profile_end()
        up_us = 1e3 * st["k_up"][1] / st["k_up"][0]
        dn_us = 1e3 * st["k_down"][1] / st["k_down"][0]
        by = k * cfg.row_bytes
        rows.append({"fraction": frac, "k": k, "bytes_per_matrix": by, "fc1_us": round(up_us, 3),
                     "fc2_us": round(dn_us, 3), "fc1_GBps": round(by / up_us / 1e3, 1),
                     "fc2_GBps": round(by / dn_us / 1e3, 1)})
    return {"mode": "m0", "workload": "one layer, d=4096, ffn=4096, fp16, batch 1, uniformly "
            "random active rows, 64 launches per point", "points": rows}


def crossover_table(args, torch, np, pf, wl):
    """Where the dense fallback of Sec. 8.2 starts to pay: one layer of the configuration, the
    predictor's time, the sparse kernels' time over uniformly random lists of swept size, the
    dense step (every neuron listed, predictor skipped) and the dense step of the adaptive
    entry point (predictor kernels launched but returning at once).  The crossover is the
    listed fraction at which predictor + sparse kernels cost what the dense step costs."""
    cfg = wl.scaled(wl.CONFIGS[args.config], layers=1)
    B = args.batch
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=B)
    lay = wl.make_layer(cfg, 0, args.seed, device="cuda")
    L = pf.Layer.from_workload(ctx, cfg, lay)
    x = wl.make_inputs(cfg, 0, args.seed, batch=B, device="cuda")
    y = torch.empty_like(x)
    words = torch.zeros(cfg.ffn // 64, dtype=torch.int64, device="cuda")
    rng = np.random.Generator(np.random.PCG64(args.seed))
    reps = 48

    def timed(fn):
        for _ in range(6):
            fn()
        torch.cuda.synchronize()
        ctx.profile_begin()
        for _ in range(reps):
            fn()
        st = ctx.profile_end()
        return {k: round(1e3 * ms / n, 3) for k, (n, ms) in st.items() if n}, \
            round(sum(1e3 * ms / reps for _, (n, ms) in st.items() if n), 3)

    pred_k, pred_us = timed(lambda: ctx.predict(L, x, None, words))
    dense_k, dense_us = timed(lambda: ctx.dense_ffn(L, x, y))
    # adaptive entry point held in its dense mode (crossover so low that every step qualifies)
    ctx.layer_step_adaptive(L, x, y, 1e-6)
    ad_k, ad_us = timed(lambda: ctx.layer_step_adaptive(L, x, y, 1e-6))
    L.adaptive_state(reset=True)
    rows = []
    for frac in (0.02, 0.05, 0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1.0):
        k = max(1, int(round(frac * cfg.ffn)))
        sel = np.sort(rng.choice(cfg.ffn, size=k, replace=False)).astype(np.int32)
        idx = torch.zeros(cfg.ffn, dtype=torch.int32, device="cuda")
        idx[:k] = torch.from_numpy(sel).cuda()
        cnt = torch.tensor([k], dtype=torch.int32, device="cuda")
        sk, sus = timed(lambda: ctx.sparse_ffn(L, x, idx, cnt, y))
        rows.append({"fraction": frac, "k": k, "sparse_us": sus, "predictor_plus_sparse_us": round(pred_us + sus, 3)})
    cross = None
    for a, b in zip(rows, rows[1:]):
        fa, fb = a["predictor_plus_sparse_us"] - dense_us, b["predictor_plus_sparse_us"] - dense_us
        if fa < 0 <= fb:
            cross = round(a["fraction"] + (b["fraction"] - a["fraction"]) * (-fa) / (fb - fa), 3)
            break
    out = {"mode": "crossover", "workload": "one %s layer (d=%d, ffn=%d, r=%d), batch %d, uniformly "
           "random lists, %d launches per point, per-kernel HIP events" % (cfg.name, cfg.d, cfg.ffn, cfg.r, B, reps),
           "predictor_us": pred_us, "predictor_kernels": pred_k, "dense_us": dense_us,
           "dense_kernels": dense_k, "adaptive_dense_step_us": ad_us, "adaptive_dense_kernels": ad_k,
           "points": rows, "crossover_fraction": cross}
    if B == 1 and cfg.wtype == wl.W_FP16 and cfg.ffn >= 8192:
        # a plain streaming GEMV over the first 8192 rows of FC1 (the predictor's hidden-layer
        # kernel: rows in order, no list) against the gather kernel over the list 0 .. 8191
        ctx2 = pf.Context(cfg.d, 8192, 8192, max_batch=1)
        w8 = lay["w_up"][:8192].contiguous()
        Ls = pf.Layer(ctx2, cfg.d, 8192, 8192, w_up=w8, w_down=w8, p1=w8,
                      p2=torch.zeros((8192, 8192), dtype=torch.float16, device="cuda"))
        w2 = torch.zeros(128, dtype=torch.int64, device="cuda")
        sk, _ = timed_on(ctx2, lambda: ctx2.predict(Ls, x, None, w2), torch, reps)
        idx = torch.arange(8192, dtype=torch.int32, device="cuda")
        cnt = torch.tensor([8192], dtype=torch.int32, device="cuda")
        y2 = torch.empty_like(x)
        gk, _ = timed_on(ctx2, lambda: ctx2.sparse_ffn(Ls, x, idx, cnt, y2), torch, reps)
        by = 8192 * cfg.row_bytes
        out["stream_vs_gather_8192_rows"] = {
            "bytes": by, "stream_gemv_us": sk["k_pred_hidden"], "gather_over_iota_us": gk["k_up"],
            "stream_GBps": round(by / sk["k_pred_hidden"] / 1e3, 1),
            "gather_GBps": round(by / gk["k_up"] / 1e3, 1)}
    return out


def timed_on(ctx, fn, torch, reps):
    for _ in range(6):
        fn()
    torch.cuda.synchronize()
    ctx.profile_begin()
    for _ in range(reps):
        fn()
    st = ctx.profile_end()
    return {k: round(1e3 * ms / n, 3) for k, (n, ms) in st.items() if n}, None


def _probe_lib():
    import ctypes
    path = os.path.join(ROOT, "paper_2312_12456_amd", "libpf_probe.so")
    if not os.path.exists(path):
        return None
    L = ctypes.CDLL(path)
    D = ctypes.POINTER(ctypes.c_double)
    L.pfp_measure.argtypes = [ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int, D, D, D]
    L.pfp_last_error.restype = ctypes.c_char_p
    return L


def device_clocks(torch):
    """Clock state recorded with the run: the shader clock measured by a probe kernel while the
    device is still warm from the timed region (cycle counter against the 100 MHz wall clock),
    and the maxima the runtime reports."""
    import ctypes
    out = {}
    try:
        prop = torch.cuda.get_device_properties(0)
        out["max_sclk_mhz"] = round(getattr(prop, "clock_rate", 0) / 1e3, 1)
        out["max_mclk_mhz"] = round(getattr(prop, "memory_clock_rate", 0) / 1e3, 1)
        out["compute_units"] = prop.multi_processor_count
    except Exception:
        pass
    L = _probe_lib()
    if L is not None:
        g, e, x = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        if L.pfp_measure(9, 0, 256, 1, 3, ctypes.byref(g), ctypes.byref(e), ctypes.byref(x)) == 0:
            out["sclk_mhz_under_load"] = round(x.value, 1)
    return out


def latency_floors():
    """Times of the probe kernels of libpf_probe.so as nodes of a replayed HIP graph (what a
    kernel of the stack is: one node among ~100) and as eager launches stamped with events."""
    import ctypes
    L = _probe_lib()
    if L is None:
        raise SystemExit("libpf_probe.so is missing: run __graft_entry__.build()")

    def m(kind, size, grid, nodes=64, reps=20):
        g, e, x = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        if L.pfp_measure(kind, size, grid, nodes, reps, ctypes.byref(g), ctypes.byref(e), ctypes.byref(x)):
            raise SystemExit("probe failed: %s" % L.pfp_last_error().decode())
        return {"graph_node_us": round(g.value, 3), "eager_event_us": round(e.value, 3), "extra": round(x.value, 3)}

    EMPTY, ONE, TWO, CHASE, STREAM, BARRIERS, EXCHANGE, STREAM_COLD, CHASE_COLD = range(9)
    out = {"mode": "floors", "unit": "us", "rows": []}

    def row(name, **kw):
        kw["probe"] = name
        out["rows"].append(kw)

    row("empty kernel, 256 workgroups", **m(EMPTY, 0, 256))
    row("one dependent load, 1024 workgroups", **m(ONE, 0, 1024))
    row("two dependent loads, 1024 workgroups", **m(TWO, 0, 1024))
    for mb in (8, 11, 32, 44, 64, 128):
        row("stream %d MiB from HBM, 256 workgroups" % mb, **m(STREAM_COLD, mb << 20, 256, reps=10))
    for mb in (8, 32):
        row("stream %d MiB cache-resident, 256 workgroups" % mb, **m(STREAM, mb << 20, 256, nodes=32))
    b0 = m(BARRIERS, 0, 256, nodes=8)
    b32 = m(BARRIERS, 32, 256, nodes=8)
    row("32 grid barriers in one launch of 256 workgroups (extra: us per barrier, device clock)", **b32)
    row("the same launch without barriers", **b0)
    row("8 rounds of 4 KB exchange per workgroup through 2 barriers (extra: mismatching words)",
        **m(EXCHANGE, 8, 256, nodes=4, reps=5))
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2312_12456_amd import pf
    from paper_2312_12456_amd import workload as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.mode == "copycal":
        # 16 copies of 256 MiB: each dispatch reads 2^28 and writes 2^28 bytes
        src = torch.empty(1 << 26, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(16):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"mode": "copycal", "copies": 16, "bytes_read_per_copy": src.numel() * 4,
                          "bytes_written_per_copy": src.numel() * 4}))
        return
    if args.mode == "floors":
        print(json.dumps(latency_floors()))
        return
    if args.mode == "m0":
        print(json.dumps(operator_microbench(args, torch, np, pf, wl)))
        return
    if args.mode == "crossover":
        print(json.dumps(crossover_table(args, torch, np, pf, wl)))
        return
    cfg = wl.CONFIGS[args.config]
    if args.layers:
        cfg = wl.scaled(cfg, layers=args.layers)
    if args.rate is not None:
        cfg = wl.scaled(cfg, rate=args.rate)
    if args.rank is not None:
        cfg = wl.scaled(cfg, r=args.rank)
    B = args.batch
    K = args.steps if args.steps is not None else cfg.tokens
    W = args.warmup
    dev = "cuda"

    # ---- workload resident in HBM ---------------------------------------------------
    t_gen = time.time()
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=B)
    if args.sort_neurons > 0:
        # hot neurons end up next to each other: have the library form its segments of 64
        # neurons with a stride over the neuron axis
        ctx.set_option(pf.OPT_SEG_STRIDED, 1)
    tensors, layers = [], []
    for l in range(cfg.layers):
        t = wl.make_layer(cfg, l, args.seed, device=dev, pred_bias=not args.no_pred_bias)
        tensors.append(t)
        layers.append(pf.Layer.from_workload(ctx, cfg, t))
    n_tok = max(K, W, args.profile_steps)
    x_all = torch.stack([wl.make_inputs(cfg, t, args.seed, batch=B) for t in range(n_tok)]).to(dev)
    x_buf = torch.empty((B, cfg.d), device=dev)
    out = torch.empty((B, cfg.d), device=dev)
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen

    if args.sort_neurons > 0:
        # activation profiler -> neuron table -> hot-first layout (the caller owns the weights,
        # so the re-layout is the caller's: here, the harness's)
        tabs = [torch.zeros(cfg.ffn, dtype=torch.int32, device=dev) for _ in range(cfg.layers)]
        xa0, y0 = torch.empty((B, cfg.d), device=dev), torch.empty((B, cfg.d), device=dev)
        for t in range(min(args.sort_neurons, n_tok)):
            xa0.copy_(x_all[t])
            for l, L in enumerate(layers):
                ctx.layer_step(L, xa0, y0)
                ctx.count_activations(L, tabs[l])
                ctx.stack_glue(xa0, y0, xa0)
        torch.cuda.synchronize()
        n_prof = min(args.sort_neurons, n_tok)
        tables, prefix = [], []
        for l in range(cfg.layers):
            order_t = torch.argsort(tabs[l], descending=True, stable=True)
            # neurons listed in at least 90 % of the profiled tokens form the always-on prefix:
            # the library lists them without evaluating their predictor rows
            hot = int((tabs[l] >= 0.9 * n_prof).sum().item())
            a_on = min(64 * (hot // 64), cfg.ffn - 64)
            tensors[l] = wl.permute_neurons(tensors[l], order_t.cpu().numpy())
            layers[l] = pf.Layer.from_workload(ctx, cfg, tensors[l])
            tables.append(order_t.to(torch.int32).contiguous())
            layers[l].set_neuron_table(tables[l], a_on)
            prefix.append(a_on)
        torch.cuda.synchronize()
        sort_info = {"profiled_tokens": n_prof, "always_on_mean": float(np.mean(prefix))}

    for kv in args.opt:
        key, _, val = kv.partition("=")
        ctx.set_option(getattr(pf, "OPT_" + key.upper()), int(val))
    ctx.set_lookahead(args.lookahead)
    plan = pf.Plan(ctx, layers, x_buf, out) if args.mode == "graph" else None

    def step(t):
        x_buf.copy_(x_all[t % n_tok])
        if plan is not None:
            plan.run()
        else:
            ctx.stack_step(layers, x_buf, out)

    for t in range(W):
        step(t)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(K):
        step(t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert bool(torch.isfinite(out).all()), "non-finite stack output"
    ms_per_step = 1e3 * elapsed / K
    tokens_per_s = B * K / elapsed

    # the same stack with look-ahead prediction (another schedule AND other lists: reported
    # beside the headline value, never in its place)
    with_la = None
    if not args.lookahead and plan is not None and cfg.layers > 1:
        ctx.set_lookahead(1)
        plan_la = pf.Plan(ctx, layers, x_buf, out)
        ctx.set_lookahead(0)
        for t in range(W):
            x_buf.copy_(x_all[t % n_tok])
            plan_la.run()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for t in range(K):
            x_buf.copy_(x_all[t % n_tok])
            plan_la.run()
        torch.cuda.synchronize()
        e_la = time.perf_counter() - t1
        plan_la.close()
        with_la = {"value": round(B * K / e_la, 2), "unit": "tokens/s", "ms_per_step": round(1e3 * e_la / K, 4),
                   "note": "look-ahead prediction at distance 1: the list of layer l comes from its "
                           "predictor applied to the input of layer l-1 (an approximation; other lists "
                           "than the headline run)"}

    # per-token latency spread: a second, short run with an event between the steps
    nl = min(K, 128)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(nl + 1)]
    evs[0].record()
    for t in range(nl):
        step(t)
        evs[t + 1].record()
    torch.cuda.synchronize()
    lat = np.array([evs[t].elapsed_time(evs[t + 1]) for t in range(nl)])
    latency = {"steps": nl, "p50_ms": round(float(np.percentile(lat, 50)), 4),
               "p95_ms": round(float(np.percentile(lat, 95)), 4), "max_ms": round(float(lat.max()), 4)}

    # ---- clocks: what the shader clock really was, measured by a kernel right after the run ----
    clocks = device_clocks(torch)

    # ---- per-kernel passes: HIP events around every launch, active counts read back ----
    P = max(1, min(args.profile_steps, n_tok))
    counts = np.zeros((P, cfg.layers), dtype=np.int64)
    y = torch.empty((B, cfg.d), device=dev)
    xa = torch.empty((B, cfg.d), device=dev)
    cnt = torch.empty(1, dtype=torch.int32, device=dev)
    ctx.set_lookahead(0)
    _, _, count_ptr = ctx.last_active()
    # active counts: the same chain of layers, one layer step at a time (not timed)
    for t in range(P):
        xa.copy_(x_all[t])
        for l, L in enumerate(layers):
            ctx.layer_step(L, xa, y)
            ctx.stack_glue(xa, y, xa)
            pf.copy_from_device_address(cnt, count_ptr)
            counts[t, l] = int(cnt.item())

    def event_pass():
        ctx.profile_begin()
        for t in range(P):
            xa.copy_(x_all[t])
            ctx.stack_step(layers, xa, y)
        return ctx.profile_end()

    # (a) the stack step as shipped, launched eagerly (the launches the graph replays)
    ctx.set_lookahead(args.lookahead)
    stats = event_pass()
    if args.lookahead and stats["k_la_up_hidden"][0] == 0:
        # look-ahead on two streams: the event pairs do not cover the second stream, so the
        # per-kernel figures are those of the same kernels in the default schedule
        ctx.set_lookahead(0)
        stats = event_pass()
    # (b) the list form of the same layers (FC1 and FC2 as kernels of their own): the direct
    # measurement behind the touched-bytes figure
    ctx.set_lookahead(0)
    fused_before = ctx.get_option(pf.OPT_FUSED)
    ctx.set_option(pf.OPT_FUSED, 0)
    stats_list = event_pass()
    ctx.set_option(pf.OPT_FUSED, fused_before)
    ctx.set_lookahead(args.lookahead)
    k_mean = float(counts.mean())
    nm = cfg.n_matrices
    alg_bytes = {
        "k_pred_hidden": 2.0 * cfg.r * cfg.d,
        "k_pred_out": 2.0 * cfg.ffn * cfg.r + (0 if args.no_pred_bias else 4.0 * cfg.ffn),
        "k_up": k_mean * (nm - 1) * cfg.row_bytes,
        "k_down": k_mean * cfg.row_bytes,
    }
    alg_bytes["k_up_mfma"] = alg_bytes["k_up"]
    # the three-launch form: predictor output layer + FC1 in one kernel, FC2 over its segments
    alg_bytes["k_out_up"] = alg_bytes["k_pred_out"] + alg_bytes["k_up"]
    alg_bytes["k_down_mask"] = alg_bytes["k_down"]
    # look-ahead in two launches: [next hidden layer | FC1], [FC2 | next output layer]
    alg_bytes["k_la_up_hidden"] = alg_bytes["k_pred_hidden"] + alg_bytes["k_up"]
    alg_bytes["k_la_down_out"] = alg_bytes["k_pred_out"] + alg_bytes["k_down"]

    def per_kernel(st):
        out_k = {}
        for name, (launches, total_ms) in st.items():
            if launches == 0:
                continue
            avg_us = 1e3 * total_ms / launches
            ent = {"launches": launches, "avg_us": round(avg_us, 3)}
            if name in alg_bytes:
                ent["alg_bytes"] = alg_bytes[name]
                ent["GBps"] = round(alg_bytes[name] / (avg_us * 1e-6) / 1e9, 1)
            out_k[name] = ent
        return out_k

    kernels = per_kernel(stats)
    kernels_list = per_kernel(stats_list)
    dominant = max((n for n in kernels if n in alg_bytes), key=lambda n: stats[n][1])
    dk = kernels[dominant]
    # measured HBM traffic of that kernel per launch, if the counter runs were summarised for
    # exactly this workload (profiles/: FETCH_SIZE + WRITE_SIZE, scaled by a plain copy of known
    # size); an overridden workload has no such summary
    traffic = None
    overridden = (args.rate is not None or args.rank is not None or args.sort_neurons > 0
                  or args.no_pred_bias or args.lookahead or args.opt)
    if not overridden:
        try:
            with open(args.traffic_file) as f:
                tf = json.load(f)
            key = "%s/b%d" % (cfg.name, B)
            if key in tf and dominant in tf[key]:
                traffic = tf[key][dominant]["hbm_bytes_per_launch"]
        except (OSError, ValueError, KeyError):
            traffic = None
    roofline = {
        "bound": "hbm", "kernel": dominant, "achieved": dk["GBps"], "peak": HBM_PEAK_GBPS,
        "unit": "GB/s", "frac": round(dk["GBps"] / HBM_PEAK_GBPS, 4), "traffic": traffic,
        "alg_bytes_per_launch": dk["alg_bytes"], "avg_us": dk["avg_us"],
    }
    touched = k_mean * nm * cfg.row_bytes
    # Touched bytes over FC1 + FC2, measured directly on the list form's own kernels.
    # (k_combine, which adds FC2's partial sums for a stand-alone layer step, is not part of
    # the stack: there the next layer's first kernel adds them while it forms x.)
    up_name = "k_up_mfma" if "k_up_mfma" in kernels_list else "k_up"
    t_sparse_us = kernels_list[up_name]["avg_us"] + kernels_list["k_down"]["avg_us"]
    touched_gbps = touched / (t_sparse_us * 1e-6) / 1e9
    touched_out = {
        "k_mean": round(k_mean, 1), "active_frac": round(k_mean / cfg.ffn, 4),
        "bytes_per_layer": touched, "sparse_us_per_layer": round(t_sparse_us, 3),
        "sparse_us_from": "%s + k_down of a list-form pass in this run" % up_name,
        "GBps": round(touched_gbps, 1), "frac_of_peak": round(touched_gbps / HBM_PEAK_GBPS, 4),
        "target_frac": 0.60, "target_met": bool(touched_gbps / HBM_PEAK_GBPS >= 0.60),
    }
    if "k_out_up" in kernels and "k_pred_out" in kernels_list:
        # the shipped three-launch form has no FC1 kernel of its own: an estimate of its share
        est = (kernels["k_out_up"]["avg_us"] - kernels_list["k_pred_out"]["avg_us"]
               + kernels["k_down_mask"]["avg_us"])
        touched_out["three_launch_estimate"] = {
            "sparse_us_per_layer": round(est, 3), "from": "k_out_up - k_pred_out + k_down_mask",
            "frac_of_peak": round(touched / (est * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}
    # layer level: every algorithmic byte of a layer over the layer's share of the step time
    pred_bytes = alg_bytes["k_pred_hidden"] + alg_bytes["k_pred_out"]
    layer_us = 1e3 * ms_per_step / cfg.layers
    layer = {"bytes_per_layer": pred_bytes + touched, "us_per_layer": round(layer_us, 3),
             "GBps": round((pred_bytes + touched) / (layer_us * 1e-6) / 1e9, 1),
             "frac_of_peak": round((pred_bytes + touched) / (layer_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
             "touched_only_GBps": round(touched / (layer_us * 1e-6) / 1e9, 1),
             "touched_only_ceiling": round(touched / (pred_bytes + touched), 4)}

    # ---- CPU oracle on the host cores, bounded sample --------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import pf_oracle
        ns = min(args.cpu_layers, cfg.layers)
        ol = []
        for l in range(ns):
            h = wl.to_host(tensors[l])
            ol.append(pf_oracle.Layer(
                cfg.d, cfg.ffn, cfg.r, act=cfg.act, wtype=cfg.wtype, threshold=cfg.threshold,
                w_up=h.get("w_up"), w_gate=h.get("w_gate"), w_down=h.get("w_down"),
                s_up=h.get("s_up"), s_gate=h.get("s_gate"), s_down=h.get("s_down"),
                b_up=h.get("b_up"), b_down=h.get("b_down"), p1=h.get("p1"), p2=h.get("p2"),
                p_bias=h.get("p_bias")))
        xs_host = x_all[:min(n_tok, 64)].cpu().numpy()

        def timed(fn, budget):
            """Whole passes over the sample layers until the budget is spent, at least 3."""
            calls, t_cpu, tok = 0, 0.0, 0
            while t_cpu < budget or tok < 3:
                xh = xs_host[tok % xs_host.shape[0]]
                c0 = time.perf_counter()
                for O in ol:
                    yh = fn(O, xh)
                    xh = pf_oracle.stack_glue(xh, yh)
                t_cpu += time.perf_counter() - c0
                calls += ns
                tok += 1
            return t_cpu / calls, tok, t_cpu

        per_layer, tok, t_cpu = timed(lambda O, xh: O.layer_step(xh), 0.7 * args.cpu_seconds)
        per_layer_dense, tok_d, t_cpu_d = timed(lambda O, xh: O.dense_ffn(xh), 0.3 * args.cpu_seconds)
        cpu = {
            "value": round(B / (per_layer * cfg.layers), 4), "unit": "tokens/s",
            "cores": pf_oracle.num_threads(), "kind": "oracle",
            "sample": "%d tokens x first %d of %d layers at full shape, fp64 oracle layer_step + "
                      "glue, %.1f s; per-layer time scaled by the layer count"
                      % (tok, ns, cfg.layers, t_cpu),
            "dense_ffn": {"value": round(B / (per_layer_dense * cfg.layers), 4), "unit": "tokens/s",
                          "sample": "%d tokens x %d layers, fp64 oracle dense_ffn + glue (no "
                                    "predictor), %.1f s" % (tok_d, ns, t_cpu_d)},
        }

    result = {
        "metric": "decode FFN-stack tokens/s at batch %d" % B,
        "value": round(tokens_per_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "weights": "int4-g128" if cfg.wtype == wl.W_INT4_G128 else "fp16",
        "config": {"workload": "%s FFN stack: %d layers, d=%d, ffn=%d, r=%d, %s, %s weights, "
                               "batch %d, Zipf(%.1f) mean rate %.0f%%, %d decode tokens"
                               % (cfg.name, cfg.layers, cfg.d, cfg.ffn, cfg.r,
                                  "ReGLU" if cfg.act == wl.ACT_REGLU else "ReLU",
                                  "int4-g128" if cfg.wtype == wl.W_INT4_G128 else "fp16",
                                  B, cfg.alpha, 100 * cfg.rate, K),
                   "launch": args.mode, "predictor_bias": not args.no_pred_bias,
                   "lookahead": args.lookahead,
                   "neuron_layout": ("hot-first from %d profiled tokens through the library's neuron "
                                     "table, always-on prefix of %.0f neurons per layer on average"
                                     % (sort_info["profiled_tokens"], sort_info["always_on_mean"]))
                   if args.sort_neurons > 0 else "as generated"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "touched": touched_out,
        "with_lookahead": with_la,
        "layer": layer,
        "latency": latency,
        "clocks": clocks,
        "kernels": kernels,
        "kernels_list_form": {k: v for k, v in kernels_list.items()
                              if k in ("k_pred_hidden", "k_pred_out", "k_up", "k_up_mfma", "k_down")},
        "setup_s": round(t_gen, 1),
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
