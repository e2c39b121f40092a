"""GPU parity at the full layer shapes of the benchmark configurations, through the same entry
points and launch configuration bench.py times (layer_step, stack_step and the recorded plan).
The oracle finishes one full-size layer in about a second, so whole outputs are compared."""
import numpy as np
import pytest
import torch

from paper_2312_12456_amd import workload as wl
from tests.util import (MaskTrace, check_active_set, check_output, oracle_chain_on_device_sets,
                        oracle_layer, oracle_lookahead_chain_on_device_sets)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pf():
    from paper_2312_12456_amd import pf as pfmod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pfmod.lib()
    return pfmod


def _mask_of(pf, ctx, ffn):
    wptr, iptr, cptr = ctx.last_active()
    words = torch.empty(ffn // 64, dtype=torch.int64, device="cuda")
    idx = torch.empty(ffn, dtype=torch.int32, device="cuda")
    cnt = torch.empty(1, dtype=torch.int32, device="cuda")
    pf.copy_from_device_address(words, wptr)
    pf.copy_from_device_address(idx, iptr)
    pf.copy_from_device_address(cnt, cptr)
    bits = np.unpackbits(words.cpu().numpy().view(np.uint8), bitorder="little")[:ffn].astype(bool)
    n = int(cnt.item())
    return bits, idx.cpu().numpy()[:n]


@pytest.mark.parametrize("name,B,layer", [
    ("opt-6.7b", 1, 0), ("opt-6.7b", 1, 31),
    ("llama2-13b-reglu", 1, 0), ("llama2-13b-reglu", 4, 20),
    ("opt-30b", 1, 0), ("opt-30b", 8, 47), ("opt-30b", 4, 24), ("opt-30b", 3, 1),
    ("falcon-40b-relu", 1, 0), ("falcon-40b-relu", 1, 59),
    ("bamboo-7b-drelu", 1, 0), ("bamboo-7b-drelu", 1, 31), ("bamboo-7b-drelu", 4, 16),
    ("opt-175b-int4", 1, 0), ("opt-175b-int4", 1, 95),
])
def test_full_shape_layer_step(pf, oracle, name, B, layer):
    cfg = wl.CONFIGS[name]
    lay = wl.make_layer(cfg, layer, seed=2312, device="cuda")
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=B)
    L = pf.Layer.from_workload(ctx, cfg, lay)
    O = oracle_layer(cfg, wl.to_host(lay))
    x = wl.make_inputs(cfg, 3, seed=2312, batch=B, device="cuda")
    xh = x.cpu().numpy()
    y = torch.full((B, cfg.d), float("nan"), device="cuda")
    ctx.layer_step(L, x, y)
    torch.cuda.synchronize()
    mask, idx = _mask_of(pf, ctx, cfg.ffn)
    ref = O.predict(xh)
    in_band = check_active_set(mask, ref["scores"], cfg.threshold, name)
    assert in_band < 0.005 * cfg.ffn * B + 16  # the excluded band stays a sliver of the set
    assert np.array_equal(idx, oracle.compact(mask))
    # the configured activation structure is what the kernels were sized for
    union = wl.expected_union_rate(lay["p"], B)
    assert abs(mask.mean() - union) < 0.25 * union + 0.01
    check_output(y.cpu().numpy(), O.masked_ffn(xh, mask), name)
    # exact-mask mode at full size: the oracle's ReLU-positive list reproduces the dense block
    exact = O.exact_mask(xh)
    eidx = oracle.compact(exact)
    didx = torch.zeros(cfg.ffn, dtype=torch.int32, device="cuda")
    didx[:eidx.size] = torch.from_numpy(eidx).cuda()
    dcnt = torch.tensor([eidx.size], dtype=torch.int32, device="cuda")
    ctx.sparse_ffn(L, x, didx, dcnt, y)
    torch.cuda.synchronize()
    check_output(y.cpu().numpy(), O.masked_ffn(xh, exact), name + " exact mask")


def test_full_shape_stack_plan_matches_layer_chain(pf):
    """Two OPT-6.7B layers through the recorded plan (what bench.py times) == the chain of
    stand-alone layer_step + stack_glue calls, replay after replay."""
    cfg = wl.scaled(wl.CONFIGS["opt-6.7b"], layers=2)
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=1)
    lays = [wl.make_layer(cfg, l, seed=2312, device="cuda") for l in range(2)]
    Ls = [pf.Layer.from_workload(ctx, cfg, t) for t in lays]
    x0 = wl.make_inputs(cfg, 0, seed=2312, batch=1, device="cuda")
    xc, yc = x0.clone(), torch.empty_like(x0)
    for L in Ls:
        ctx.layer_step(L, xc, yc)
        ctx.stack_glue(xc, yc, xc)
    out = torch.zeros_like(x0)
    plan = pf.Plan(ctx, Ls, x0, out)
    for _ in range(3):
        out.zero_()
        plan.run()
        torch.cuda.synchronize()
        np.testing.assert_allclose(out.cpu().numpy(), xc.cpu().numpy(), atol=1e-4, rtol=0)
        _ = (x0 + 1).sum().item()
    plan.close()


@pytest.mark.parametrize("name,B", [("opt-6.7b", 1), ("opt-6.7b", 3), ("opt-30b", 2),
                                    ("bamboo-7b-drelu", 1)])
def test_full_shape_stack_three_launch_form_matches_oracle(pf, oracle, name, B):
    """Three full-size layers through the recorded plan, at the shapes and batches where the
    stack's inner layers take the three-launch form (output layer + FC1 fused, FC2 over
    segments): the oracle's stack, the list-form chain, and the launch counts."""
    cfg = wl.scaled(wl.CONFIGS[name], layers=3)
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=B)
    lays = [wl.make_layer(cfg, l, seed=2312, device="cuda") for l in range(cfg.layers)]
    Ls = [pf.Layer.from_workload(ctx, cfg, t) for t in lays]
    x0 = wl.make_inputs(cfg, 1, seed=2312, batch=B, device="cuda")
    out = torch.full_like(x0, float("nan"))
    plan = pf.Plan(ctx, Ls, x0, out)
    plan.run()
    torch.cuda.synchronize()
    plan.close()
    eager = torch.empty_like(x0)
    ctx.profile_begin()
    ctx.stack_step(Ls, x0, eager)
    stats = ctx.profile_end()
    assert stats["k_out_up"][0] == 2 and stats["k_down_mask"][0] == 2, stats
    assert torch.equal(eager, out)
    xc, yc = x0.clone(), torch.empty_like(x0)
    for L in Ls:
        ctx.layer_step(L, xc, yc)
        ctx.stack_glue(xc, yc, xc)
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy(), xc.cpu().numpy(), atol=2e-4, rtol=0)
    # the oracle's stack, driven by the sets the plan used (read through the mask trace of a
    # second replay): every set bit-exact outside the score band, output within the bar
    trace = MaskTrace(ctx, cfg.layers, cfg.ffn)
    out2 = torch.full_like(x0, float("nan"))
    plan = pf.Plan(ctx, Ls, x0, out2)
    plan.run()
    torch.cuda.synchronize()
    plan.close()
    ctx.set_mask_trace(None)
    assert torch.equal(out2, out)
    Os = [oracle_layer(cfg, wl.to_host(t)) for t in lays]
    ref, n_cmp, in_band = oracle_chain_on_device_sets(oracle, Os, x0.cpu().numpy(), trace.masks(),
                                                      cfg.threshold, name)
    assert n_cmp == cfg.layers
    assert in_band < 0.005 * cfg.ffn * B * cfg.layers + 16
    check_output(out.cpu().numpy(), ref, name + " three-launch stack")


@pytest.mark.parametrize("name,B", [("opt-6.7b", 1), ("opt-6.7b", 3), ("llama2-13b-reglu", 2), ("opt-30b", 2),
                                    # the same form from the matrix-core kernels ...
                                    ("opt-30b", 3), ("opt-30b", 4), ("opt-30b", 8), ("llama2-13b-reglu", 4),
                                    ("bamboo-7b-drelu", 4),
                                    # ... and from the int4 kernels
                                    ("opt-175b-int4", 1)])
def test_full_shape_lookahead_two_launch_form_matches_oracle(pf, oracle, name, B):
    """Three full-size layers with look-ahead prediction through the recorded plan, in the form
    with two launches per layer (next layer's predictor beside this layer's sparse kernels;
    vector, matrix-core and int4 kernels):
    every layer's set against the oracle's look-ahead rule outside the score band, the output
    against the oracle's stack run on those sets."""
    cfg = wl.scaled(wl.CONFIGS[name], layers=3)
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=B)
    ctx.set_lookahead(1)
    lays = [wl.make_layer(cfg, l, seed=2312, device="cuda") for l in range(cfg.layers)]
    Ls = [pf.Layer.from_workload(ctx, cfg, t) for t in lays]
    x0 = wl.make_inputs(cfg, 2, seed=2312, batch=B, device="cuda")
    trace = MaskTrace(ctx, cfg.layers, cfg.ffn)
    out = torch.full_like(x0, float("nan"))
    plan = pf.Plan(ctx, Ls, x0, out)
    plan.run()
    torch.cuda.synchronize()
    plan.close()
    eager = torch.empty_like(x0)
    ctx.profile_begin()
    ctx.stack_step(Ls, x0, eager)
    stats = ctx.profile_end()
    ctx.set_mask_trace(None)
    assert stats["k_la_up_hidden"][0] == 3 and stats["k_la_down_out"][0] == 3, stats
    assert torch.equal(eager, out)
    Os = [oracle_layer(cfg, wl.to_host(t)) for t in lays]
    ref, n_cmp, in_band = oracle_lookahead_chain_on_device_sets(
        oracle, Os, x0.cpu().numpy(), trace.masks(), cfg.threshold, name)
    assert n_cmp == cfg.layers
    assert in_band < 0.005 * cfg.ffn * B * cfg.layers + 16
    check_output(out.cpu().numpy(), ref, name + " look-ahead stack")
