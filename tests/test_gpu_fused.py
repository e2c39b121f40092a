"""GPU parity of the three-launch form of the layer step used inside a stack (predictor output
layer and FC1 in one kernel per 64-neuron segment, FC2 over the segments; PowerInfer Sec. 5.1 +
5.4): against the fp64 oracle -- every layer's active set bit-exact outside the score band,
and the stack output against the oracle's stack run on those sets -- and against the
four-launch form of the same library, for both ways of forming segments, batch 1..3, both
activations, ragged row lengths, and densities from a few to most neurons of a segment (every
round of the FC2 kernel)."""
import numpy as np
import pytest
import torch

from paper_2312_12456_amd import workload as wl
from tests.util import (MaskTrace, check_output, oracle_chain_on_device_sets, oracle_layer,
                        small_cfg)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pf():
    from paper_2312_12456_amd import pf as pfmod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pfmod.lib()
    return pfmod


def _ctx(pf, cfg, B, fused, strided):
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=B)
    ctx.set_option(pf.OPT_FUSED, fused)
    ctx.set_option(pf.OPT_SEG_STRIDED, strided)
    return ctx


CASES = [
    # d,    ffn,  r,   rate  (ffn / 64 segments; d with a ragged last chunk; r likewise)
    (520, 1344, 136, 0.10),
    (2056, 2048, 264, 0.15),
    (1024, 4160, 512, 0.04),
    (520, 1344, 136, 0.60),   # most segments need 4 to 6 rounds of 8 entries
]


@pytest.mark.parametrize("strided", [0, 1])
@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_REGLU, wl.ACT_DRELU])
@pytest.mark.parametrize("B", [1, 2, 3])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_fused_stack_matches_oracle_and_list_form(pf, oracle, case, B, act, strided):
    d, ffn, r, rate = CASES[case]
    cfg = small_cfg(d=d, ffn=ffn, r=r, act=act, rate=rate, layers=4)
    seed = 100 + 7 * case + B
    lays = [wl.make_layer(cfg, l, seed, device="cuda") for l in range(cfg.layers)]
    Os = [oracle_layer(cfg, wl.to_host(t)) for t in lays]
    x0 = wl.make_inputs(cfg, 0, seed=seed, batch=B, device="cuda")
    outs, compared = {}, 0
    for fused in (0, 2):
        ctx = _ctx(pf, cfg, B, fused, strided)
        assert ctx.get_option(pf.OPT_FUSED) == fused
        Ls = [pf.Layer.from_workload(ctx, cfg, t) for t in lays]
        trace = MaskTrace(ctx, cfg.layers, cfg.ffn)
        out = torch.full_like(x0, float("nan"))
        ctx.profile_begin()
        ctx.stack_step(Ls, x0, out)
        stats = ctx.profile_end()
        torch.cuda.synchronize()
        # the form asked for is the form that ran
        assert stats["k_out_up"][0] == (cfg.layers - 1 if fused else 0), stats
        assert stats["k_down_mask"][0] == (cfg.layers - 1 if fused else 0), stats
        outs[fused] = out.cpu().numpy()
        # against the oracle, always: the oracle's stack driven by the sets this run used, each
        # set bit-exact outside the score band
        ref, n_cmp, _ = oracle_chain_on_device_sets(oracle, Os, x0.cpu().numpy(), trace.masks(),
                                                    cfg.threshold, "fused=%d" % fused)
        check_output(outs[fused], ref, "stack (fused=%d) case %d B %d" % (fused, case, B))
        compared += n_cmp
        if fused:
            # the last layer keeps the caller-visible list: ascending, no duplicates, in range
            _, iptr, cptr = ctx.last_active()
            idx = torch.empty(cfg.ffn, dtype=torch.int32, device="cuda")
            cnt = torch.empty(1, dtype=torch.int32, device="cuda")
            pf.copy_from_device_address(idx, iptr)
            pf.copy_from_device_address(cnt, cptr)
            n = int(cnt.item())
            lst = idx.cpu().numpy()[:n]
            assert np.array_equal(lst, np.flatnonzero(trace.masks()[-1]))
            # replayed plan == eager, bit for bit (the plan also fills the trace)
            first = [m.copy() for m in trace.masks()]
            out_plan = torch.zeros_like(x0)
            plan = pf.Plan(ctx, Ls, x0, out_plan)
            for _ in range(2):
                out_plan.fill_(float("nan"))
                trace.buf.fill_(-1)
                plan.run()
                torch.cuda.synchronize()
                assert torch.equal(out_plan, out)
                assert all(np.array_equal(a, b) for a, b in zip(trace.masks(), first))
            plan.close()
        ctx.set_mask_trace(None)
    assert compared == 2 * cfg.layers
    # same predictor arithmetic, same FC1 arithmetic, another order of FC2's sum
    np.testing.assert_allclose(outs[2], outs[0], atol=2e-4, rtol=0)


def test_fused_form_is_what_runs_by_default(pf):
    """At the headline shape class (d <= 4096, batch 1) the inner layers of a stack take the
    three-launch form: the per-kernel profile of an eager step shows its kernels."""
    cfg = small_cfg(d=1024, ffn=2048, r=128, layers=3)
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=1)
    lays = [wl.make_layer(cfg, l, 5, device="cuda") for l in range(cfg.layers)]
    Ls = [pf.Layer.from_workload(ctx, cfg, t) for t in lays]
    x0 = wl.make_inputs(cfg, 0, seed=5, batch=1, device="cuda")
    out = torch.empty_like(x0)
    ctx.profile_begin()
    ctx.stack_step(Ls, x0, out)
    stats = ctx.profile_end()
    assert stats["k_out_up"][0] == 2 and stats["k_down_mask"][0] == 2
    assert stats["k_pred_out"][0] == 1 and stats["k_up"][0] == 1 and stats["k_down"][0] == 1
