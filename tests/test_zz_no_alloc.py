"""pf_layer_step_noalloc (the layer step for callers that cannot allocate: its scratch is a
fixed array in the library's device image) against pf_layer_step, through the C ABI: two calls
in a row on the same GPU, the second on a smaller layer, so that the shared array still holds
the first call's contents; and the limits are enforced before anything is launched."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2312_12456_amd import workload as wl
from tests.util import check_output, small_cfg

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pf():
    from paper_2312_12456_amd import pf as pfmod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pfmod.lib()
    return pfmod


def _both(pf, cfg, seed, B):
    lay = wl.make_layer(cfg, 0, seed, device="cuda")
    x = wl.make_inputs(cfg, 0, seed=seed, batch=B, device="cuda")
    # the existing entry point, with a context of its own
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=B)
    L = pf.Layer.from_workload(ctx, cfg, lay)
    y_ref = torch.full((B, cfg.d), float("nan"), device="cuda")
    ctx.layer_step(L, x, y_ref)
    torch.cuda.synchronize()
    # the entry point under test
    y = torch.full((B, cfg.d), float("nan"), device="cuda")
    pf.layer_step_noalloc(cfg, lay, x, y)
    torch.cuda.synchronize()
    return y.cpu().numpy(), y_ref.cpu().numpy()


def test_noalloc_layer_step_twice_second_call_smaller(pf):
    big = small_cfg(d=2056, ffn=4160, r=264, rate=0.15)
    small = small_cfg(d=520, ffn=1344, r=136, rate=0.08, act=wl.ACT_REGLU)
    for cfg, seed, B in ((big, 71, 3), (small, 72, 1), (big, 73, 4)):
        y, y_ref = _both(pf, cfg, seed, B)
        assert np.abs(y_ref).max() > 0.1
        check_output(y, y_ref, "noalloc vs layer_step d=%d B=%d" % (cfg.d, B))
        # the same kernels in the same launch shapes: not just within the bar but the same bits
        assert np.array_equal(y, y_ref)


def test_noalloc_on_matrix_cores_same_bits_from_fp32_operands(pf):
    """Batch 4 with rows of a multiple of 32 elements runs on the matrix cores.  pf_layer_step
    hands FC1 and the hidden layer the activations as fp16 hi + lo planes written by a small
    kernel in front; the entry point that allocates nothing has no buffer for the planes and
    splits inside the kernels.  Both are the same arithmetic: the outputs are equal bit for bit."""
    for act in (wl.ACT_RELU, wl.ACT_REGLU):
        cfg = small_cfg(d=6144, ffn=4160, r=256, rate=0.15, act=act)  # B * d above the hidden layer's matrix-core threshold
        y, y_ref = _both(pf, cfg, 74 + act, 4)
        assert np.abs(y_ref).max() > 0.1
        assert np.array_equal(y, y_ref)


def test_noalloc_rejects_sizes_beyond_its_limits(pf):
    lib = pf.lib()
    one = ctypes.c_void_p(256)  # never dereferenced: the limits are checked first
    w = pf.LayerWeights(*([one] * 11))
    for d, ffn, r, B in ((8192 + 8, 1024, 64, 1), (1024, 32768 + 64, 64, 1), (1024, 1024, 2048 + 8, 1),
                         (1024, 1024, 64, 5)):
        desc = pf.LayerDesc(d, ffn, r, pf.ACT_RELU, pf.W_FP16, 0.5)
        st = lib.pf_layer_step_noalloc(ctypes.byref(desc), ctypes.byref(w), one, B, one, None)
        assert st == pf.PF_ELIMIT, (d, ffn, r, B, st)
    assert b"limits" in lib.pf_strerror(pf.PF_ELIMIT)
    desc = pf.LayerDesc(1024, 1000, 64, pf.ACT_RELU, pf.W_FP16, 0.5)
    assert lib.pf_layer_step_noalloc(ctypes.byref(desc), ctypes.byref(w), one, 1, one, None) == pf.PF_ESHAPE
    assert lib.pf_layer_step_noalloc(None, None, None, 1, None, None) == pf.PF_EINVAL
