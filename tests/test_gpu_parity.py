"""GPU parity: every entry point of libpf against the CPU oracle, element by element, on the
same seeded inputs.  Sizes span several 512-element chunks with ragged tails, several mask
words, several column tiles and neuron chunks."""
import numpy as np
import pytest
import torch

from paper_2312_12456_amd import workload as wl
from tests.util import check_active_set, check_output, oracle_layer, small_cfg

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pf():
    from paper_2312_12456_amd import pf as pfmod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pfmod.lib()
    return pfmod


def _setup(pf, cfg, seed, max_batch=8, pred_bias=True, layer=0):
    lay = wl.make_layer(cfg, layer, seed, device="cuda", pred_bias=pred_bias)
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=max_batch)
    L = pf.Layer.from_workload(ctx, cfg, lay)
    O = oracle_layer(cfg, wl.to_host(lay))
    return ctx, L, O, lay


def _words_to_mask(words, ffn):
    w = words.cpu().numpy().view(np.uint64)
    bits = np.unpackbits(w.view(np.uint8), bitorder="little")
    return bits[:ffn].astype(bool)


SHAPES = [
    # d, ffn, r : ragged last chunk (520 = 512 + 8), 21 mask words, r below one chunk
    dict(d=520, ffn=1344, r=136),
    # the OPT-125m layer of the first configuration
    dict(d=768, ffn=3072, r=128),
    # several chunks in both GEMVs, ragged r
    dict(d=2056, ffn=2048, r=1032),
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("B", [1, 3, 8])
def test_predict(pf, shape, B):
    cfg = small_cfg(rate=0.1, **shape)
    ctx, L, O, _ = _setup(pf, cfg, seed=100 + B)
    x = wl.make_inputs(cfg, 0, seed=5, batch=B, device="cuda")
    scores = torch.full((B, cfg.ffn), -1.0, device="cuda")
    words = torch.zeros(cfg.ffn // 64, dtype=torch.int64, device="cuda")
    ctx.predict(L, x, scores, words)
    torch.cuda.synchronize()
    ref = O.predict(x.cpu().numpy())
    np.testing.assert_allclose(scores.cpu().numpy(), ref["scores"], atol=2e-5, rtol=0)
    mask = _words_to_mask(words, cfg.ffn)
    check_active_set(mask, ref["scores"], cfg.threshold, "predict")
    assert 0 < mask.sum() < cfg.ffn
    # without the optional scores output the mask is the same
    words2 = torch.zeros_like(words)
    ctx.predict(L, x, None, words2)
    torch.cuda.synchronize()
    assert torch.equal(words, words2)


def test_predict_threshold_other_than_half(pf):
    cfg = wl.scaled(small_cfg(d=520, ffn=1344, r=136), threshold=0.8)
    ctx, L, O, _ = _setup(pf, cfg, seed=7)
    x = wl.make_inputs(cfg, 1, seed=5, batch=2, device="cuda")
    words = torch.zeros(cfg.ffn // 64, dtype=torch.int64, device="cuda")
    ctx.predict(L, x, None, words)
    torch.cuda.synchronize()
    ref = O.predict(x.cpu().numpy())
    check_active_set(_words_to_mask(words, cfg.ffn), ref["scores"], 0.8, "predict tau=0.8")


@pytest.mark.parametrize("ffn,density", [(64, 0.5), (128, 0.0), (128, 1.0), (3072, 0.1),
                                         (16384, 0.08), (49152, 0.04), (49152, 1.0),
                                         (65536 * 2, 0.3)])
def test_compact_bit_exact(pf, oracle, ffn, density):
    rng = np.random.default_rng(ffn + int(density * 100))
    mask = rng.random(ffn) < density if 0 < density < 1 else np.full(ffn, density == 1.0)
    words_np = np.packbits(mask, bitorder="little").view(np.uint64)
    words = torch.from_numpy(words_np.view(np.int64).copy()).cuda()
    ctx = pf.Context(64, 64, 8)
    idx = torch.full((ffn,), -7, dtype=torch.int32, device="cuda")
    count = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    ctx.compact(words, ffn, idx, count)
    torch.cuda.synchronize()
    ref = oracle.compact(mask)
    n = int(count.item())
    assert n == ref.size
    assert np.array_equal(idx.cpu().numpy()[:n], ref)


@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_REGLU, wl.ACT_DRELU])
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("B", [1, 2, 5, 8])
def test_sparse_ffn_exact_mask(pf, oracle, act, shape, B):
    """Exact-mask mode: the list is built by the oracle, so only the FFN arithmetic is compared."""
    cfg = small_cfg(rate=0.12, act=act, **shape)
    ctx, L, O, lay = _setup(pf, cfg, seed=200 + B + act)
    x = wl.make_inputs(cfg, 0, seed=6, batch=B, device="cuda")
    xh = x.cpu().numpy()
    mask = O.exact_mask(xh)
    ref_idx = oracle.compact(mask)
    idx = torch.zeros(cfg.ffn, dtype=torch.int32, device="cuda")
    idx[:ref_idx.size] = torch.from_numpy(ref_idx).cuda()
    count = torch.tensor([ref_idx.size], dtype=torch.int32, device="cuda")
    y = torch.full((B, cfg.d), float("nan"), device="cuda")
    ctx.sparse_ffn(L, x, idx, count, y)
    torch.cuda.synchronize()
    ref = O.masked_ffn(xh, mask)
    check_output(y.cpu().numpy(), ref, "exact mask")
    # the paper's identity: the exact mask reproduces the dense block
    check_output(y.cpu().numpy(), O.dense_ffn(xh), "exact mask vs dense")
    # deterministic: a second run gives the same bits
    y2 = torch.empty_like(y)
    ctx.sparse_ffn(L, x, idx, count, y2)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)


@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_REGLU])
def test_sparse_ffn_degenerate_lists(pf, oracle, act):
    cfg = small_cfg(d=520, ffn=1344, r=136, act=act)
    ctx, L, O, lay = _setup(pf, cfg, seed=31 + act)
    B = 2
    x = wl.make_inputs(cfg, 0, seed=6, batch=B, device="cuda")
    xh = x.cpu().numpy()
    y = torch.full((B, cfg.d), float("nan"), device="cuda")
    # empty list: y = b_down (or zero)
    idx = torch.zeros(cfg.ffn, dtype=torch.int32, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    ctx.sparse_ffn(L, x, idx, count, y)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().astype(np.float64),
                          O.masked_ffn(xh, np.zeros(cfg.ffn, bool)))
    # full list: the dense block
    idx = torch.arange(cfg.ffn, dtype=torch.int32, device="cuda")
    count = torch.tensor([cfg.ffn], dtype=torch.int32, device="cuda")
    ctx.sparse_ffn(L, x, idx, count, y)
    torch.cuda.synchronize()
    check_output(y.cpu().numpy(), O.dense_ffn(xh), "all-ones mask")
    # a single neuron, and a count larger than the capacity is clamped
    one = torch.tensor([cfg.ffn - 1], dtype=torch.int32, device="cuda")
    idx1 = torch.zeros(cfg.ffn, dtype=torch.int32, device="cuda")
    idx1[0] = one[0]
    ctx.sparse_ffn(L, x, idx1, torch.tensor([1], dtype=torch.int32, device="cuda"), y)
    torch.cuda.synchronize()
    m = np.zeros(cfg.ffn, bool)
    m[-1] = True
    check_output(y.cpu().numpy(), O.masked_ffn(xh, m), "single neuron")
    # out-of-range entries are skipped, not read
    bad = torch.tensor([3, 7, cfg.ffn + 5, -2], dtype=torch.int32, device="cuda")
    idxb = torch.zeros(cfg.ffn, dtype=torch.int32, device="cuda")
    idxb[:4] = bad
    ctx.sparse_ffn(L, x, idxb, torch.tensor([4], dtype=torch.int32, device="cuda"), y)
    torch.cuda.synchronize()
    m = np.zeros(cfg.ffn, bool)
    m[[3, 7]] = True
    check_output(y.cpu().numpy(), O.masked_ffn(xh, m), "skip invalid")


@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_REGLU, wl.ACT_DRELU])
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("B", [1, 4])
def test_layer_step_predicted_mask(pf, oracle, act, shape, B):
    cfg = small_cfg(rate=0.1, act=act, **shape)
    ctx, L, O, lay = _setup(pf, cfg, seed=300 + B + act)
    x = wl.make_inputs(cfg, 2, seed=8, batch=B, device="cuda")
    xh = x.cpu().numpy()
    y = torch.full((B, cfg.d), float("nan"), device="cuda")
    ctx.layer_step(L, x, y)
    torch.cuda.synchronize()
    # the active set the library used
    wptr, iptr, cptr = ctx.last_active()
    n_words = cfg.ffn // 64
    words = torch.empty(n_words, dtype=torch.int64, device="cuda")
    idx = torch.empty(cfg.ffn, dtype=torch.int32, device="cuda")
    count = torch.empty(1, dtype=torch.int32, device="cuda")
    pf.copy_from_device_address(words, wptr)
    pf.copy_from_device_address(idx, iptr)
    pf.copy_from_device_address(count, cptr)
    n = int(count.item())
    mask = _words_to_mask(words, cfg.ffn)
    ref = O.predict(xh)
    check_active_set(mask, ref["scores"], cfg.threshold, "layer_step")
    # index list == compaction of the mask, bit exact
    assert n == int(mask.sum())
    assert np.array_equal(idx.cpu().numpy()[:n], oracle.compact(mask))
    # output against the oracle run on the library's own set (band flips kept out)
    check_output(y.cpu().numpy(), O.masked_ffn(xh, mask), "layer_step")


def test_layer_step_bias_free_predictor_fires_half(pf, oracle):
    """First configuration as stated: random predictor without logit bias (about half fire)."""
    cfg = wl.CONFIGS["opt-125m-layer"]
    ctx, L, O, lay = _setup(pf, cfg, seed=1, pred_bias=False, max_batch=1)
    compared = 0
    for t in range(4):
        x = wl.make_inputs(cfg, t, seed=1, batch=1, device="cuda")
        y = torch.empty((1, cfg.d), device="cuda")
        ctx.layer_step(L, x, y)
        torch.cuda.synchronize()
        wptr, _, _ = ctx.last_active()
        words = torch.empty(cfg.ffn // 64, dtype=torch.int64, device="cuda")
        pf.copy_from_device_address(words, wptr)
        mask = _words_to_mask(words, cfg.ffn)
        xh = x.cpu().numpy()
        assert 0.4 < mask.mean() < 0.6
        # the set bit-exact outside the score band; the output against the oracle run on the
        # library's own set, so a flip inside the band cannot leak into the comparison
        check_active_set(mask, O.predict(xh)["scores"], cfg.threshold, "bias-free token %d" % t)
        check_output(y.cpu().numpy(), O.masked_ffn(xh, mask), "layer_step token %d" % t)
        compared += 1
    assert compared == 4


def test_stack_step_teacher_forced_and_plan_replay(pf, oracle):
    cfg = small_cfg(d=520, ffn=1344, r=136, layers=3)
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=2)
    lays = [wl.make_layer(cfg, l, seed=9, device="cuda") for l in range(cfg.layers)]
    Ls = [pf.Layer.from_workload(ctx, cfg, t) for t in lays]
    Os = [oracle_layer(cfg, wl.to_host(t)) for t in lays]
    B = 2
    x0 = wl.make_inputs(cfg, 0, seed=9, batch=B, device="cuda")
    # teacher forcing: every GPU layer + glue starts from the oracle's input to that layer
    xo = x0.cpu().numpy()
    for l in range(cfg.layers):
        xg = torch.from_numpy(xo).cuda()
        y = torch.empty((B, cfg.d), device="cuda")
        xn = torch.empty((B, cfg.d), device="cuda")
        ctx.layer_step(Ls[l], xg, y)
        ctx.stack_glue(xg, y, xn)
        torch.cuda.synchronize()
        wptr, _, _ = ctx.last_active()
        words = torch.empty(cfg.ffn // 64, dtype=torch.int64, device="cuda")
        pf.copy_from_device_address(words, wptr)
        mask = _words_to_mask(words, cfg.ffn)
        check_active_set(mask, Os[l].predict(xo)["scores"], cfg.threshold, "stack layer %d" % l)
        y_ref = Os[l].masked_ffn(xo, mask)
        check_output(y.cpu().numpy(), y_ref, "stack layer %d" % l)
        x_ref = oracle.stack_glue(xo, y_ref)
        np.testing.assert_allclose(xn.cpu().numpy(), x_ref, atol=2e-2, rtol=0)
        np.testing.assert_allclose((xn.double() ** 2).sum(dim=1).cpu().numpy(), cfg.d, rtol=1e-4)
        xo = oracle.stack_glue(xo, Os[l].layer_step(xo))
    # whole stack on the device: eager == graph replay, bit for bit, replay after replay
    out_eager = torch.empty_like(x0)
    ctx.stack_step(Ls, x0, out_eager)
    torch.cuda.synchronize()
    assert torch.isfinite(out_eager).all()
    # the stack fuses the glue into the next layer's predictor kernel: it must agree with the
    # chain of stand-alone layer_step + stack_glue calls checked above (same sets, fp32 rounding)
    xc = x0.clone()
    yc = torch.empty_like(x0)
    for l in range(cfg.layers):
        ctx.layer_step(Ls[l], xc, yc)
        ctx.stack_glue(xc, yc, xc)
    torch.cuda.synchronize()
    np.testing.assert_allclose(out_eager.cpu().numpy(), xc.cpu().numpy(), atol=1e-4, rtol=0)
    out_plan = torch.zeros_like(x0)
    plan = pf.Plan(ctx, Ls, x0, out_plan)
    for _ in range(3):
        out_plan.zero_()
        plan.run()
        torch.cuda.synchronize()
        assert torch.equal(out_plan, out_eager)
        _ = (x0 * 2).sum().item()  # eager work between replays
    plan.close()


def test_argument_errors_reach_the_caller(pf):
    cfg = small_cfg(d=520, ffn=1344, r=136)
    ctx, L, O, lay = _setup(pf, cfg, seed=3, max_batch=2)
    x = wl.make_inputs(cfg, 0, seed=1, batch=3, device="cuda")
    y = torch.empty((3, cfg.d), device="cuda")
    with pytest.raises(pf.PfError) as e:
        ctx.layer_step(L, x, y)
    assert e.value.status == pf.PF_EINVAL
    with pytest.raises(pf.PfError) as e:
        pf.Layer(ctx, 520, 1000, 136, w_up=lay["w_up"], w_down=lay["w_down"])
    assert e.value.status == pf.PF_ESHAPE
    big = torch.zeros((1344, 1024), dtype=torch.float16, device="cuda")
    with pytest.raises(pf.PfError) as e:
        pf.Layer(ctx, 1024, 1344, 136, w_up=big, w_down=big)   # wider than the context
    assert e.value.status == pf.PF_ESHAPE
    for gated in (pf.ACT_REGLU, pf.ACT_DRELU):   # a gated layer needs its gate matrix
        with pytest.raises(pf.PfError) as e:
            pf.Layer(ctx, 520, 1344, 136, act=gated, w_up=lay["w_up"], w_down=lay["w_down"])
        assert e.value.status == pf.PF_EINVAL
    with pytest.raises(pf.PfError) as e:
        pf.Layer(ctx, 520, 1344, 136, act=3, w_up=lay["w_up"], w_down=lay["w_down"])
    assert e.value.status == pf.PF_EUNSUPPORTED


INT4_SHAPES = [
    # d % 128 == 0; 640 = a third of one 2048-element chunk, 2304 = one chunk + a ragged second
    dict(d=640, ffn=1344, r=136),
    dict(d=2304, ffn=2048, r=264),
]


@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_REGLU, wl.ACT_DRELU])
@pytest.mark.parametrize("shape", INT4_SHAPES)
@pytest.mark.parametrize("B", [1, 3])
def test_int4_exact_mask_and_layer_step(pf, oracle, act, shape, B):
    """int4 group-128 weights dequantised in the kernels: both the list-driven FFN and the
    whole layer step against the oracle, which reads the same packed bytes."""
    cfg = small_cfg(rate=0.12, act=act, wtype=wl.W_INT4_G128, **shape)
    ctx, L, O, lay = _setup(pf, cfg, seed=400 + B + act)
    x = wl.make_inputs(cfg, 0, seed=6, batch=B, device="cuda")
    xh = x.cpu().numpy()
    mask = O.exact_mask(xh)
    ref_idx = oracle.compact(mask)
    idx = torch.zeros(cfg.ffn, dtype=torch.int32, device="cuda")
    idx[:ref_idx.size] = torch.from_numpy(ref_idx).cuda()
    count = torch.tensor([ref_idx.size], dtype=torch.int32, device="cuda")
    y = torch.full((B, cfg.d), float("nan"), device="cuda")
    ctx.sparse_ffn(L, x, idx, count, y)
    torch.cuda.synchronize()
    check_output(y.cpu().numpy(), O.masked_ffn(xh, mask), "int4 exact mask")
    check_output(y.cpu().numpy(), O.dense_ffn(xh), "int4 exact mask vs dense")
    # empty list
    ctx.sparse_ffn(L, x, idx, torch.zeros(1, dtype=torch.int32, device="cuda"), y)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().astype(np.float64),
                          O.masked_ffn(xh, np.zeros(cfg.ffn, bool)))
    # whole layer step with the predicted set
    y.fill_(float("nan"))
    ctx.layer_step(L, x, y)
    torch.cuda.synchronize()
    wptr, iptr, cptr = ctx.last_active()
    words = torch.empty(cfg.ffn // 64, dtype=torch.int64, device="cuda")
    pf.copy_from_device_address(words, wptr)
    pmask = _words_to_mask(words, cfg.ffn)
    check_active_set(pmask, O.predict(xh)["scores"], cfg.threshold, "int4 layer_step")
    check_output(y.cpu().numpy(), O.masked_ffn(xh, pmask), "int4 layer_step")
    y2 = torch.empty_like(y)
    ctx.layer_step(L, x, y2)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)


@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_REGLU, wl.ACT_DRELU])
@pytest.mark.parametrize("d", [800, 2080])          # 25 and 65 K-steps of 32: ragged unroll tails
@pytest.mark.parametrize("B", [4, 7, 8])
def test_fc1_on_matrix_cores_matches_oracle_and_vector_path(pf, oracle, act, d, B):
    """From batch 4 on FC1 runs on MFMA (fp16 hi/lo split of x): same oracle bar, list slots
    spanning several 32-row passes with a ragged last pass, and agreement with the vector-ALU
    kernel forced through the PF_OPT_MFMA_MIN_BATCH option."""
    cfg = small_cfg(d=d, ffn=1344, r=136, rate=0.12, act=act)
    lay = wl.make_layer(cfg, 0, seed=500 + B + act, device="cuda")
    O = oracle_layer(cfg, wl.to_host(lay))
    x = wl.make_inputs(cfg, 0, seed=6, batch=B, device="cuda")
    xh = x.cpu().numpy()
    mask = O.exact_mask(xh)
    if mask.sum() % 32 == 0:          # keep the last 32-row pass ragged
        mask[np.flatnonzero(mask)[-1]] = False
    ref_idx = oracle.compact(mask)
    assert ref_idx.size % 32 != 0 and ref_idx.size > 64
    idx = torch.zeros(cfg.ffn, dtype=torch.int32, device="cuda")
    idx[:ref_idx.size] = torch.from_numpy(ref_idx).cuda()
    count = torch.tensor([ref_idx.size], dtype=torch.int32, device="cuda")
    outs = {}
    for name, min_b in (("mfma", 4), ("valu", 99)):
        ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=B)
        ctx.set_option(pf.OPT_MFMA_MIN_BATCH, min_b)
        L = pf.Layer.from_workload(ctx, cfg, lay)
        y = torch.full((B, cfg.d), float("nan"), device="cuda")
        ctx.sparse_ffn(L, x, idx, count, y)
        torch.cuda.synchronize()
        check_output(y.cpu().numpy(), O.masked_ffn(xh, mask), name + " exact mask")
        yl = torch.full((B, cfg.d), float("nan"), device="cuda")
        ctx.layer_step(L, x, yl)
        torch.cuda.synchronize()
        wptr, iptr, cptr = ctx.last_active()
        words = torch.empty(cfg.ffn // 64, dtype=torch.int64, device="cuda")
        lidx = torch.empty(cfg.ffn, dtype=torch.int32, device="cuda")
        cnt = torch.empty(1, dtype=torch.int32, device="cuda")
        pf.copy_from_device_address(words, wptr)
        pf.copy_from_device_address(lidx, iptr)
        pf.copy_from_device_address(cnt, cptr)
        pmask = _words_to_mask(words, cfg.ffn)
        assert np.array_equal(lidx.cpu().numpy()[:int(cnt.item())], oracle.compact(pmask))
        check_output(yl.cpu().numpy(), O.masked_ffn(xh, pmask), name + " layer_step")
        outs[name] = (y.cpu().numpy(), yl.cpu().numpy())
    np.testing.assert_allclose(outs["mfma"][0], outs["valu"][0], atol=2e-4, rtol=0)
    np.testing.assert_allclose(outs["mfma"][1], outs["valu"][1], atol=2e-4, rtol=0)


@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_REGLU])
def test_batch3_on_matrix_cores_small_shape(pf, oracle, act):
    """The batch-3 dispatch of long rows (d > 4096 sends three tokens to the matrix-core FC1
    and predictor kernels) exercised cheaply: the same kernels forced at a small shape."""
    cfg = small_cfg(d=800, ffn=1344, r=136, rate=0.12, act=act)
    lay = wl.make_layer(cfg, 0, seed=611 + act, device="cuda")
    O = oracle_layer(cfg, wl.to_host(lay))
    B = 3
    x = wl.make_inputs(cfg, 0, seed=6, batch=B, device="cuda")
    xh = x.cpu().numpy()
    ctx = pf.Context(cfg.d, cfg.ffn, cfg.r, max_batch=B)
    ctx.set_option(pf.OPT_MFMA_MIN_BATCH, 3)
    L = pf.Layer.from_workload(ctx, cfg, lay)
    y = torch.full((B, cfg.d), float("nan"), device="cuda")
    ctx.profile_begin()
    ctx.layer_step(L, x, y)
    stats = ctx.profile_end()
    torch.cuda.synchronize()
    assert stats["k_up_mfma"][0] == 1 and stats["k_up"][0] == 0, stats
    wptr, iptr, cptr = ctx.last_active()
    words = torch.empty(cfg.ffn // 64, dtype=torch.int64, device="cuda")
    pf.copy_from_device_address(words, wptr)
    pmask = _words_to_mask(words, cfg.ffn)
    check_active_set(pmask, O.predict(xh)["scores"], cfg.threshold, "batch 3 on the matrix cores")
    check_output(y.cpu().numpy(), O.masked_ffn(xh, pmask), "batch 3 on the matrix cores")
