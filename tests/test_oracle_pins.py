"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests calls the HIP library.  Each is chosen so that a plausible mistake
in oracle/pf_oracle.c (dropped bias, wrong sign, transposed operand, wrong nibble,
mask ignored, wrong union rule) fails at least one of them.
"""
import itertools
import os

import numpy as np
import pytest

from paper_2312_12456_amd import workload as wl
from tests.util import oracle_layer, small_cfg

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rand_layer(oracle, d, F, r, act, seed, wtype=wl.W_FP16, with_bias=True):
    rng = np.random.default_rng(seed)
    kw = {}
    if wtype == wl.W_FP16:
        for nm in ("w_up", "w_down") + (("w_gate",) if act != wl.ACT_RELU else ()):
            kw[nm] = (rng.standard_normal((F, d)) / np.sqrt(d)).astype(np.float16)
    else:
        for nm in ("up", "down") + (("gate",) if act != wl.ACT_RELU else ()):
            kw["w_" + nm] = rng.integers(0, 256, (F, d // 2), dtype=np.uint8)
            kw["s_" + nm] = (rng.uniform(0.01, 0.05, (F, d // 128))).astype(np.float16)
    if with_bias:
        kw["b_up"] = rng.standard_normal(F).astype(np.float32) - 1.0
        kw["b_down"] = rng.standard_normal(d).astype(np.float32)
    kw["p1"] = (rng.standard_normal((r, d)) / np.sqrt(d)).astype(np.float16)
    kw["p2"] = (rng.standard_normal((F, r)) / np.sqrt(r)).astype(np.float16)
    kw["p_bias"] = rng.standard_normal(F).astype(np.float32) * 0.5
    L = oracle.Layer(d, F, r, act=act, wtype=wtype, threshold=0.5, **kw)
    return L, kw, rng


def _widen(oracle, L, kw, which):
    """Stored matrix -> float64 values, computed here independently of the oracle."""
    w = kw["w_" + which]
    if w.dtype == np.float16:
        return w.astype(np.float64)
    s = kw["s_" + which].astype(np.float64)
    lo = (w & 15).astype(np.int64) - 8
    hi = (w >> 4).astype(np.int64) - 8
    q = np.stack([lo, hi], axis=2).reshape(w.shape[0], -1)
    return q * np.repeat(s, 128, axis=1)


# --------------------------------------------------------------------------- fp16
def test_half_conversion_all_bit_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    same = (got == ref) | (np.isnan(got) & np.isnan(ref))
    assert same.all()
    assert np.array_equal(np.signbit(got), np.signbit(ref))


# ------------------------------------------------- I5: library matmul, closed forms
@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_REGLU, wl.ACT_DRELU])
@pytest.mark.parametrize("B", [1, 3])
def test_dense_ffn_matches_fp64_matmul(oracle, act, B):
    d, F, r = 96, 160, 16
    L, kw, rng = _rand_layer(oracle, d, F, r, act, seed=10 + act)
    x = rng.standard_normal((B, d)).astype(np.float32)
    X = x.astype(np.float64)
    Wu, Wd = kw["w_up"].astype(np.float64), kw["w_down"].astype(np.float64)
    if act == wl.ACT_RELU:
        pre = X @ Wu.T + kw["b_up"].astype(np.float64)
        h = np.maximum(pre, 0)
    elif act == wl.ACT_REGLU:
        pre = X @ kw["w_gate"].astype(np.float64).T + kw["b_up"].astype(np.float64)
        h = np.maximum(pre, 0) * (X @ Wu.T)
    else:
        g = X @ kw["w_gate"].astype(np.float64).T + kw["b_up"].astype(np.float64)
        u = X @ Wu.T
        pre = np.minimum(g, u)
        h = np.maximum(g, 0) * np.maximum(u, 0)
    y = h @ Wd + kw["b_down"].astype(np.float64)
    np.testing.assert_allclose(L.preact(x), pre, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(L.dense_ffn(x), y, rtol=1e-11, atol=1e-12)


def test_fc2_is_not_transposed_or_unbiased(oracle):
    """One neuron, unit input: y must be b_down + h * (that neuron's stored row)."""
    d, F, r = 8, 4, 2
    w_up = np.zeros((F, d), np.float16)
    w_down = np.zeros((F, d), np.float16)
    w_up[2, 5] = 2.0                      # neuron 2 looks at x[5]
    w_down[2, :] = np.arange(1, d + 1)    # and writes 1..d
    b_up = np.array([0, 0, 0.5, 0], np.float32)
    b_down = np.full(d, 10.0, np.float32)
    L = oracle.Layer(d, F, r, w_up=w_up, w_down=w_down, b_up=b_up, b_down=b_down)
    x = np.zeros((1, d), np.float32)
    x[0, 5] = 3.0
    want = 10.0 + (2 * 3 + 0.5) * np.arange(1, d + 1)
    assert np.array_equal(L.dense_ffn(x)[0], want)
    x[0, 5] = -3.0                         # ReLU closes the neuron: only the bias is left
    assert np.array_equal(L.dense_ffn(x)[0], np.full(d, 10.0))


def test_drelu_closes_on_either_branch(oracle):
    """dReLU (ReLU on the gate branch and on the up branch; the Bamboo-7B row of the paper's
    model table): one neuron whose gate reads x[0] and whose up branch reads x[1].  It
    contributes g * u only when both are positive; the plain gated form differs exactly where
    the up branch is negative."""
    d, F, r = 8, 2, 2
    w_gate = np.zeros((F, d), np.float16)
    w_up = np.zeros((F, d), np.float16)
    w_down = np.zeros((F, d), np.float16)
    w_gate[1, 0] = 1.0
    w_up[1, 1] = 1.0
    w_down[1, :] = 1.0
    for gx, ux in ((2.0, 3.0), (2.0, -3.0), (-2.0, 3.0), (-2.0, -3.0)):
        x = np.zeros((1, d), np.float32)
        x[0, 0], x[0, 1] = gx, ux
        both = max(gx, 0.0) * max(ux, 0.0)
        kw = dict(w_gate=w_gate, w_up=w_up, w_down=w_down, b_up=np.zeros(F, np.float32))
        Ld = oracle.Layer(d, F, r, act=wl.ACT_DRELU, **kw)
        Lg = oracle.Layer(d, F, r, act=wl.ACT_REGLU, **kw)
        assert np.array_equal(Ld.dense_ffn(x)[0], np.full(d, both))
        assert np.array_equal(Lg.dense_ffn(x)[0], np.full(d, max(gx, 0.0) * ux))
        assert Ld.exact_mask(x).tolist() == [False, gx > 0 and ux > 0]
        assert Lg.exact_mask(x).tolist() == [False, gx > 0]
        # with a gate bias: the bias belongs to the gate branch only
        kw["b_up"] = np.array([0.0, 5.0], np.float32)
        Lb = oracle.Layer(d, F, r, act=wl.ACT_DRELU, **kw)
        assert np.array_equal(Lb.dense_ffn(x)[0], np.full(d, max(gx + 5.0, 0.0) * max(ux, 0.0)))


def test_predictor_matches_fp64_matmul_and_threshold_is_strict(oracle):
    d, F, r = 64, 200, 24
    L, kw, rng = _rand_layer(oracle, d, F, r, wl.ACT_RELU, seed=3)
    x = rng.standard_normal((4, d)).astype(np.float32)
    t = np.maximum(x.astype(np.float64) @ kw["p1"].astype(np.float64).T, 0)
    logit = t @ kw["p2"].astype(np.float64).T + kw["p_bias"].astype(np.float64)
    score = 1 / (1 + np.exp(-logit))
    out = L.predict(x)
    np.testing.assert_allclose(out["hidden"], t, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(out["logits"], logit, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(out["scores"], score, rtol=1e-12)
    assert np.array_equal(out["active_rows"], out["scores"] > 0.5)
    assert np.array_equal(out["active"], (out["scores"] > 0.5).any(axis=0))
    # strict comparison: a logit of exactly 0 scores exactly 0.5 and is NOT active
    z = oracle.Layer(d, F, r, threshold=0.5, p1=np.zeros((r, d), np.float16), p2=kw["p2"])
    o = z.predict(x[:1])
    assert np.all(o["scores"] == 0.5) and not o["active"].any()


def test_predictor_selector_special_case(oracle):
    """P1 picks coordinates, P2 = +/- identity-like rows: the active set is readable."""
    d, F, r = 16, 6, 4
    p1 = np.zeros((r, d), np.float16)
    for m in range(r):
        p1[m, m] = 1.0                       # hidden m = relu(x[m])
    p2 = np.zeros((F, r), np.float16)
    p2[0, 0] = 1.0                           # fires iff x0 > 0
    p2[1, 1] = -1.0                          # never fires (-relu <= 0, strict)
    p2[2, 2] = 1.0
    p2[3, 3] = 1.0
    p_bias = np.array([0, 0, 0, 0, 50.0, -50.0], np.float32)
    L = oracle.Layer(d, F, r, p1=p1, p2=p2, p_bias=p_bias)
    x = np.zeros((1, d), np.float32)
    x[0, :4] = [2.0, 5.0, -1.0, 0.0]
    assert L.predict(x)["active"].tolist() == [True, False, False, False, True, False]
    # union over a batch: second token opens neuron 2
    x2 = np.concatenate([x, x])
    x2[1, 2] = 4.0
    x2[1, 0] = -4.0
    out = L.predict(x2)
    assert out["active"].tolist() == [True, False, True, False, True, False]
    assert out["active_rows"][1].tolist() == [False, False, True, False, True, False]


# -------------------------------------------- I1, I2, I3, I8: the paper's identities
@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_REGLU, wl.ACT_DRELU])
@pytest.mark.parametrize("wtype", [wl.W_FP16, wl.W_INT4_G128])
def test_mask_identities(oracle, act, wtype):
    d, F, r = 128, 192, 16
    L, kw, rng = _rand_layer(oracle, d, F, r, act, seed=20 + act + 2 * wtype, wtype=wtype)
    B = 3
    x = rng.standard_normal((B, d)).astype(np.float32)
    dense = L.dense_ffn(x)
    bd = kw["b_down"].astype(np.float64)
    # I1: all-ones mask == dense
    assert np.array_equal(L.masked_ffn(x, np.ones(F, bool)), dense)
    # I2: exact ReLU-positive mask (union over the batch) == dense
    pre = L.preact(x)
    exact = (pre > 0).any(axis=0)
    assert np.array_equal(L.exact_mask(x), exact)
    assert 0 < exact.sum() < F
    assert np.array_equal(L.masked_ffn(x, exact), dense)
    # I3a: false positives are harmless
    fp = exact.copy()
    fp[np.flatnonzero(~exact)[:17]] = True
    assert np.array_equal(L.masked_ffn(x, fp), dense)
    # I3b: dropping one true positive removes exactly that neuron's term
    i = int(np.flatnonzero(pre[0] > 0)[3])
    fn = exact.copy()
    fn[i] = False
    Wd = _widen(oracle, L, kw, "down")
    Wu = _widen(oracle, L, kw, "up")
    X = x.astype(np.float64)
    if act == wl.ACT_RELU:
        h_i = np.maximum(pre[:, i], 0)
    elif act == wl.ACT_REGLU:
        h_i = np.maximum(pre[:, i], 0) * (X @ Wu[i])
    else:
        Wg = _widen(oracle, L, kw, "gate")
        h_i = np.maximum(X @ Wg[i] + float(kw["b_up"][i]), 0) * np.maximum(X @ Wu[i], 0)
    np.testing.assert_allclose(dense - L.masked_ffn(x, fn), np.outer(h_i, Wd[i]),
                               rtol=1e-9, atol=1e-12)
    # empty mask leaves the FC2 bias
    assert np.array_equal(L.masked_ffn(x, np.zeros(F, bool)), np.broadcast_to(bd, (B, d)))
    # I8: linearity over disjoint masks
    m1 = np.zeros(F, bool)
    m1[::3] = True
    m2 = np.zeros(F, bool)
    m2[1::3] = True
    lhs = L.masked_ffn(x, m1 | m2) - bd
    rhs = (L.masked_ffn(x, m1) - bd) + (L.masked_ffn(x, m2) - bd)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-10, atol=1e-12)
    # index-list form == mask form, and layer_step == predict -> masked_ffn
    idx = oracle.compact(fp)
    y_idx, h = L.sparse_ffn_idx(x, idx, return_h=True)
    assert np.array_equal(y_idx, L.masked_ffn(x, fp))
    if act == wl.ACT_RELU:
        assert np.array_equal(h, np.maximum(pre[:, idx], 0))
    y_step, m_step = L.layer_step(x, return_mask=True)
    assert np.array_equal(m_step, L.predict(x)["active"])
    assert np.array_equal(y_step, L.masked_ffn(x, m_step))


def test_paper_single_layer_example_sets(oracle):
    """Sec. 4.2 example: predicted {3,4,5}; GPU part {3,5} + CPU part {4} merge to it."""
    sets = {}
    with open(os.path.join(GOLDEN, "single_layer_example.txt")) as f:
        for line in f:
            if line.startswith("#") or "=" not in line:
                continue
            k, v = line.split("=")
            sets[k.strip()] = [int(t) for t in v.split()]
    d, F, r = 32, 8, 4
    L, kw, rng = _rand_layer(oracle, d, F, r, wl.ACT_RELU, seed=5)
    x = rng.standard_normal((1, d)).astype(np.float32)

    def m(ids):
        a = np.zeros(F, bool)
        a[ids] = True
        return a

    assert oracle.compact(m(sets["predicted"])).tolist() == sets["predicted"]
    assert sorted(set(sets["predicted"]) & set(sets["hot"])) == sets["gpu_computes"]
    assert sorted(set(sets["predicted"]) - set(sets["hot"])) == sets["cpu_computes"]
    bd = kw["b_down"].astype(np.float64)
    merged = (L.masked_ffn(x, m(sets["gpu_computes"])) - bd) + \
             (L.masked_ffn(x, m(sets["cpu_computes"])) - bd) + bd
    np.testing.assert_allclose(L.masked_ffn(x, m(sets["predicted"])), merged, rtol=1e-12)
    # neuron 7 is hot but not predicted: it must not contribute
    with7 = L.masked_ffn(x, m(sets["predicted"] + sets["skipped_hot"]))
    pre7 = L.preact(x)[0, 7]
    changed = not np.array_equal(with7, L.masked_ffn(x, m(sets["predicted"])))
    assert changed == (pre7 > 0)


# ------------------------------------------------ I4: brute force on tiny layers
def _brute_force(act, W_up, W_gate, W_dT, b_up, b_down, x, mask):
    """Scalar loops in exact integer arithmetic (python ints)."""
    F, d = len(W_up), len(x)
    y = [int(v) for v in b_down]
    for i in range(F):
        if not mask[i]:
            continue
        if act == wl.ACT_RELU:
            z = sum(int(W_up[i][c]) * int(x[c]) for c in range(d)) + int(b_up[i])
            h = z if z > 0 else 0
        else:
            g = sum(int(W_gate[i][c]) * int(x[c]) for c in range(d)) + int(b_up[i])
            u = sum(int(W_up[i][c]) * int(x[c]) for c in range(d))
            if act == wl.ACT_DRELU and u < 0:
                u = 0
            h = (g if g > 0 else 0) * u
        for c in range(d):
            y[c] += h * int(W_dT[i][c])
    return y


@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_REGLU, wl.ACT_DRELU])
def test_brute_force_all_masks_tiny_layer(oracle, act):
    d, F, r = 6, 9, 2
    rng = np.random.default_rng(77 + act)
    W_up = rng.integers(-4, 5, (F, d))
    W_gate = rng.integers(-4, 5, (F, d))
    W_dT = rng.integers(-4, 5, (F, d))
    b_up = rng.integers(-3, 4, F)
    b_down = rng.integers(-3, 4, d)
    x = rng.integers(-3, 4, d)
    L = oracle.Layer(d, F, r, act=act, w_up=W_up.astype(np.float16),
                     w_gate=W_gate.astype(np.float16), w_down=W_dT.astype(np.float16),
                     b_up=b_up.astype(np.float32), b_down=b_down.astype(np.float32))
    xf = x.astype(np.float32)[None]
    dense = L.dense_ffn(xf)[0]
    for bits in itertools.product([0, 1], repeat=F):
        mask = np.array(bits, bool)
        want = _brute_force(act, W_up, W_gate, W_dT, b_up, b_down, x, mask)
        got = L.masked_ffn(xf, mask)[0]
        assert got.tolist() == [float(v) for v in want], bits
        got_idx = L.sparse_ffn_idx(xf, np.flatnonzero(mask))[0]
        assert got_idx.tolist() == [float(v) for v in want]
    assert dense.tolist() == [float(v) for v in
                              _brute_force(act, W_up, W_gate, W_dT, b_up, b_down, x, [1] * F)]


def test_compact_all_16_bit_masks(oracle):
    for v in range(1 << 16):
        mask = [(v >> b) & 1 for b in range(16)]
        want = [b for b in range(16) if mask[b]]
        assert oracle.compact(np.array(mask)).tolist() == want


def test_compact_long_random(oracle):
    rng = np.random.default_rng(1)
    for F in (1, 63, 64, 65, 3072, 49152):
        mask = rng.random(F) < 0.07
        idx = oracle.compact(mask)
        assert np.array_equal(idx, np.flatnonzero(mask))
        assert idx.dtype == np.int32


# ----------------------------------------------------------------- I6: int4 format
def test_int4_dequant_all_nibbles_and_positions(oracle):
    d, F, r = 256, 3, 2
    q = np.zeros((F, d // 2), np.uint8)
    s = np.array([[0.5, 0.25], [1.0, 2.0], [0.125, 3.0]], np.float16)
    # row 0: element c holds nibble c % 16 -> byte j = (2j % 16) | ((2j+1) % 16) << 4
    for j in range(d // 2):
        q[0, j] = ((2 * j) % 16) | (((2 * j + 1) % 16) << 4)
        q[1, j] = (15 - (2 * j) % 16) | ((15 - (2 * j + 1) % 16) << 4)
        q[2, j] = 0x8F if j % 2 else 0xF8
    L = oracle.Layer(d, F, r, wtype=wl.W_INT4_G128, w_up=q, s_up=s, w_down=q, s_down=s)
    for c in range(d):
        g = c // 128
        assert L.weight_value("up", 0, c) == float(s[0, g]) * ((c % 16) - 8)
        assert L.weight_value("down", 1, c) == float(s[1, g]) * ((15 - c % 16) - 8)
    # byte 0xF8: low nibble 8 -> 0, high nibble 15 -> +7 * scale
    assert L.weight_value("up", 2, 0) == 0.0 and L.weight_value("up", 2, 1) == 7 * 0.125
    assert L.weight_value("up", 2, 2) == 7 * 0.125 and L.weight_value("up", 2, 3) == 0.0


def test_int4_ffn_equals_ffn_on_dequantised_values(oracle):
    """masked_ffn on packed int4 == fp64 matmul on the dequantised arrays."""
    d, F, r = 256, 96, 8
    L, kw, rng = _rand_layer(oracle, d, F, r, wl.ACT_RELU, seed=9, wtype=wl.W_INT4_G128)
    x = rng.standard_normal((2, d)).astype(np.float32)
    Wu, Wd = _widen(oracle, L, kw, "up"), _widen(oracle, L, kw, "down")
    pre = x.astype(np.float64) @ Wu.T + kw["b_up"].astype(np.float64)
    mask = rng.random(F) < 0.5
    y = (np.maximum(pre, 0) * mask) @ Wd + kw["b_down"].astype(np.float64)
    np.testing.assert_allclose(L.masked_ffn(x, mask), y, rtol=1e-11, atol=1e-11)


def test_quantiser_round_trip_error_bound(oracle):
    """workload.quantize_int4_g128 -> oracle dequant is within half a step of the input."""
    import torch
    g = torch.Generator().manual_seed(4)
    w = torch.randn((8, 256), generator=g) * 0.05
    q, s = wl.quantize_int4_g128(w)
    L = oracle.Layer(256, 8, 2, wtype=wl.W_INT4_G128, w_up=q.numpy(), s_up=s.numpy())
    deq = np.array([[L.weight_value("up", i, c) for c in range(256)] for i in range(8)])
    step = np.repeat(s.numpy().astype(np.float64), 128, axis=1)
    assert np.all(np.abs(deq - w.numpy()) <= 0.5 * step + 1e-6)


# ------------------------------------------------------------------- stack glue
def test_stack_glue_norm_and_direction(oracle):
    rng = np.random.default_rng(2)
    x = rng.standard_normal((3, 40)).astype(np.float32)
    y = rng.standard_normal((3, 40))
    out = oracle.stack_glue(x, y)
    v = x.astype(np.float64) + y
    want = v * np.sqrt(40.0) / np.linalg.norm(v, axis=1)[:, None]
    np.testing.assert_allclose(np.sum(out.astype(np.float64) ** 2, axis=1), 40.0, rtol=1e-6)
    np.testing.assert_allclose(out[0], want[0], rtol=1e-6)            # row 0: no sign change
    np.testing.assert_allclose(np.abs(out), np.abs(want), rtol=1e-6)  # other rows: magnitudes kept
    assert np.array_equal(oracle.stack_glue(np.zeros((1, 8), np.float32), np.zeros((1, 8))),
                          np.zeros((1, 8), np.float32))


def test_stack_glue_sign_pattern_decorrelates_rows(oracle):
    """Rows b >= 1 get a fixed +/-1 pattern: the same whatever the values, balanced, different
    from row to row, and it turns identical rows into nearly orthogonal ones."""
    d, B = 4096, 8
    ones = np.ones((B, d), np.float32)
    s = oracle.stack_glue(ones, np.zeros((B, d)))       # = the pattern itself (unit rms input)
    assert np.array_equal(np.abs(s), ones) and np.array_equal(s[0], ones[0])
    rng = np.random.default_rng(9)
    x = rng.standard_normal((B, d)).astype(np.float32)
    y = rng.standard_normal((B, d))
    out = oracle.stack_glue(x, y)
    assert np.array_equal(np.sign(out), np.sign(x + y) * s)  # independent of the values
    for b in range(1, B):
        assert abs(s[b].mean()) < 0.06                       # balanced: |mean| < 4 sigma
        for b2 in range(b):
            assert abs(np.mean(s[b] * s[b2])) < 0.07         # rows uncorrelated
    same = np.tile(x[:1], (B, 1))
    o = oracle.stack_glue(same, np.zeros((B, d))).astype(np.float64)
    cos = (o @ o.T) / d
    assert np.all(np.abs(cos[np.triu_indices(B, 1)]) < 0.08)


# ------------------------------------------------- I7: the generator's statistics
def test_workload_activation_statistics(oracle):
    cfg = small_cfg(d=256, ffn=1024, r=32, rate=0.08, alpha=1.2)
    lay = wl.make_layer(cfg, 0, seed=11)
    p = lay["p"]
    assert abs(p.mean() - 0.08) < 1e-6 and p.max() <= wl.P_MAX
    L = oracle_layer(cfg, wl.to_host(lay))
    T = 2048
    x = np.concatenate([wl.make_inputs(cfg, t, seed=11, batch=64).numpy()
                        for t in range(T // 64)])
    fired = L.preact(x) > 0
    rate = fired.mean(axis=0)
    assert abs(fired.mean() - 0.08) < 0.01
    sigma = np.sqrt(p * (1 - p) / T)
    # weights are N(0,1/d) samples, so a row's norm deviates from 1 by ~1/sqrt(2d):
    # allow that model error on top of the binomial noise
    assert np.mean(np.abs(rate - p) < 4 * sigma + 0.03) > 0.99
    # power-law skew: a minority of neurons carries 80 % of all activations
    order = np.sort(rate)[::-1]
    share = np.searchsorted(np.cumsum(order) / order.sum(), 0.8) / cfg.ffn
    assert share < 0.45
    # predicted set with the logit bias fires at a similar mean rate
    pr = L.predict(x[:256])["active_rows"].mean()
    assert abs(pr - 0.08) < 0.02
    # expected union growth with batch
    u4 = wl.expected_union_rate(p, 4)
    got4 = fired[:1024].reshape(256, 4, -1).any(axis=1).mean()
    assert abs(got4 - u4) < 0.02


def test_workload_is_seeded_and_layers_differ():
    cfg = small_cfg()
    a = wl.make_layer(cfg, 0, seed=1)
    b = wl.make_layer(cfg, 0, seed=1)
    c = wl.make_layer(cfg, 1, seed=1)
    assert all(np.array_equal(wl.to_host(a)[k], wl.to_host(b)[k]) for k in ("w_up", "p2", "b_up"))
    assert not np.array_equal(wl.to_host(a)["w_up"], wl.to_host(c)["w_up"])
    assert np.array_equal(wl.make_inputs(cfg, 3, 1).numpy(), wl.make_inputs(cfg, 3, 1).numpy())


def test_neuron_permutation_leaves_the_function_unchanged(oracle):
    """Renumbering the neurons (frequency-sorted layout) permutes the predictor's mask and
    leaves dense, masked and predicted-mask outputs unchanged up to the order of an fp64 sum."""
    for act, wtype in ((wl.ACT_RELU, wl.W_FP16), (wl.ACT_REGLU, wl.W_FP16), (wl.ACT_RELU, wl.W_INT4_G128),
                       (wl.ACT_DRELU, wl.W_FP16)):
        cfg = small_cfg(d=256, ffn=320, r=48, act=act, wtype=wtype, rate=0.2)
        lay = wl.to_host(wl.make_layer(cfg, 0, seed=5))
        order = np.random.Generator(np.random.PCG64(3)).permutation(cfg.ffn)
        lay2 = wl.permute_neurons(lay, order)
        O, O2 = oracle_layer(cfg, lay), oracle_layer(cfg, lay2)
        x = wl.make_inputs(cfg, 0, seed=5, batch=2).numpy()
        np.testing.assert_allclose(O2.dense_ffn(x), O.dense_ffn(x), rtol=0, atol=1e-12)
        y, m = O.layer_step(x, return_mask=True)
        y2, m2 = O2.layer_step(x, return_mask=True)
        assert np.array_equal(m2, m[order]) and 0 < m.sum() < cfg.ffn
        np.testing.assert_allclose(y2, y, rtol=0, atol=1e-12)
        np.testing.assert_array_equal(O2.predict(x)["scores"], O.predict(x)["scores"][:, order])


def test_stack_lookahead_reads_the_previous_layers_input(oracle):
    """Look-ahead at distance 1, pinned with selector predictors whose active set can be read
    off the vector they are given: neuron m fires iff coordinate m of that vector is positive.
    Layer l >= 1 must list the sign pattern of the INPUT of layer l-1 -- not of its own input,
    which the layers here flip on purpose -- and layer 0 that of its own input."""
    d, F, r = 16, 16, 16
    eye = np.eye(d, dtype=np.float16)

    def layer(flip):
        # FFN: h_m = ReLU(x_m) on the listed coordinates, y = -2 h when flip (so that a listed
        # positive coordinate changes sign in x + y), else y = 0
        w_up = eye.copy()
        w_down = (-2.0 * eye if flip else 0.0 * eye).astype(np.float16)
        return oracle.Layer(d, F, r, w_up=w_up, w_down=w_down, p1=eye, p2=eye)

    layers = [layer(True), layer(False), layer(False)]
    x0 = np.array([[3, -1, 2, -4, 1, 5, -2, 6, -3, 1, 2, -1, 4, -5, 1, 2]], np.float32)
    out, masks = oracle.stack_lookahead(layers, x0)
    pos0 = x0[0] > 0
    assert np.array_equal(masks[0], pos0)            # layer 0: own input
    assert np.array_equal(masks[1], pos0)            # layer 1: input of layer 0
    # input of layer 1 = glue(x0 + y0): positive listed coordinates flipped, the rest kept
    x1 = x0[0].astype(np.float64).copy()
    x1[pos0] *= -1.0
    x1 *= np.sqrt(d) / np.linalg.norm(x1)
    assert not np.array_equal(x1 > 0, pos0)
    assert np.array_equal(masks[2], x1 > 0)          # layer 2: input of layer 1
    # layers 1 and 2 add nothing, so the output is the input of layer 1 (already unit rms)
    np.testing.assert_allclose(out[0], x1, rtol=0, atol=1e-6)
    # one layer: look-ahead is the plain layer step followed by the glue
    y, m = layers[0].layer_step(x0, return_mask=True)
    o1, m1 = oracle.stack_lookahead(layers[:1], x0)
    assert np.array_equal(m1[0], m)
    np.testing.assert_array_equal(o1, oracle.stack_glue(x0, y))


def test_oracle_is_clean_under_the_undefined_behaviour_sanitizer():
    """The identities, the brute-force enumeration and the int4 cases once more against a build
    of the oracle that traps on undefined behaviour (a crash of the child = a finding)."""
    import subprocess
    import sys
    from oracle import pf_oracle
    lib = pf_oracle.build_checked()
    env = dict(os.environ, PF_ORACLE_LIB=lib)
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                        os.path.join(root, "tests", "test_oracle_pins.py"), "-k",
                        "mask_identities or brute or int4 or half_to_double or stack_glue or lookahead"],
                       cwd=root, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert " passed" in r.stdout
