"""Helpers shared by the tests: oracle layers from workload tensors, acceptance checks."""
import numpy as np

from oracle import pf_oracle
from paper_2312_12456_amd import workload as wl

# Acceptance bar for fp16 weights with fp32 accumulation against the fp64 oracle.
MAX_ABS = 2e-2
MAX_REL = 1e-2
SCORE_BAND = 1e-3


def oracle_layer(cfg, host, threshold=None):
    """pf_oracle.Layer over the numpy tensors of workload.to_host(make_layer(...))."""
    return pf_oracle.Layer(
        cfg.d, cfg.ffn, cfg.r, act=cfg.act, wtype=cfg.wtype,
        threshold=cfg.threshold if threshold is None else threshold,
        w_up=host.get("w_up"), w_gate=host.get("w_gate"), w_down=host.get("w_down"),
        s_up=host.get("s_up"), s_gate=host.get("s_gate"), s_down=host.get("s_down"),
        b_up=host.get("b_up"), b_down=host.get("b_down"), p1=host.get("p1"), p2=host.get("p2"),
        p_bias=host.get("p_bias"))


def small_cfg(name="t", d=256, ffn=512, r=64, act=wl.ACT_RELU, wtype=wl.W_FP16, rate=0.1,
              alpha=1.2, layers=1):
    return wl.StackConfig(name, layers, d, ffn, r, act, wtype, rate, alpha, 8, (1,))


def check_output(y_dev, y_ref, what=""):
    """max-abs <= 2e-2 and max-abs / max|ref| <= 1e-2."""
    y_dev = np.asarray(y_dev, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    assert y_dev.shape == y_ref.shape, (y_dev.shape, y_ref.shape)
    assert np.isfinite(y_dev).all(), what
    err = float(np.max(np.abs(y_dev - y_ref))) if y_ref.size else 0.0
    scale = float(np.max(np.abs(y_ref))) if y_ref.size else 0.0
    assert err <= MAX_ABS, "%s max-abs %.3e" % (what, err)
    if scale > 0:
        assert err / scale <= MAX_REL, "%s rel %.3e" % (what, err / scale)
    return err


def check_active_set(dev_mask, ref_scores, threshold, what="", always_on=None):
    """Bit-exact union mask outside the 1e-3 score band around the threshold.  Neurons of an
    always-on set (listed without prediction) must be on and are otherwise not compared."""
    ref_scores = np.atleast_2d(ref_scores)
    ref_rows = ref_scores > threshold
    ref_mask = ref_rows.any(axis=0)
    # a neuron is comparable if no token's score sits in the band, or some token
    # outside the band already decides it active
    in_band = np.abs(ref_scores - threshold) < SCORE_BAND
    decided_on = (ref_rows & ~in_band).any(axis=0)
    comparable = decided_on | ~in_band.any(axis=0)
    if always_on is not None:
        always_on = np.asarray(always_on, bool)
        assert np.asarray(dev_mask, bool)[always_on].all(), "%s: an always-on neuron is off" % what
        comparable &= ~always_on
    bad = comparable & (np.asarray(dev_mask, bool) != ref_mask)
    assert not bad.any(), "%s: %d active-set mismatches outside the band, first %s" % (
        what, int(bad.sum()), np.flatnonzero(bad)[:8])
    return int((~comparable).sum())


def words_to_mask(words, ffn):
    """uint64 / int64 mask words (numpy) -> bool [ffn]; bit b of word w = neuron 64 w + b."""
    w = np.ascontiguousarray(np.asarray(words)).view(np.uint8)
    return np.unpackbits(w, bitorder="little")[:ffn].astype(bool)


class MaskTrace:
    """Device buffer the library fills with every layer's mask words during a stack step."""

    def __init__(self, ctx, n_layers, ffn):
        import torch
        self.n_layers, self.ffn, self.stride = n_layers, ffn, ctx.max_ffn // 64
        self.buf = torch.full((n_layers * self.stride,), -1, dtype=torch.int64, device="cuda")
        ctx.set_mask_trace(self.buf, n_layers)

    def masks(self):
        host = self.buf.cpu().numpy().reshape(self.n_layers, self.stride)
        return [words_to_mask(host[l, :self.ffn // 64], self.ffn) for l in range(self.n_layers)]


def oracle_chain_on_device_sets(oracle_mod, Os, x0, masks, threshold, what="", always_on=None):
    """The oracle's stack driven by the active sets the device used, layer by layer: the set of
    layer l must equal the oracle's prediction on the oracle's own input to that layer outside
    the score band; the oracle then runs its masked FFN on exactly that set, so a flip inside
    the band never leaks into the output comparison.  -> (oracle stack output, number of
    layers compared, number of (token, neuron) scores that lay inside the band)."""
    xo = np.asarray(x0, dtype=np.float32)
    in_band = 0
    for l, (O, m) in enumerate(zip(Os, masks)):
        sc = O.predict(xo)["scores"]
        in_band += check_active_set(m, sc, threshold, "%s layer %d" % (what, l),
                                    None if always_on is None else always_on[l])
        xo = oracle_mod.stack_glue(xo, O.masked_ffn(xo, m))
    return xo, len(masks), in_band


def oracle_lookahead_chain_on_device_sets(oracle_mod, Os, x0, masks, threshold, what=""):
    """The same for look-ahead prediction at distance 1: the set of layer l is checked against
    layer l's predictor applied to the oracle's input of layer l - 1 (layer 0: its own input)."""
    xo = np.asarray(x0, dtype=np.float32)
    inputs, in_band = [], 0
    for l, (O, m) in enumerate(zip(Os, masks)):
        inputs.append(xo)
        seen = inputs[0] if l == 0 else inputs[l - 1]
        in_band += check_active_set(m, O.predict(seen)["scores"], threshold, "%s layer %d" % (what, l))
        xo = oracle_mod.stack_glue(xo, O.masked_ffn(xo, m))
    return xo, len(masks), in_band
