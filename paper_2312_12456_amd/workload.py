"""Seeded synthetic workloads: FFN-stack shapes, weights, biases and decode inputs.

This module holds none of the method's arithmetic (no predictor, no FFN, no
compaction): it only draws the random tensors that both the HIP library and the CPU
oracle are fed, so that the two can be compared on identical bytes.

The inputs stand in for what the paper measures on (real OPT / ReLU-gated LLaMA
checkpoints driven by chat prompts, Sec. 8.1), which need datasets and weights that
are not available offline.  They keep what matters to the sparse operators: the FFN
shapes of those models, fp16 / int4 weights, and the power-law ("hot"/"cold") skew of
neuron activation frequencies the paper reports (Sec. 3.1, Insight-1).

Recipe
  * Neuron i gets a target activation probability p_i = min(p_max, c * rank_i^-alpha),
    rank_i drawn from a seeded permutation, c found by bisection so mean(p_i) equals
    the configured rate.
  * FC1 / gate / FC2^T rows ~ N(0, 1/d) rounded to fp16, x ~ N(0, I_d).  Then a
    pre-activation without bias is ~ N(0, 1) and the FC1 (or gate) bias
    b_i = Phi^-1(p_i) makes P(neuron i fires) ~= p_i.
  * Predictor weights P1 ~ N(0, 1/d), P2 ~ N(0, 1/r).  With a ReLU hidden layer the
    logits are ~ N(0, 1/2); the optional logit bias sqrt(1/2) * Phi^-1(p_i) gives the
    predicted set the same per-neuron rates (which cold neurons are marked is then
    unrelated to the ones that fire; byte counts and oracle parity do not care).
  * int4: symmetric group-128 quantisation of the same Gaussian rows.
"""
import hashlib
import math
from dataclasses import dataclass, replace

import numpy as np
import torch
from scipy.special import ndtri

ACT_RELU = 0
ACT_REGLU = 1
ACT_DRELU = 2
W_FP16 = 0
W_INT4_G128 = 1

P_MAX = 0.995


@dataclass(frozen=True)
class StackConfig:
    name: str
    layers: int
    d: int
    ffn: int
    r: int
    act: int
    wtype: int
    rate: float        # mean per-token activation probability
    alpha: float       # Zipf exponent of the per-neuron probabilities
    tokens: int        # decode steps of the benchmark run
    batches: tuple     # batch sizes the configuration is quoted at
    threshold: float = 0.5

    @property
    def n_matrices(self):
        return 2 if self.act == ACT_RELU else 3

    @property
    def row_bytes(self):
        return 2 * self.d if self.wtype == W_FP16 else self.d // 2 + (self.d // 128) * 2

    def predictor_bytes(self):
        return 2 * self.r * (self.d + self.ffn)

    def touched_bytes(self, k):
        return k * self.n_matrices * self.row_bytes


CONFIGS = {
    "opt-125m-layer": StackConfig("opt-125m-layer", 1, 768, 3072, 128, ACT_RELU, W_FP16,
                                  0.10, 1.2, 64, (1,)),
    "opt-6.7b": StackConfig("opt-6.7b", 32, 4096, 16384, 1024, ACT_RELU, W_FP16,
                            0.08, 1.2, 256, (1,)),
    "llama2-13b-reglu": StackConfig("llama2-13b-reglu", 40, 5120, 13824, 1024, ACT_REGLU,
                                    W_FP16, 0.15, 1.0, 256, (1, 4)),
    "opt-30b": StackConfig("opt-30b", 48, 7168, 28672, 1536, ACT_RELU, W_FP16,
                           0.06, 1.3, 256, (1, 4, 8)),
    "opt-175b-int4": StackConfig("opt-175b-int4", 96, 12288, 49152, 2048, ACT_RELU,
                                 W_INT4_G128, 0.04, 1.3, 256, (1,)),
    # the dReLU model of the paper's list (Bamboo-7B: a Mistral-7B-shaped gated FFN with ReLU
    # on both branches, 90 % sparsity in the model table)
    "bamboo-7b-drelu": StackConfig("bamboo-7b-drelu", 32, 4096, 14336, 1024, ACT_DRELU, W_FP16,
                                   0.10, 1.2, 256, (1,)),
    # a second OPT-like shape beside the benchmark configurations: the ReLU Falcon-40B FFN
    # (95 % sparsity in the paper's model table), 60 layers
    "falcon-40b-relu": StackConfig("falcon-40b-relu", 60, 8192, 32768, 1024, ACT_RELU, W_FP16,
                                   0.05, 1.2, 256, (1,)),
}


def scaled(cfg, **kw):
    """A copy of cfg with some fields replaced (reduced shapes for quick tests)."""
    return replace(cfg, **kw)


def _seed64(master, *names):
    h = hashlib.blake2b(("%d/" % master + "/".join(str(n) for n in names)).encode(),
                        digest_size=8).digest()
    return int.from_bytes(h, "little") & ((1 << 63) - 1)


def _generator(device, master, *names):
    g = torch.Generator(device=device)
    g.manual_seed(_seed64(master, *names))
    return g


def zipf_probabilities(ffn, alpha, mean_rate, seed):
    """Per-neuron activation probabilities: clipped power law over a random ranking."""
    rng = np.random.Generator(np.random.PCG64(_seed64(seed, "zipf-perm")))
    rank = rng.permutation(ffn).astype(np.float64) + 1.0
    base = rank ** (-alpha)
    lo, hi = 0.0, 1.0
    while np.minimum(P_MAX, hi * base).mean() < mean_rate:
        hi *= 2.0
        if hi > 1e12:
            break
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if np.minimum(P_MAX, mid * base).mean() < mean_rate:
            lo = mid
        else:
            hi = mid
    return np.minimum(P_MAX, hi * base)


def expected_union_rate(p, batch):
    """Expected fraction of neurons fired by at least one of `batch` independent tokens."""
    return float(np.mean(1.0 - (1.0 - p) ** batch))


def _normal_fp16(shape, std, device, g, chunk_rows=4096):
    out = torch.empty(shape, dtype=torch.float16, device=device)
    rows = shape[0]
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        blk = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=g, device=device,
                          dtype=torch.float32)
        out[r0:r1] = (blk * std).to(torch.float16)
    return out


def quantize_int4_g128(w):
    """fp32 [F][d] -> (packed uint8 [F][d/2], fp16 scales [F][d/128]).

    Symmetric, no zero point: scale = fp16(absmax / 7) per 128 consecutive elements of
    a row, code u = clamp(round(w / scale), -7, 7) + 8, element 2j in the low nibble
    and 2j+1 in the high nibble of byte j.
    """
    F, d = w.shape
    assert d % 128 == 0
    g = w.reshape(F, d // 128, 128).to(torch.float32)
    s = (g.abs().amax(dim=2) / 7.0).to(torch.float16)
    sf = s.to(torch.float32).clamp_min(1e-8).unsqueeze(2)
    u = (torch.round(g / sf).clamp_(-7, 7) + 8).to(torch.uint8).reshape(F, d // 2, 2)
    q = (u[:, :, 0] | (u[:, :, 1] << 4)).contiguous()
    return q, s.contiguous()


def _weight_matrix(cfg, device, g, chunk_rows=2048):
    """One [ffn][d] neuron-major matrix ~ N(0, 1/d): fp16, or (int4 bytes, scales)."""
    std = 1.0 / math.sqrt(cfg.d)
    if cfg.wtype == W_FP16:
        return _normal_fp16((cfg.ffn, cfg.d), std, device, g), None
    q = torch.empty((cfg.ffn, cfg.d // 2), dtype=torch.uint8, device=device)
    s = torch.empty((cfg.ffn, cfg.d // 128), dtype=torch.float16, device=device)
    for r0 in range(0, cfg.ffn, chunk_rows):
        r1 = min(cfg.ffn, r0 + chunk_rows)
        blk = torch.randn((r1 - r0, cfg.d), generator=g, device=device,
                          dtype=torch.float32) * std
        q[r0:r1], s[r0:r1] = quantize_int4_g128(blk)
    return q, s


def make_layer(cfg, layer, seed, device="cpu", pred_bias=True):
    """Tensors of one FFN layer and its predictor, on `device`.

    Keys: w_up, w_gate (gated only), w_down ([ffn][d], FC2 transposed), s_* (int4
    only), b_up ([ffn] fp32: FC1 bias, or the gate bias when gated), b_down ([d] fp32
    or None), p1 [r][d], p2 [ffn][r] fp16, p_bias ([ffn] fp32 or None), p (float64
    numpy, the target probabilities).
    """
    device = torch.device(device)
    p = zipf_probabilities(cfg.ffn, cfg.alpha, cfg.rate, _seed64(seed, "layer", layer))
    out = {"p": p}
    names = ["w_up", "w_down"] + (["w_gate"] if cfg.act != ACT_RELU else [])
    for nm in names:
        w, s = _weight_matrix(cfg, device, _generator(device, seed, "layer", layer, nm))
        out[nm] = w
        if s is not None:
            out["s_" + nm[2:]] = s
    quant = ndtri(p)
    # dReLU: a neuron fires when the gate AND the (bias-free, sign-symmetric) up branch are
    # positive, so the gate is opened twice as often to keep the firing rate at p_i
    gate_quant = ndtri(np.minimum(P_MAX, 2.0 * p)) if cfg.act == ACT_DRELU else quant
    out["b_up"] = torch.from_numpy(gate_quant.astype(np.float32)).to(device)
    if cfg.act == ACT_RELU:
        g = _generator("cpu", seed, "layer", layer, "b_down")
        out["b_down"] = (torch.randn(cfg.d, generator=g, dtype=torch.float32) * 0.1).to(device)
    else:
        out["b_down"] = None
    out["p1"] = _normal_fp16((cfg.r, cfg.d), 1.0 / math.sqrt(cfg.d), device,
                             _generator(device, seed, "layer", layer, "p1"))
    out["p2"] = _normal_fp16((cfg.ffn, cfg.r), 1.0 / math.sqrt(cfg.r), device,
                             _generator(device, seed, "layer", layer, "p2"))
    if pred_bias:
        out["p_bias"] = torch.from_numpy((math.sqrt(0.5) * quant).astype(np.float32)).to(device)
    else:
        out["p_bias"] = None
    return out


NEURON_AXIS_KEYS = ("w_up", "w_gate", "w_down", "s_up", "s_gate", "s_down", "b_up", "p2", "p_bias")


def permute_neurons(layer, order):
    """The same layer with its neurons renumbered: new neuron j is old neuron order[j].

    Every tensor with a neuron axis (rows of the three FFN matrices and their scales, FC1
    bias, rows of the predictor's output layer and its bias, the target probabilities) is
    reordered alike, so the FFN computes the same function and the predictor marks the same
    neurons under their new numbers.  Used to lay neurons out hot-first from profiled counts
    (the frequency-sorted layout a neuron table makes possible)."""
    out = dict(layer)
    for k in NEURON_AXIS_KEYS:
        v = layer.get(k)
        if v is None:
            continue
        if isinstance(v, torch.Tensor):
            idx = torch.as_tensor(np.asarray(order), dtype=torch.long, device=v.device)
            out[k] = v.index_select(0, idx).contiguous()
        else:
            out[k] = np.ascontiguousarray(np.asarray(v)[np.asarray(order)])
    if layer.get("p") is not None:
        out["p"] = np.asarray(layer["p"])[np.asarray(order)]
    return out


def make_inputs(cfg, token, seed, batch=1, device="cpu"):
    """Hidden states entering the stack at decode step `token`: [batch][d] ~ N(0, I)."""
    g = _generator("cpu", seed, "token", token, "batch", batch)
    x = torch.randn((batch, cfg.d), generator=g, dtype=torch.float32)
    return x.to(device)


def to_host(layer):
    """Copy a layer's tensors to numpy (fp16 stays fp16) for the CPU side of a test."""
    out = {}
    for k, v in layer.items():
        out[k] = v.detach().cpu().numpy() if isinstance(v, torch.Tensor) else v
    return out
