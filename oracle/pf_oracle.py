"""ctypes front-end of the plain CPU oracle (pf_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module and
this module never imports the product package.

Arrays go in and out as numpy: fp16 weights as float16 (or their uint16 bits), int4
weights as packed uint8 with float16 scales, activations float32, results float64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pf_oracle.c")
_LIB = os.path.join(_HERE, "libpf_oracle.so")

ACT_RELU = 0
ACT_REGLU = 1
ACT_DRELU = 2
W_FP16 = 0
W_INT4_G128 = 1


def build_checked():
    """A second build with the undefined-behaviour sanitizer trapping on the first finding
    (signed overflow, misaligned or out-of-bounds access the compiler can see, bad shifts):
    oracle/libpf_oracle_ubsan.so.  PF_ORACLE_LIB selects it for a test run."""
    out = os.path.join(_HERE, "libpf_oracle_ubsan.so")
    tmp = out + ".tmp.%d" % os.getpid()
    subprocess.check_call(
        ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
         "-fsanitize=undefined", "-fsanitize-undefined-trap-on-error", "-fno-sanitize-recover=all",
         "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, out)
    return out


def build(force=False):
    """Compile pf_oracle.c with gcc into oracle/libpf_oracle.so."""
    override = os.environ.get("PF_ORACLE_LIB")
    if override:
        return override
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _CLayer(ctypes.Structure):
    _fields_ = [
        ("d", ctypes.c_int32), ("ffn", ctypes.c_int32), ("r", ctypes.c_int32),
        ("act", ctypes.c_int32), ("wtype", ctypes.c_int32), ("pad_", ctypes.c_int32),
        ("threshold", ctypes.c_double),
        ("w_up", ctypes.c_void_p), ("w_gate", ctypes.c_void_p), ("w_down", ctypes.c_void_p),
        ("s_up", ctypes.c_void_p), ("s_gate", ctypes.c_void_p), ("s_down", ctypes.c_void_p),
        ("b_up", ctypes.c_void_p), ("b_down", ctypes.c_void_p),
        ("p1", ctypes.c_void_p), ("p2", ctypes.c_void_p), ("p_bias", ctypes.c_void_p),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        P = ctypes.c_void_p
        LP = ctypes.POINTER(_CLayer)
        I = ctypes.c_int
        L.pfo_half_to_double.restype = ctypes.c_double
        L.pfo_half_to_double.argtypes = [ctypes.c_uint16]
        L.pfo_num_threads.restype = I
        L.pfo_weight_value.restype = ctypes.c_double
        L.pfo_weight_value.argtypes = [LP, I, I, I]
        L.pfo_preact.argtypes = [LP, P, I, P]
        L.pfo_dense_ffn.argtypes = [LP, P, I, P]
        L.pfo_masked_ffn.argtypes = [LP, P, I, P, P]
        L.pfo_compact.restype = I
        L.pfo_compact.argtypes = [P, I, P]
        L.pfo_sparse_ffn_idx.argtypes = [LP, P, I, P, I, P, P]
        L.pfo_predict.argtypes = [LP, P, I, P, P, P, P, P]
        L.pfo_exact_mask.argtypes = [LP, P, I, P]
        L.pfo_layer_step.argtypes = [LP, P, I, P, P]
        L.pfo_stack_glue.argtypes = [P, P, I, I, P]
        for f in (L.pfo_preact, L.pfo_dense_ffn, L.pfo_masked_ffn, L.pfo_sparse_ffn_idx,
                  L.pfo_predict, L.pfo_exact_mask, L.pfo_layer_step, L.pfo_stack_glue):
            f.restype = None
        _lib = L
    return _lib


def num_threads():
    return int(lib().pfo_num_threads())


def _ptr(a):
    return None if a is None else a.ctypes.data


def _bits16(a, shape):
    """float16 (or uint16 bit pattern) array -> contiguous uint16 view of `shape`."""
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    a = np.ascontiguousarray(a)
    assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _f32(a, shape):
    a = np.ascontiguousarray(np.asarray(a), dtype=np.float32)
    assert a.shape == tuple(shape), (a.shape, shape)
    return a


class Layer:
    """One FFN layer with its predictor, held as host arrays for the oracle.

    act: ACT_RELU (w_up, b_up, w_down, b_down), ACT_REGLU or ACT_DRELU (w_gate, b_up = gate
    bias, w_up, w_down).  w_down is FC2 transposed: [ffn][d].  For W_INT4_G128 the w_* are
    uint8 [ffn][d/2] and s_* float16 [ffn][d/128].
    """

    def __init__(self, d, ffn, r, act=ACT_RELU, wtype=W_FP16, threshold=0.5, w_up=None,
                 w_gate=None, w_down=None, s_up=None, s_gate=None, s_down=None, b_up=None,
                 b_down=None, p1=None, p2=None, p_bias=None):
        self.d, self.ffn, self.r = int(d), int(ffn), int(r)
        self.act, self.wtype, self.threshold = int(act), int(wtype), float(threshold)
        keep = {}

        def wmat(a):
            if a is None:
                return None
            if wtype == W_FP16:
                return _bits16(a, (ffn, d))
            a = np.ascontiguousarray(np.asarray(a), dtype=np.uint8)
            assert d % 128 == 0 and a.shape == (ffn, d // 2), a.shape
            return a

        def smat(a):
            if a is None or wtype == W_FP16:
                return None
            return _bits16(a, (ffn, d // 128))

        keep["w_up"], keep["w_gate"], keep["w_down"] = wmat(w_up), wmat(w_gate), wmat(w_down)
        keep["s_up"], keep["s_gate"], keep["s_down"] = smat(s_up), smat(s_gate), smat(s_down)
        keep["b_up"] = None if b_up is None else _f32(b_up, (ffn,))
        keep["b_down"] = None if b_down is None else _f32(b_down, (d,))
        keep["p1"] = None if p1 is None else _bits16(p1, (r, d))
        keep["p2"] = None if p2 is None else _bits16(p2, (ffn, r))
        keep["p_bias"] = None if p_bias is None else _f32(p_bias, (ffn,))
        if act != ACT_RELU and w_up is not None:
            assert keep["w_gate"] is not None
        if wtype == W_INT4_G128:
            for k in ("up", "gate", "down"):
                assert (keep["w_" + k] is None) == (keep["s_" + k] is None)
        self._keep = keep
        self.c = _CLayer(self.d, self.ffn, self.r, self.act, self.wtype, 0, self.threshold,
                         *[_ptr(keep[k]) for k in ("w_up", "w_gate", "w_down", "s_up", "s_gate",
                                                   "s_down", "b_up", "b_down", "p1", "p2",
                                                   "p_bias")])

    def _x(self, x):
        x = np.ascontiguousarray(np.asarray(x), dtype=np.float32)
        if x.ndim == 1:
            x = x[None, :]
        assert x.ndim == 2 and x.shape[1] == self.d, x.shape
        return x

    # --- plain definitions -------------------------------------------------------
    def preact(self, x):
        x = self._x(x)
        out = np.empty((x.shape[0], self.ffn), np.float64)
        lib().pfo_preact(ctypes.byref(self.c), _ptr(x), x.shape[0], _ptr(out))
        return out

    def dense_ffn(self, x):
        x = self._x(x)
        y = np.empty((x.shape[0], self.d), np.float64)
        lib().pfo_dense_ffn(ctypes.byref(self.c), _ptr(x), x.shape[0], _ptr(y))
        return y

    def masked_ffn(self, x, mask):
        x = self._x(x)
        mask = np.ascontiguousarray(np.asarray(mask) != 0).astype(np.uint8)
        assert mask.shape == (self.ffn,)
        y = np.empty((x.shape[0], self.d), np.float64)
        lib().pfo_masked_ffn(ctypes.byref(self.c), _ptr(x), x.shape[0], _ptr(mask), _ptr(y))
        return y

    def sparse_ffn_idx(self, x, idx, return_h=False):
        x = self._x(x)
        idx = np.ascontiguousarray(np.asarray(idx), dtype=np.int32)
        assert idx.ndim == 1
        if idx.size:
            assert idx.min() >= 0 and idx.max() < self.ffn
        y = np.empty((x.shape[0], self.d), np.float64)
        h = np.empty((x.shape[0], idx.size), np.float64)
        lib().pfo_sparse_ffn_idx(ctypes.byref(self.c), _ptr(x), x.shape[0], _ptr(idx),
                                 int(idx.size), _ptr(y), _ptr(h) if idx.size else None)
        return (y, h) if return_h else y

    def predict(self, x):
        """-> dict(hidden [B][r], logits, scores [B][F], active [F] bool, active_rows)."""
        x = self._x(x)
        B = x.shape[0]
        hidden = np.empty((B, self.r), np.float64)
        logits = np.empty((B, self.ffn), np.float64)
        scores = np.empty((B, self.ffn), np.float64)
        active = np.empty((self.ffn,), np.uint8)
        rows = np.empty((B, self.ffn), np.uint8)
        lib().pfo_predict(ctypes.byref(self.c), _ptr(x), B, _ptr(hidden), _ptr(logits),
                          _ptr(scores), _ptr(active), _ptr(rows))
        return dict(hidden=hidden, logits=logits, scores=scores, active=active.astype(bool),
                    active_rows=rows.astype(bool))

    def exact_mask(self, x):
        x = self._x(x)
        mask = np.empty((self.ffn,), np.uint8)
        lib().pfo_exact_mask(ctypes.byref(self.c), _ptr(x), x.shape[0], _ptr(mask))
        return mask.astype(bool)

    def layer_step(self, x, return_mask=False):
        x = self._x(x)
        y = np.empty((x.shape[0], self.d), np.float64)
        mask = np.empty((self.ffn,), np.uint8)
        lib().pfo_layer_step(ctypes.byref(self.c), _ptr(x), x.shape[0], _ptr(y), _ptr(mask))
        return (y, mask.astype(bool)) if return_mask else y

    def weight_value(self, which, i, c):
        return float(lib().pfo_weight_value(ctypes.byref(self.c), {"up": 0, "gate": 1,
                                                                   "down": 2}[which], i, c))


def compact(mask):
    mask = np.ascontiguousarray(np.asarray(mask) != 0).astype(np.uint8)
    idx = np.empty((mask.size,), np.int32)
    n = lib().pfo_compact(_ptr(mask), int(mask.size), _ptr(idx))
    return idx[:n].copy()


def stack_glue(x, y):
    x = np.ascontiguousarray(np.asarray(x), dtype=np.float32)
    if x.ndim == 1:
        x = x[None, :]
    y = np.ascontiguousarray(np.asarray(y), dtype=np.float64).reshape(x.shape)
    out = np.empty_like(x)
    lib().pfo_stack_glue(_ptr(x), _ptr(y), x.shape[1], x.shape[0], _ptr(out))
    return out


def stack_lookahead(layers, x0):
    """A stack of layers with look-ahead prediction at distance 1 (PowerInfer Sec. 2.1: the
    activations of a layer can be predicted from an earlier layer's input): the active set of
    layer l >= 1 is layer l's predictor applied to the input of layer l - 1; layer 0 uses its
    own input.  Between layers the stack glue.  -> (output of the stack [B][d] fp32,
    list of the masks used)."""
    x = np.ascontiguousarray(np.asarray(x0), dtype=np.float32)
    if x.ndim == 1:
        x = x[None, :]
    inputs, masks = [], []
    for l, layer in enumerate(layers):
        inputs.append(x)
        seen = inputs[0] if l == 0 else inputs[l - 1]
        mask = layer.predict(seen)["active"]
        masks.append(mask)
        y = layer.masked_ffn(x, mask)
        x = stack_glue(x, y)
    return x, masks


def half_to_double(bits):
    return float(lib().pfo_half_to_double(int(bits)))
