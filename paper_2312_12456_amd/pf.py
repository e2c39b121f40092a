"""Thin ctypes binding of libpf.so (include/pf.h): argument marshalling only.

Every step of the path runs in the HIP kernels of the library; torch tensors are used as
device memory and their data pointers are handed over.  There is no CPU fallback: if the
library has not been built, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# PF_LIB_PATH selects another build of the same library (kernel tuning experiments)
LIB_PATH = os.environ.get("PF_LIB_PATH") or os.path.join(_HERE, "libpf.so")

PF_OK, PF_EINVAL, PF_ESHAPE, PF_ENOMEM, PF_EHIP, PF_EUNSUPPORTED, PF_ELIMIT = range(7)
ACT_RELU, ACT_REGLU, ACT_DRELU = 0, 1, 2
W_FP16, W_INT4_G128 = 0, 1

EXPORTS = [
    "pf_ctx_create", "pf_ctx_destroy", "pf_layer_create", "pf_layer_destroy", "pf_predict",
    "pf_compact", "pf_sparse_ffn", "pf_layer_step", "pf_ctx_last_active", "pf_stack_glue",
    "pf_stack_step", "pf_plan_create", "pf_plan_run", "pf_plan_destroy", "pf_strerror",
    "pf_last_error", "pf_version", "pf_profile_begin", "pf_profile_end", "pf_dense_ffn",
    "pf_layer_step_auto", "pf_count_activations", "pf_ctx_set_lookahead", "pf_ctx_set_option",
    "pf_ctx_get_option", "pf_ctx_set_mask_trace", "pf_layer_step_noalloc",
    "pf_layer_set_neuron_table", "pf_layer_active_original", "pf_layer_step_adaptive",
    "pf_layer_adaptive_state",
]

# pf_option keys
(OPT_FUSED, OPT_SEG_STRIDED, OPT_MFMA_MIN_BATCH, OPT_HIDDEN_MFMA_MIN_ELEMS, OPT_UP_GRID,
 OPT_MFMA_GRID, OPT_DOWN_SPLIT, OPT_LOOKAHEAD_FORM) = range(8)


class PfError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("libpf status %d: %s" % (status, text))
        self.status = status


class LayerDesc(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int32), ("ffn", ctypes.c_int32), ("r", ctypes.c_int32),
                ("act", ctypes.c_int32), ("wtype", ctypes.c_int32), ("threshold", ctypes.c_float)]


class LayerWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("w_up", "w_gate", "w_down", "s_up", "s_gate", "s_down", "b_up", "b_down", "p1",
                 "p2", "p_bias")]


class KernelStat(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char_p), ("launches", ctypes.c_uint64),
                ("total_ms", ctypes.c_double)]


_lib = None


def lib():
    """The loaded C-ABI library; raises if libpf.so has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise PfError(PF_EHIP, "%s is missing: run __graft_entry__.build() "
                          "(python paper_2312_12456_amd/build.py)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        P, I = ctypes.c_void_p, ctypes.c_int
        PP = ctypes.POINTER(ctypes.c_void_p)
        L.pf_ctx_create.argtypes = [PP, I, I, I, I, I]
        L.pf_ctx_destroy.argtypes = [P]
        L.pf_ctx_destroy.restype = None
        L.pf_layer_create.argtypes = [P, ctypes.POINTER(LayerDesc), ctypes.POINTER(LayerWeights), PP]
        L.pf_layer_destroy.argtypes = [P]
        L.pf_layer_destroy.restype = None
        L.pf_predict.argtypes = [P, P, P, I, P, P, P]
        L.pf_compact.argtypes = [P, P, I, P, P, P]
        L.pf_sparse_ffn.argtypes = [P, P, P, I, P, P, P, P]
        L.pf_layer_step.argtypes = [P, P, P, I, P, P]
        L.pf_ctx_last_active.argtypes = [P, PP, PP, PP]
        L.pf_dense_ffn.argtypes = [P, P, P, I, P, P]
        L.pf_layer_step_auto.argtypes = [P, P, P, I, ctypes.c_float, ctypes.c_float, P, P]
        L.pf_count_activations.argtypes = [P, P, P, P]
        L.pf_ctx_set_lookahead.argtypes = [P, I]
        L.pf_ctx_set_option.argtypes = [P, I, I]
        L.pf_ctx_get_option.argtypes = [P, I, ctypes.POINTER(I)]
        L.pf_ctx_set_mask_trace.argtypes = [P, P, I]
        L.pf_layer_step_adaptive.argtypes = [P, P, P, I, ctypes.c_float, P, P]
        L.pf_layer_adaptive_state.argtypes = [P, ctypes.POINTER(ctypes.c_int32), I]
        L.pf_layer_set_neuron_table.argtypes = [P, P, I]
        L.pf_layer_active_original.argtypes = [P, P, P, P, P, P]
        L.pf_layer_step_noalloc.argtypes = [ctypes.POINTER(LayerDesc), ctypes.POINTER(LayerWeights),
                                            P, I, P, P]
        L.pf_stack_glue.argtypes = [P, P, P, I, I, P, P]
        L.pf_stack_step.argtypes = [P, PP, I, P, I, P, P]
        L.pf_plan_create.argtypes = [P, PP, I, P, I, P, P, PP]
        L.pf_plan_run.argtypes = [P, P]
        L.pf_plan_destroy.argtypes = [P]
        L.pf_plan_destroy.restype = None
        L.pf_strerror.argtypes = [I]
        L.pf_strerror.restype = ctypes.c_char_p
        L.pf_last_error.argtypes = [P]
        L.pf_last_error.restype = ctypes.c_char_p
        L.pf_version.restype = ctypes.c_char_p
        L.pf_profile_begin.argtypes = [P]
        L.pf_profile_end.argtypes = [P, ctypes.POINTER(KernelStat), I, ctypes.POINTER(I)]
        _lib = L
    return _lib


def _dev_ptr(t, dtype=None, numel=None):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("expected a device tensor")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, t.dtype))
    if numel is not None and t.numel() < numel:
        raise ValueError("tensor has %d elements, %d needed" % (t.numel(), numel))
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


class Context:
    """pf_ctx: scratch for layers up to (max_d, max_ffn, max_r) and batches up to max_batch."""

    def __init__(self, max_d, max_ffn, max_r, max_batch=1, device=0):
        self._h = ctypes.c_void_p()
        st = lib().pf_ctx_create(ctypes.byref(self._h), device, max_d, max_ffn, max_r, max_batch)
        if st != PF_OK:
            raise PfError(st, lib().pf_strerror(st).decode())
        self.device = device
        self.max_ffn = max_ffn
        self._trace = None

    def check(self, st):
        if st != PF_OK:
            raise PfError(st, "%s: %s" % (lib().pf_strerror(st).decode(),
                                          lib().pf_last_error(self._h).decode()))

    def close(self):
        if self._h:
            lib().pf_ctx_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- entry points -------------------------------------------------------------
    def predict(self, layer, x, scores, mask_words, stream=None):
        B = x.shape[0]
        self.check(lib().pf_predict(self._h, layer._h, _dev_ptr(x, torch.float32, B * layer.d), B,
                                    _dev_ptr(scores, torch.float32, B * layer.ffn),
                                    _dev_ptr(mask_words, torch.int64, layer.ffn // 64),
                                    _stream_ptr(stream)))

    def compact(self, mask_words, ffn, idx, count, stream=None):
        self.check(lib().pf_compact(self._h, _dev_ptr(mask_words, torch.int64, ffn // 64), ffn,
                                    _dev_ptr(idx, torch.int32, ffn), _dev_ptr(count, torch.int32, 1),
                                    _stream_ptr(stream)))

    def sparse_ffn(self, layer, x, idx, count, y, stream=None):
        B = x.shape[0]
        self.check(lib().pf_sparse_ffn(self._h, layer._h, _dev_ptr(x, torch.float32, B * layer.d), B,
                                       _dev_ptr(idx, torch.int32, layer.ffn),
                                       _dev_ptr(count, torch.int32, 1),
                                       _dev_ptr(y, torch.float32, B * layer.d), _stream_ptr(stream)))

    def layer_step(self, layer, x, y, stream=None):
        B = x.shape[0]
        self.check(lib().pf_layer_step(self._h, layer._h, _dev_ptr(x, torch.float32, B * layer.d), B,
                                       _dev_ptr(y, torch.float32, B * layer.d), _stream_ptr(stream)))

    def dense_ffn(self, layer, x, y, stream=None):
        B = x.shape[0]
        self.check(lib().pf_dense_ffn(self._h, layer._h, _dev_ptr(x, torch.float32, B * layer.d), B,
                                      _dev_ptr(y, torch.float32, B * layer.d), _stream_ptr(stream)))

    def layer_step_auto(self, layer, x, y, density_hint, crossover, stream=None):
        B = x.shape[0]
        self.check(lib().pf_layer_step_auto(self._h, layer._h, _dev_ptr(x, torch.float32, B * layer.d),
                                            B, ctypes.c_float(density_hint), ctypes.c_float(crossover),
                                            _dev_ptr(y, torch.float32, B * layer.d), _stream_ptr(stream)))

    def layer_step_adaptive(self, layer, x, y, crossover, stream=None):
        B = x.shape[0]
        self.check(lib().pf_layer_step_adaptive(self._h, layer._h, _dev_ptr(x, torch.float32, B * layer.d),
                                                B, ctypes.c_float(crossover),
                                                _dev_ptr(y, torch.float32, B * layer.d), _stream_ptr(stream)))

    def count_activations(self, layer, counts, stream=None):
        """counts [ffn] int32 on the device (non-negative values, read as uint32 by the library)."""
        self.check(lib().pf_count_activations(self._h, layer._h, _dev_ptr(counts, torch.int32, layer.ffn),
                                              _stream_ptr(stream)))

    def set_lookahead(self, distance):
        self.check(lib().pf_ctx_set_lookahead(self._h, int(distance)))

    def set_option(self, key, value):
        self.check(lib().pf_ctx_set_option(self._h, int(key), int(value)))

    def get_option(self, key):
        v = ctypes.c_int(0)
        self.check(lib().pf_ctx_get_option(self._h, int(key), ctypes.byref(v)))
        return v.value

    def set_mask_trace(self, trace, n_layers=0):
        """trace: int64 device tensor of n_layers * (max_ffn / 64) words, or None to switch off."""
        if trace is None:
            self.check(lib().pf_ctx_set_mask_trace(self._h, None, 0))
        else:
            self.check(lib().pf_ctx_set_mask_trace(
                self._h, _dev_ptr(trace, torch.int64, n_layers * (self.max_ffn // 64)), n_layers))
        self._trace = trace  # keeps the buffer alive while the library may write to it

    def active_original(self, layer, mask_words, idx, count, stream=None):
        """Last active set in the model's neuron numbering (through the layer's neuron table)."""
        self.check(lib().pf_layer_active_original(
            self._h, layer._h, _dev_ptr(mask_words, torch.int64, layer.ffn // 64),
            _dev_ptr(idx, torch.int32, layer.ffn), _dev_ptr(count, torch.int32, 1), _stream_ptr(stream)))

    def last_active(self):
        """(mask_words, idx, count) device addresses left by the last layer_step."""
        m, i, c = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
        self.check(lib().pf_ctx_last_active(self._h, ctypes.byref(m), ctypes.byref(i), ctypes.byref(c)))
        return m.value, i.value, c.value

    def stack_glue(self, x, y, x_next, stream=None):
        B, d = x.shape
        self.check(lib().pf_stack_glue(self._h, _dev_ptr(x, torch.float32), _dev_ptr(y, torch.float32, B * d),
                                       d, B, _dev_ptr(x_next, torch.float32, B * d), _stream_ptr(stream)))

    def profile_begin(self):
        self.check(lib().pf_profile_begin(self._h))

    def profile_end(self):
        """-> {kernel name: (launches, total_ms)} measured with HIP events per launch."""
        stats = (KernelStat * 16)()
        n = ctypes.c_int(0)
        self.check(lib().pf_profile_end(self._h, stats, 16, ctypes.byref(n)))
        return {stats[k].name.decode(): (int(stats[k].launches), float(stats[k].total_ms))
                for k in range(n.value)}

    def stack_step(self, layers, x, x_out, stream=None):
        B = x.shape[0]
        arr = (ctypes.c_void_p * len(layers))(*[l._h for l in layers])
        self.check(lib().pf_stack_step(self._h, arr, len(layers), _dev_ptr(x, torch.float32), B,
                                       _dev_ptr(x_out, torch.float32, x.numel()), _stream_ptr(stream)))


class Layer:
    """pf_layer over borrowed device tensors (kept referenced here so they stay alive)."""

    def __init__(self, ctx, d, ffn, r, act=ACT_RELU, wtype=W_FP16, threshold=0.5, w_up=None,
                 w_gate=None, w_down=None, s_up=None, s_gate=None, s_down=None, b_up=None,
                 b_down=None, p1=None, p2=None, p_bias=None):
        self.ctx, self.d, self.ffn, self.r, self.act, self.wtype = ctx, d, ffn, r, act, wtype
        self._keep = (w_up, w_gate, w_down, s_up, s_gate, s_down, b_up, b_down, p1, p2, p_bias)
        wdt = torch.float16 if wtype == W_FP16 else torch.uint8
        wn = ffn * d if wtype == W_FP16 else ffn * d // 2
        desc = LayerDesc(d, ffn, r, act, wtype, threshold)
        w = LayerWeights(
            _dev_ptr(w_up, wdt, wn), _dev_ptr(w_gate, wdt, wn), _dev_ptr(w_down, wdt, wn),
            _dev_ptr(s_up, torch.float16), _dev_ptr(s_gate, torch.float16),
            _dev_ptr(s_down, torch.float16), _dev_ptr(b_up, torch.float32, ffn),
            _dev_ptr(b_down, torch.float32, d), _dev_ptr(p1, torch.float16, r * d),
            _dev_ptr(p2, torch.float16, ffn * r), _dev_ptr(p_bias, torch.float32, ffn))
        self._h = ctypes.c_void_p()
        ctx.check(lib().pf_layer_create(ctx._h, ctypes.byref(desc), ctypes.byref(w),
                                        ctypes.byref(self._h)))

    @classmethod
    def from_workload(cls, ctx, cfg, tensors):
        """Layer over the tensors of workload.make_layer(cfg, ..., device='cuda')."""
        g = tensors.get
        return cls(ctx, cfg.d, cfg.ffn, cfg.r, act=cfg.act, wtype=cfg.wtype, threshold=cfg.threshold,
                   w_up=g("w_up"), w_gate=g("w_gate"), w_down=g("w_down"), s_up=g("s_up"),
                   s_gate=g("s_gate"), s_down=g("s_down"), b_up=g("b_up"), b_down=g("b_down"),
                   p1=g("p1"), p2=g("p2"), p_bias=g("p_bias"))

    def adaptive_state(self, reset=False):
        """(dense next step?, neurons seen at the last adaptive step, last step dense?); syncs."""
        st = (ctypes.c_int32 * 3)()
        self.ctx.check(lib().pf_layer_adaptive_state(self._h, st, 1 if reset else 0))
        return bool(st[0]), int(st[1]), bool(st[2])

    def set_neuron_table(self, stored_to_original, always_on=0):
        """stored_to_original: int32 device tensor [ffn] (a permutation) or None; always_on: length
        of the stored prefix that is listed without being predicted (a multiple of 64)."""
        self.ctx.check(lib().pf_layer_set_neuron_table(
            self._h, _dev_ptr(stored_to_original, torch.int32, self.ffn), int(always_on)))
        self._table = stored_to_original  # borrowed by the library: keep it alive

    def close(self):
        if self._h:
            lib().pf_layer_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Plan:
    """pf_plan: one decode step of a stack recorded into a HIP graph."""

    def __init__(self, ctx, layers, x, x_out, stream=None):
        self.ctx, self._keep = ctx, (layers, x, x_out)
        B = x.shape[0]
        arr = (ctypes.c_void_p * len(layers))(*[l._h for l in layers])
        self._h = ctypes.c_void_p()
        ctx.check(lib().pf_plan_create(ctx._h, arr, len(layers), _dev_ptr(x, torch.float32), B,
                                       _dev_ptr(x_out, torch.float32, x.numel()),
                                       _stream_ptr(stream), ctypes.byref(self._h)))

    def run(self, stream=None):
        self.ctx.check(lib().pf_plan_run(self._h, _stream_ptr(stream)))

    def close(self):
        if self._h:
            lib().pf_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def layer_step_noalloc(cfg, tensors, x, y, stream=None):
    """pf_layer_step_noalloc on the current device: the layer step of the tensors of
    workload.make_layer(cfg, ...) with the library's fixed scratch array, no context."""
    g = tensors.get
    wdt = torch.float16 if cfg.wtype == W_FP16 else torch.uint8
    wn = cfg.ffn * cfg.d if cfg.wtype == W_FP16 else cfg.ffn * cfg.d // 2
    desc = LayerDesc(cfg.d, cfg.ffn, cfg.r, cfg.act, cfg.wtype, cfg.threshold)
    w = LayerWeights(
        _dev_ptr(g("w_up"), wdt, wn), _dev_ptr(g("w_gate"), wdt, wn), _dev_ptr(g("w_down"), wdt, wn),
        _dev_ptr(g("s_up"), torch.float16), _dev_ptr(g("s_gate"), torch.float16),
        _dev_ptr(g("s_down"), torch.float16), _dev_ptr(g("b_up"), torch.float32, cfg.ffn),
        _dev_ptr(g("b_down"), torch.float32, cfg.d), _dev_ptr(g("p1"), torch.float16, cfg.r * cfg.d),
        _dev_ptr(g("p2"), torch.float16, cfg.ffn * cfg.r), _dev_ptr(g("p_bias"), torch.float32, cfg.ffn))
    B = x.shape[0]
    st = lib().pf_layer_step_noalloc(ctypes.byref(desc), ctypes.byref(w),
                                     _dev_ptr(x, torch.float32, B * cfg.d), B,
                                     _dev_ptr(y, torch.float32, B * cfg.d), _stream_ptr(stream))
    if st != PF_OK:
        raise PfError(st, lib().pf_strerror(st).decode())


_hip = None


def copy_from_device_address(dst, address, stream=None):
    """Device-to-device copy of dst.numel() elements from a raw device address into dst."""
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    torch.cuda.synchronize()
    err = _hip.hipMemcpy(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(address),
                         dst.numel() * dst.element_size(), 3)  # hipMemcpyDeviceToDevice
    if err != 0:
        raise PfError(PF_EHIP, "hipMemcpy failed with %d" % err)


def version():
    return lib().pf_version().decode()
