"""The C-ABI library loads on a machine without a GPU and exports what include/pf.h declares;
argument errors are reported without touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pflib():
    from paper_2312_12456_amd import pf
    if not os.path.exists(pf.LIB_PATH):
        from paper_2312_12456_amd import build
        build.build()
    return pf.lib()


def test_header_symbols_are_exported(pflib):
    from paper_2312_12456_amd import pf
    text = open(os.path.join(ROOT, "include", "pf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(pf_[a-z_]+)\s*\(", text))
    assert declared == set(pf.EXPORTS)
    for name in declared:
        assert hasattr(pflib, name), name


def test_probe_library_exports_its_header():
    """libpf_probe.so (latency-floor probes of the measurement harness) loads without a GPU and
    exports what include/pf_probe.h declares."""
    from paper_2312_12456_amd import build
    if not os.path.exists(build.PROBE_LIB):
        build.build_probe()
    lib = ctypes.CDLL(build.PROBE_LIB)
    text = open(os.path.join(ROOT, "include", "pf_probe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(pfp_[a-z_]+)\s*\(", text))
    assert declared == {"pfp_measure", "pfp_last_error"}
    for name in declared:
        assert hasattr(lib, name), name
    lib.pfp_measure.argtypes = [ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.pfp_measure(0, 0, 256, 1, 1, None, None, None) == 1   # null outputs: refused


def test_strerror_and_version(pflib):
    from paper_2312_12456_amd import pf
    assert pflib.pf_strerror(pf.PF_OK) == b"ok"
    seen = {pflib.pf_strerror(s) for s in range(7)}
    assert len(seen) == 7
    assert b"gfx950" in pflib.pf_version()


def test_ctx_create_rejects_bad_arguments_on_host(pflib):
    from paper_2312_12456_amd import pf
    h = ctypes.c_void_p()
    assert pflib.pf_ctx_create(None, 0, 64, 64, 8, 1) == pf.PF_EINVAL
    assert pflib.pf_ctx_create(ctypes.byref(h), 0, 0, 64, 8, 1) == pf.PF_EINVAL
    assert pflib.pf_ctx_create(ctypes.byref(h), 0, 64, 64, 8, 9) == pf.PF_EINVAL
    assert pflib.pf_ctx_create(ctypes.byref(h), -1, 64, 64, 8, 1) == pf.PF_EINVAL
    assert pflib.pf_ctx_create(ctypes.byref(h), 0, 64, 100, 8, 1) == pf.PF_ESHAPE
    assert pflib.pf_ctx_create(ctypes.byref(h), 0, 60, 64, 8, 1) == pf.PF_ESHAPE
    assert h.value is None


def test_null_context_is_an_error_everywhere(pflib):
    from paper_2312_12456_amd import pf
    h = ctypes.c_void_p()
    assert pflib.pf_layer_create(None, None, None, ctypes.byref(h)) == pf.PF_EINVAL
    assert pflib.pf_predict(None, None, None, 1, None, None, None) == pf.PF_EINVAL
    assert pflib.pf_compact(None, None, 64, None, None, None) == pf.PF_EINVAL
    assert pflib.pf_sparse_ffn(None, None, None, 1, None, None, None, None) == pf.PF_EINVAL
    assert pflib.pf_layer_step(None, None, None, 1, None, None) == pf.PF_EINVAL
    assert pflib.pf_stack_step(None, None, 1, None, 1, None, None) == pf.PF_EINVAL
    assert pflib.pf_plan_run(None, None) == pf.PF_EINVAL
    pflib.pf_ctx_destroy(None)
    pflib.pf_layer_destroy(None)
    pflib.pf_plan_destroy(None)
    assert pflib.pf_last_error(None) == b""


def test_noalloc_entry_point_checks_its_limits_on_the_host(pflib):
    """pf_layer_step_noalloc refuses null arguments and sizes beyond its fixed scratch array
    before it touches a device."""
    from paper_2312_12456_amd import pf
    one = ctypes.c_void_p(256)  # never dereferenced
    w = pf.LayerWeights(*([one] * 11))
    assert pflib.pf_layer_step_noalloc(None, None, None, 1, None, None) == pf.PF_EINVAL
    for d, ffn, r, B in ((8200, 1024, 64, 1), (1024, 32832, 64, 1), (1024, 1024, 2056, 1),
                         (1024, 1024, 64, 5)):
        desc = pf.LayerDesc(d, ffn, r, pf.ACT_RELU, pf.W_FP16, 0.5)
        assert pflib.pf_layer_step_noalloc(ctypes.byref(desc), ctypes.byref(w), one, B, one,
                                           None) == pf.PF_ELIMIT


def test_product_package_does_not_touch_the_oracle():
    """No file of the product package imports or names the oracle."""
    pkg = os.path.join(ROOT, "paper_2312_12456_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "pf_oracle" not in src and "import oracle" not in src and \
                    "from oracle" not in src, f
