"""Builds libpf.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpf.so")
SOURCES = [os.path.join(CSRC, "pf.hip")]
PROBE_LIB = os.path.join(HERE, "libpf_probe.so")          # latency-floor probes for bench.py
PROBE_SOURCES = [os.path.join(CSRC, "probe.hip")]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _compile(lib, sources, verbose, extra):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = lib + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + list(extra) + ["-o", tmp] + sources
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, lib)
    return lib


def build_probe(verbose=False, extra=()):
    return _compile(PROBE_LIB, PROBE_SOURCES, verbose, extra)


def build(verbose=False, extra=()):
    build_probe(verbose, extra)
    return _compile(LIB, SOURCES, verbose, extra)


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
