"""Build libmpo.so (hand-written HIP for gfx950 + the C entry points) in-tree with hipcc, and
libmpo_probe.so, the bandwidth probe bench.py measures the step kernel against."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmpo.so")
SOURCES = [os.path.join(CSRC, "mpo_host.cpp"), os.path.join(CSRC, "mpo_kernels.hip")]
HEADERS = [os.path.join(CSRC, "mpo_internal.h"), os.path.join(ROOT, "include", "mpo.h")]
PROBE_LIB = os.path.join(HERE, "libmpo_probe.so")
PROBE_SOURCES = [os.path.join(CSRC, "stream_probe.hip")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# One IEEE operation per source-level operation: no contraction into FMA, correctly rounded
# division and square root, denormals kept; no fast-math anywhere.  Packed fp32 VALU forms are
# switched off (the compiler would otherwise pair independent fp32 operations).
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-fast-math",
    "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _stale(lib, inputs) -> bool:
    if not os.path.exists(lib):
        return True
    t = os.path.getmtime(lib)
    return any(os.path.getmtime(f) > t for f in inputs)


def needs_build() -> bool:
    return _stale(LIB, SOURCES + HEADERS)


def _compile(sources, out, extra=()):
    tmp = out + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, *FLAGS, *extra, "-x", "hip", *sources, "-o", tmp])
    os.replace(tmp, out)
    return out


def build(force: bool = False, extra=(), out: str = LIB) -> str:
    """Compile the library.  `extra` adds compiler flags for experiments."""
    if not force and out == LIB and not needs_build():
        return out
    return _compile(SOURCES, out, extra)


def build_probe(force: bool = False) -> str:
    """Compile the bandwidth probe (a measuring aid; the library does not depend on it)."""
    if force or _stale(PROBE_LIB, PROBE_SOURCES):
        _compile(PROBE_SOURCES, PROBE_LIB)
    return PROBE_LIB


if __name__ == "__main__":
    print(build(force=True, extra=sys.argv[1:]))
    print(build_probe(force=True))
