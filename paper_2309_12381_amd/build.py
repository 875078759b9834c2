"""Build libmpo.so (hand-written HIP for gfx950 + the C entry points) in-tree with hipcc, and
libmpo_probe.so, the bandwidth probe bench.py measures the step kernel against (and the native placement search)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmpo.so")
# (source, extra flags): the step kernels are one source compiled in four parts (Adam / SGD, gradient
# pointers from the plan / per call) so that the parts build side by side
PARTS = [("mpo_host.cpp", ()), ("mpo_split_merge.hip", ()), ("mpo_noalloc.hip", ()),
         ("mpo_step.hip", ("-DMPO_PART_OPT=0", "-DMPO_PART_OV=0")), ("mpo_step.hip", ("-DMPO_PART_OPT=0", "-DMPO_PART_OV=1")),
         ("mpo_step.hip", ("-DMPO_PART_OPT=1", "-DMPO_PART_OV=0")), ("mpo_step.hip", ("-DMPO_PART_OPT=1", "-DMPO_PART_OV=1"))]
SOURCES = sorted({os.path.join(CSRC, src) for src, _ in PARTS})
HEADERS = [os.path.join(CSRC, "mpo_internal.h"), os.path.join(CSRC, "mpo_device.h"), os.path.join(ROOT, "include", "mpo.h")]
PROBE_LIB = os.path.join(HERE, "libmpo_probe.so")
PROBE_SOURCES = [os.path.join(CSRC, "stream_probe.hip"), os.path.join(CSRC, "place_second.cpp")]
PROBE_HEADERS = [os.path.join(ROOT, "include", "mpo_probe.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# One IEEE operation per source-level operation: no contraction into FMA, correctly rounded
# division and square root, denormals kept; no fast-math anywhere.  Packed fp32 VALU forms are
# switched off (the compiler would otherwise pair independent fp32 operations).
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
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


def probe_needs_build() -> bool:
    return _stale(PROBE_LIB, PROBE_SOURCES + PROBE_HEADERS)


def _compile(sources, out, extra=()):
    tmp = out + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, *FLAGS, "-shared", *extra, "-x", "hip", *sources, "-o", tmp])
    os.replace(tmp, out)
    return out


def build(force: bool = False, extra=(), out: str = LIB, csrc: str = CSRC) -> str:
    """Compile the library: every part to an object file (in parallel), then one link.
    `extra` adds compiler flags, `out` and `csrc` name another output and another copy of the sources:
    for experiments (bench.py --compare-lib times two builds against each other in one process)."""
    if not force and out == LIB and not needs_build():
        return out
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    flags = FLAGS[:-1] + [csrc]         # the last flag is the include path of the sources' own headers
    with tempfile.TemporaryDirectory(prefix="mpo_build_") as tmpdir:
        def one(i):
            src, defs = PARTS[i]
            obj = os.path.join(tmpdir, "part%d.o" % i)
            subprocess.check_call([HIPCC, *flags, *extra, *defs, "-x", "hip", "-c", os.path.join(csrc, src), "-o", obj])
            return obj
        with ThreadPoolExecutor(min(len(PARTS), os.cpu_count() or 1)) as ex:
            objs = list(ex.map(one, range(len(PARTS))))
        tmp = out + ".tmp.%d" % os.getpid()
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-fPIC", "-shared", *objs, "-o", tmp])
        os.replace(tmp, out)
    return out


def build_probe(force: bool = False) -> str:
    """Compile the bandwidth probe (a measuring aid; the library does not depend on it)."""
    if force or probe_needs_build():
        _compile(PROBE_SOURCES, PROBE_LIB)
    return PROBE_LIB


C_CALLER = os.path.join(HERE, "mpo_c_caller")
C_CALLER_SOURCES = [os.path.join(CSRC, "c_caller.cpp")]


def build_c_caller(force: bool = False) -> str:
    """Compile the stand-alone program that uses the C interface alone (bench.py --c-caller runs it); it finds
    libmpo.so and libmpo_probe.so beside itself."""
    if force or _stale(C_CALLER, C_CALLER_SOURCES + HEADERS + PROBE_HEADERS + [LIB, PROBE_LIB]):
        tmp = C_CALLER + ".tmp.%d" % os.getpid()
        subprocess.check_call([HIPCC, "-O2", "-std=c++17", "-Wall", "-Wextra", "-I", os.path.join(ROOT, "include"),
                               "-x", "hip", "--offload-arch=gfx950", *C_CALLER_SOURCES, "-x", "none", LIB, PROBE_LIB,
                               "-Wl,-rpath,$ORIGIN", "-o", tmp])
        os.replace(tmp, C_CALLER)
    return C_CALLER


if __name__ == "__main__":
    print(build(force=True, extra=sys.argv[1:]))
    print(build_probe(force=True))
    print(build_c_caller(force=True))
