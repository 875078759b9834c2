"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU code involved).

* the oracle: a driver in C calls every entry point on every storage kind with arrays of exactly
  the stated sizes;
* the library's host side (csrc/mpo_host.cpp: validation, overlap detection, plan building, layout
  queries): a driver builds host plans over hundreds of tensors and walks every error path, with
  the kernel launchers replaced by stubs that must not be reached;
* the entry point that allocates nothing (csrc/mpo_noalloc.hip, a HIP file: built with hipcc, sanitizers on the
  host side only): lists of up to 1024 tensors through its validation, layer ordering and chunk layout, all of
  which live in fixed-size stack arrays, up to the first HIP call, which fails on a machine without a GPU.
"""
import os
import subprocess

from oracle import build as obuild

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(exe):
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=600, env=ENV)
    assert out.returncode == 0, (out.stdout + out.stderr)[-4000:]
    return out.stdout


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "sanitize_oracle"
    subprocess.check_call(["gcc", "-std=c11", *SAN, "-ffp-contract=off", "-fno-fast-math", "-I", obuild.HERE,
                           obuild.SRC, os.path.join(HERE, "sanitize_oracle_main.c"), "-o", str(exe), "-lm"])
    assert "cases" in _run(exe)


def test_library_host_side_is_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "sanitize_host"
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    csrc = os.path.join(ROOT, "paper_2309_12381_amd", "csrc")
    subprocess.check_call(["g++", "-std=c++17", *SAN, "-w", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
                           "-I", os.path.join(ROOT, "include"), "-I", csrc, os.path.join(csrc, "mpo_host.cpp"),
                           os.path.join(HERE, "sanitize_host_main.cpp"), "-o", str(exe),
                           "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath," + os.path.join(rocm, "lib")])
    assert "plans" in _run(exe)


def test_noalloc_entry_point_host_side_is_clean_under_asan_and_ubsan(tmp_path):
    import shutil
    import pytest
    from paper_2309_12381_amd import build as lbuild
    if not shutil.which(lbuild.HIPCC) and not os.path.exists(lbuild.HIPCC):
        pytest.skip("no hipcc")
    exe = tmp_path / "sanitize_noalloc"
    csrc = os.path.join(ROOT, "paper_2309_12381_amd", "csrc")
    host_san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"):
        host_san += ["-Xarch_host", f]
    subprocess.check_call([lbuild.HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-w", *host_san,
                           "-I", os.path.join(ROOT, "include"), "-I", csrc, "-x", "hip",
                           os.path.join(csrc, "mpo_noalloc.hip"), os.path.join(csrc, "mpo_host.cpp"),
                           os.path.join(HERE, "sanitize_noalloc_main.cpp"), "-o", str(exe)])
    assert "lists" in _run(exe)
