"""Compile the CPU oracle (oracle/mpo_ref.c) into oracle/libmpo_ref.so with gcc.

Test infrastructure only: nothing in the product package imports this.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "mpo_ref.c")
LIB = os.path.join(HERE, "libmpo_ref.so")

# No FMA contraction, no fast-math: every fp32 operation rounds on its own and
# denormals are kept (Section 3.1: the update is carried out in full precision).
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
          "-Wall", "-Wextra", "-Werror"]


def build(force: bool = False) -> str:
    stale = (not os.path.exists(LIB)
             or os.path.getmtime(LIB) < max(os.path.getmtime(SRC),
                                            os.path.getmtime(os.path.join(HERE, "mpo_ref.h"))))
    if force or stale:
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, SRC, "-lm"])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
