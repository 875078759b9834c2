"""ctypes access to libmpo_probe.so: the step's memory traffic without its arithmetic.

A measuring aid for bench.py (what this access pattern reaches on the GPU at hand); the
library proper does not depend on it.  The probe overwrites the arrays it is given.
"""
import ctypes
import os

import torch  # noqa: F401  (first, so that the probe library binds to the HIP runtime torch loaded)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmpo_probe.so")
_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build          # nothing built yet: build once (needs hipcc)
            _build.build_probe()
        _lib = ctypes.CDLL(LIB_PATH)
        _lib.mpo_probe_stream.restype = ctypes.c_int
        _lib.mpo_probe_stream.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_longlong, ctypes.c_void_p]
    return _lib


def stream_probe(hi, res, grad, m, v, n: int, stream=None) -> None:
    """Read hi, res, grad (16-bit) and m, v (fp32) and write hi, res, m, v back, over the first
    n - n % 4096 elements.  v=None: the 18-byte (SGD-shaped) traffic.  Device tensors, 16-byte aligned."""
    rc = _load().mpo_probe_stream(hi.data_ptr(), res.data_ptr(), grad.data_ptr(), m.data_ptr(),
                                  v.data_ptr() if v is not None else None, n,
                                  stream.cuda_stream if stream is not None else None)
    if rc != 0:
        raise RuntimeError("mpo_probe_stream failed (%d)" % rc)
