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


class mpo_place_report(ctypes.Structure):
    _fields_ = [("split", ctypes.c_int32), ("candidates", ctypes.c_int32), ("chosen", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("one_region_GBps", ctypes.c_double * 4), ("chosen_GBps", ctypes.c_double * 4),
                ("peak_transient_bytes", ctypes.c_uint64), ("max_transient_bytes", ctypes.c_uint64),
                ("block_bytes", ctypes.c_uint64), ("v_offset", ctypes.c_uint64), ("grad_offset", ctypes.c_uint64)]


def _load():
    global _lib
    if _lib is None:
        from . import build as _build
        if not os.path.exists(LIB_PATH) or (_build.probe_needs_build() and os.path.exists(_build.HIPCC)):
            _build.build_probe()                   # nothing built yet, or older than its source: build (needs hipcc)
        _lib = ctypes.CDLL(LIB_PATH)
        _lib.mpo_probe_stream.restype = ctypes.c_int
        _lib.mpo_probe_stream.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_longlong, ctypes.c_void_p]
        _lib.mpo_probe_num_variants.restype = ctypes.c_int
        _lib.mpo_probe_variant_name.restype = ctypes.c_char_p
        _lib.mpo_probe_variant_name.argtypes = [ctypes.c_int]
        _lib.mpo_probe_variant.restype = ctypes.c_int
        _lib.mpo_probe_variant.argtypes = [ctypes.c_int] + [ctypes.c_void_p] * 5 + [ctypes.c_longlong, ctypes.c_int,
                                                                                   ctypes.c_void_p]
        _lib.mpo_probe_plain.restype = ctypes.c_int
        _lib.mpo_probe_plain.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_ulonglong,
                                         ctypes.c_void_p, ctypes.c_void_p]
        _lib.mpo_place_second.restype = ctypes.c_int
        _lib.mpo_place_second.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64,
                                          ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int,
                                          ctypes.POINTER(ctypes.c_void_p),
                                          ctypes.POINTER(mpo_place_report), ctypes.c_void_p]
        _lib.mpo_place_free.restype = ctypes.c_int
        _lib.mpo_place_free.argtypes = [ctypes.c_void_p]
    return _lib


def stream_probe(hi, res, grad, m, v, n: int, stream=None) -> None:
    """Read hi, res, grad (16-bit) and m, v (fp32) and write hi, res, m, v back, over the first
    n - n % 4096 elements.  v=None: the 18-byte (SGD-shaped) traffic.  Device tensors, 16-byte aligned."""
    rc = _load().mpo_probe_stream(hi.data_ptr(), res.data_ptr(), grad.data_ptr(), m.data_ptr(),
                                  v.data_ptr() if v is not None else None, n,
                                  stream.cuda_stream if stream is not None else None)
    if rc != 0:
        raise RuntimeError("mpo_probe_stream failed (%d)" % rc)


def variants():
    """Descriptions of the launch-shape variants mpo_probe_variant knows, in order (0 = the step kernel's shape)."""
    lib = _load()
    return [lib.mpo_probe_variant_name(i).decode() for i in range(lib.mpo_probe_num_variants())]


def stream_variant(variant: int, hi, res, grad, m, v, n: int, compute_units: int, stream=None) -> None:
    """The Adam-shaped traffic over the first n - n % 131072 elements in variant `variant` of the launch shape."""
    rc = _load().mpo_probe_variant(variant, hi.data_ptr(), res.data_ptr(), grad.data_ptr(), m.data_ptr(), v.data_ptr(), n,
                                   compute_units, stream.cuda_stream if stream is not None else None)
    if rc != 0:
        raise RuntimeError("mpo_probe_variant failed (%d)" % rc)


PLAIN_READ, PLAIN_WRITE, PLAIN_INPLACE = 0, 1, 2


def plain_streams(mode: int, arrays, nbytes: int, sink, stream=None) -> None:
    """k (1 to 8) device arrays of nbytes bytes each walked in lock step: read, written, or read and written back.
    `sink`: a 4-byte device tensor."""
    ptrs = (ctypes.c_void_p * len(arrays))(*[a.data_ptr() for a in arrays])
    rc = _load().mpo_probe_plain(mode, ptrs, len(arrays), nbytes, sink.data_ptr(),
                                 stream.cuda_stream if stream is not None else None)
    if rc != 0:
        raise RuntimeError("mpo_probe_plain failed (%d)" % rc)


def place_second_native(hi, m, res_bytes: int, v_bytes: int, grad_bytes: int, max_transient_bytes: int = 0,
                        keep_hi: bool = True, stream=None):
    """mpo_place_second, the C interface's placement search (placement.py is the same search on torch tensors):
    returns (device address of a block allocated with hipMalloc that holds res, v and grad, report as a dict with
    the offsets of v and grad).  Free the block with place_free.  `m` is overwritten."""
    block = ctypes.c_void_p()
    rep = mpo_place_report()
    rc = _load().mpo_place_second(hi.data_ptr(), hi.numel() * hi.element_size(), m.data_ptr(), m.numel() * m.element_size(),
                                  res_bytes, v_bytes, grad_bytes, max_transient_bytes, 1 if keep_hi else 0, ctypes.byref(block),
                                  ctypes.byref(rep), stream.cuda_stream if stream is not None else None)
    if rc != 0:
        raise RuntimeError("mpo_place_second failed (%d)" % rc)
    return block.value, {"split": bool(rep.split), "candidates": rep.candidates, "chosen": rep.chosen,
                         "one_region_GBps": list(rep.one_region_GBps), "chosen_GBps": list(rep.chosen_GBps),
                         "peak_transient_bytes": rep.peak_transient_bytes, "max_transient_bytes": rep.max_transient_bytes,
                         "block_bytes": rep.block_bytes, "v_offset": rep.v_offset, "grad_offset": rep.grad_offset}


def place_free(block: int) -> None:
    rc = _load().mpo_place_free(block)
    if rc != 0:
        raise RuntimeError("mpo_place_free failed (%d)" % rc)
