"""Thin ctypes binding of libmpo.so (include/mpo.h): argument marshalling only.

Function names match the C entry points.  Tensors may be given as torch
tensors (their device pointer is taken) or as plain integer addresses.  Every
step of the method runs inside the library's HIP kernels; there is no Python
or CPU fallback: if the library is missing, importing this module fails.
"""
import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

# PyTorch first: it brings the process's HIP runtime (its own copy of libamdhip64.so.7).  Loaded in
# this order, libmpo.so binds to that same copy; loaded the other way round, the process would hold
# two runtimes and the library's launches would go to one that never saw torch's streams and memory.
import torch  # noqa: F401

from . import build as _build

MPO_OK = 0
MPO_ERR_INVALID_ARG = 1
MPO_ERR_UNSUPPORTED = 2
MPO_ERR_ALIAS = 3
MPO_ERR_HIP = 4
MPO_ERR_NOMEM = 5
MPO_ERR_TOO_LARGE = 6

MPO_BF16 = 0
MPO_FP16 = 1

MPO_ROUND_TRUNC = 0
MPO_ROUND_NEAREST = 1
MPO_ROUND_STOCHASTIC = 2

MPO_OPT_ADAM = 0
MPO_OPT_SGD = 1

MPO_MAX_LAYER_GRADS = 64
MPO_NOALLOC_MAX_TENSORS = 1024
MPO_NOALLOC_MAX_CHUNKS = 1 << 21


class mpo_tensor(ctypes.Structure):
    _fields_ = [("hi", ctypes.c_void_p), ("res", ctypes.c_void_p), ("grad", ctypes.c_void_p),
                ("m", ctypes.c_void_p), ("v", ctypes.c_void_p), ("n", ctypes.c_uint64),
                ("layer", ctypes.c_int32), ("res_bits", ctypes.c_int32), ("res_packed", ctypes.c_int32)]


class mpo_plan_opts(ctypes.Structure):
    _fields_ = [("small_layer_params", ctypes.c_uint64), ("host_only", ctypes.c_int32)]


class mpo_adam_cfg(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("weight_decay", ctypes.c_double),
                ("decoupled_wd", ctypes.c_int32), ("loss_scale", ctypes.c_double),
                ("weight_fmt", ctypes.c_int32), ("grad_fmt", ctypes.c_int32), ("round", ctypes.c_int32),
                ("seed", ctypes.c_uint64), ("grad_clip", ctypes.c_double)]


class mpo_sgd_cfg(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("momentum", ctypes.c_double), ("weight_decay", ctypes.c_double),
                ("loss_scale", ctypes.c_double),
                ("weight_fmt", ctypes.c_int32), ("grad_fmt", ctypes.c_int32), ("round", ctypes.c_int32),
                ("seed", ctypes.c_uint64), ("grad_clip", ctypes.c_double)]


EXPORTS = {
    "mpo_res_bytes": ([ctypes.c_uint64, ctypes.c_int32, ctypes.c_int32], ctypes.c_uint64),
    "mpo_split": ([ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int,
                   ctypes.c_int32, ctypes.c_int32, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p],
                  ctypes.c_int),
    "mpo_merge": ([ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int,
                   ctypes.c_int32, ctypes.c_int32, ctypes.c_int, ctypes.c_void_p], ctypes.c_int),
    "mpo_plan_create": ([ctypes.POINTER(mpo_tensor), ctypes.c_uint64, ctypes.POINTER(ctypes.c_void_p)], ctypes.c_int),
    "mpo_plan_create_host": ([ctypes.POINTER(mpo_tensor), ctypes.c_uint64, ctypes.POINTER(ctypes.c_void_p)],
                             ctypes.c_int),
    "mpo_plan_create_opts": ([ctypes.POINTER(mpo_tensor), ctypes.c_uint64, ctypes.POINTER(mpo_plan_opts),
                              ctypes.POINTER(ctypes.c_void_p)], ctypes.c_int),
    "mpo_plan_destroy": ([ctypes.c_void_p], ctypes.c_int),
    "mpo_plan_chunk_elems": ([ctypes.c_void_p], ctypes.c_uint64),
    "mpo_plan_num_chunks": ([ctypes.c_void_p], ctypes.c_uint64),
    "mpo_plan_num_params": ([ctypes.c_void_p], ctypes.c_uint64),
    "mpo_plan_get_chunk": ([ctypes.c_void_p, ctypes.c_uint64] + [ctypes.POINTER(ctypes.c_uint64)] * 3, ctypes.c_int),
    "mpo_plan_layer_info": ([ctypes.c_void_p, ctypes.c_int32] + [ctypes.POINTER(ctypes.c_uint64)] * 5, ctypes.c_int),
    "mpo_adam_step": ([ctypes.c_void_p, ctypes.POINTER(mpo_adam_cfg), ctypes.c_uint64, ctypes.c_void_p], ctypes.c_int),
    "mpo_sgd_step": ([ctypes.c_void_p, ctypes.POINTER(mpo_sgd_cfg), ctypes.c_uint64, ctypes.c_void_p], ctypes.c_int),
    "mpo_step_layer": ([ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint64,
                        ctypes.c_int, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p], ctypes.c_int),
    "mpo_adam_step_noalloc": ([ctypes.POINTER(mpo_tensor), ctypes.c_uint64, ctypes.POINTER(mpo_adam_cfg), ctypes.c_uint64,
                               ctypes.c_void_p], ctypes.c_int),
    "mpo_status_string": ([ctypes.c_int], ctypes.c_char_p),
    "mpo_last_hip_error": ([], ctypes.c_int),
}


def load_library(path: str):
    """A build of libmpo.so with the argument types of every export set."""
    lib = ctypes.CDLL(path)
    for name, (argtypes, restype) in EXPORTS.items():
        fn = getattr(lib, name)
        fn.argtypes = argtypes
        fn.restype = restype
    return lib


def _load():
    path = _build.LIB
    if not os.path.exists(path) or (_build.needs_build() and os.path.exists(_build.HIPCC)):
        # nothing built yet, or the sources are newer than the library (and there is a compiler):
        # build (a no-op when fresh); never fall back to another implementation
        path = _build.build()
    return load_library(path)


lib = _load()


class MpoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.mpo_status_string(status).decode()
        if status in (MPO_ERR_HIP, MPO_ERR_NOMEM):
            msg += " (hipError_t %d)" % lib.mpo_last_hip_error()
        super().__init__("%s: %s" % (where, msg))


def _check(status: int, where: str):
    if status != MPO_OK:
        raise MpoError(status, where)


def _ptr(x) -> Optional[int]:
    """Device address of a torch tensor, or an int / None passed through."""
    if x is None:
        return None
    if isinstance(x, int):
        return x or None
    return x.data_ptr() or None


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None        # torch.cuda.Stream


@dataclass
class AdamCfg:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0
    decoupled_wd: bool = True
    loss_scale: float = 1.0
    weight_fmt: int = MPO_BF16
    grad_fmt: int = MPO_BF16
    round: int = MPO_ROUND_TRUNC
    seed: int = 0
    grad_clip: float = 0.0

    def c(self) -> mpo_adam_cfg:
        return mpo_adam_cfg(self.lr, self.beta1, self.beta2, self.eps, self.weight_decay, int(self.decoupled_wd),
                            self.loss_scale, self.weight_fmt, self.grad_fmt, self.round, self.seed, self.grad_clip)


@dataclass
class SgdCfg:
    lr: float = 1e-2
    momentum: float = 0.9
    weight_decay: float = 0.0
    loss_scale: float = 1.0
    weight_fmt: int = MPO_BF16
    grad_fmt: int = MPO_BF16
    round: int = MPO_ROUND_TRUNC
    seed: int = 0
    grad_clip: float = 0.0

    def c(self) -> mpo_sgd_cfg:
        return mpo_sgd_cfg(self.lr, self.momentum, self.weight_decay, self.loss_scale, self.weight_fmt,
                           self.grad_fmt, self.round, self.seed, self.grad_clip)


def mpo_res_bytes(n: int, res_bits: int = 0, res_packed: bool = False) -> int:
    """Bytes of the residual buffer of a tensor of n parameters."""
    return int(lib.mpo_res_bytes(n, res_bits, int(res_packed)))


def mpo_split(w32, hi, res, n: int, fmt: int = MPO_BF16, res_bits: int = 0, round: int = MPO_ROUND_TRUNC,
              seed: int = 0, tensor_id: int = 0, res_packed: bool = False, stream=None):
    _check(lib.mpo_split(_ptr(w32), _ptr(hi), _ptr(res), n, fmt, res_bits, int(res_packed), round, seed, tensor_id,
                         _stream(stream)), "mpo_split")


def mpo_merge(hi, res, w32, n: int, fmt: int = MPO_BF16, res_bits: int = 0, round: int = MPO_ROUND_TRUNC,
              res_packed: bool = False, stream=None):
    _check(lib.mpo_merge(_ptr(hi), _ptr(res), _ptr(w32), n, fmt, res_bits, int(res_packed), round, _stream(stream)),
           "mpo_merge")


@dataclass
class Tensor:
    """One parameter tensor of a plan; fields as in mpo_tensor."""
    hi: object
    res: object
    grad: object
    m: object
    v: object
    n: int
    layer: int = 0
    res_bits: int = 0
    res_packed: bool = False


def _tensor_array(tensors: Sequence[Tensor]):
    arr = (mpo_tensor * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        arr[i] = mpo_tensor(_ptr(t.hi), _ptr(t.res), _ptr(t.grad), _ptr(t.m), _ptr(t.v), t.n, t.layer, t.res_bits,
                            int(t.res_packed))
    return arr


# mpo_plan_opts.small_layer_params of plans made without an explicit value (0 = the library's default);
# the GPU tests set it to run the same cases with short and with long chunks
default_small_layer_params = 0


class Plan:
    """Owns an mpo_plan*.  Keeps references to torch tensors so their memory outlives the plan.
    small_layer_params: see mpo_plan_opts in include/mpo.h (a tuning knob; None = the default)."""

    def __init__(self, tensors: Sequence[Tensor], host_only: bool = False, small_layer_params: Optional[int] = None):
        self._keep = list(tensors)
        arr = _tensor_array(tensors)
        handle = ctypes.c_void_p()
        opts = mpo_plan_opts(default_small_layer_params if small_layer_params is None else small_layer_params,
                             int(host_only))
        _check(lib.mpo_plan_create_opts(arr, len(tensors), ctypes.byref(opts), ctypes.byref(handle)), "mpo_plan_create")
        self._h = handle

    def destroy(self):
        if self._h is not None:
            h, self._h = self._h, None
            _check(lib.mpo_plan_destroy(h), "mpo_plan_destroy")

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # layout queries
    @property
    def chunk_elems(self) -> int:
        return lib.mpo_plan_chunk_elems(self._h)

    @property
    def num_chunks(self) -> int:
        return lib.mpo_plan_num_chunks(self._h)

    @property
    def num_params(self) -> int:
        return lib.mpo_plan_num_params(self._h)

    def chunk(self, i: int):
        """(tensor, first element, number of elements) of chunk i, in launch order."""
        t, f, c = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
        _check(lib.mpo_plan_get_chunk(self._h, i, ctypes.byref(t), ctypes.byref(f), ctypes.byref(c)),
               "mpo_plan_get_chunk")
        return t.value, f.value, c.value

    def layer_info(self, layer: int):
        a, b, c, d, e = (ctypes.c_uint64() for _ in range(5))
        _check(lib.mpo_plan_layer_info(self._h, layer, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c),
                                       ctypes.byref(d), ctypes.byref(e)), "mpo_plan_layer_info")
        return {"first_chunk": a.value, "num_chunks": b.value, "num_tensors": c.value, "num_params": d.value,
                "chunk_elems": e.value}


def mpo_adam_step(plan: Plan, cfg: AdamCfg, step: int, stream=None):
    c = cfg.c()
    _check(lib.mpo_adam_step(plan._h, ctypes.byref(c), step, _stream(stream)), "mpo_adam_step")


def mpo_adam_step_noalloc(tensors, cfg: AdamCfg, step: int, stream=None):
    """mpo_adam_step without a plan, for callers that cannot allocate device memory.  `tensors` is a
    sequence of Tensor, or an array made by tensor_array() (marshalled once, reused on every call)."""
    arr, n = tensors if isinstance(tensors, tuple) else (_tensor_array(tensors), len(tensors))
    c = cfg.c()
    _check(lib.mpo_adam_step_noalloc(arr, n, ctypes.byref(c), step, _stream(stream)), "mpo_adam_step_noalloc")


def tensor_array(tensors: Sequence[Tensor]):
    """A C array of mpo_tensor for mpo_adam_step_noalloc, with its length."""
    return _tensor_array(tensors), len(tensors)


def mpo_sgd_step(plan: Plan, cfg: SgdCfg, step: int, stream=None):
    c = cfg.c()
    _check(lib.mpo_sgd_step(plan._h, ctypes.byref(c), step, _stream(stream)), "mpo_sgd_step")


def mpo_step_layer(plan: Plan, layer: int, cfg, step: int, grads: Optional[Sequence] = None, stream=None):
    """cfg is an AdamCfg or an SgdCfg; grads is None (plan's own) or one tensor/address per tensor of the layer."""
    opt = MPO_OPT_ADAM if isinstance(cfg, AdamCfg) else MPO_OPT_SGD
    c = cfg.c()
    if grads is None:
        gp, ng = None, 0
    else:
        ng = len(grads)
        gp = (ctypes.c_void_p * max(ng, 1))(*[_ptr(g) for g in grads])
    _check(lib.mpo_step_layer(plan._h, layer, gp, ng, opt, ctypes.cast(ctypes.byref(c), ctypes.c_void_p), step,
                              _stream(stream)), "mpo_step_layer")
