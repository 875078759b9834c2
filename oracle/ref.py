"""ctypes access to the CPU oracle (oracle/mpo_ref.c) on numpy arrays.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports it.

Each function forwards to the C routine of the same name; there is no
arithmetic here.  Arrays are updated in place, as the C routines do.

`Oracle(path)` wraps one compiled library; the module-level functions use the
one built from oracle/mpo_ref.c.  (Tests of the pins load deliberately broken
builds through the same class to show that the pins notice.)
"""
import ctypes
from dataclasses import dataclass

import numpy as np

from . import build as _build

BF16 = 0
FP16 = 1

TRUNC = 0
NEAREST = 1
STOCHASTIC = 2

_u16p = ctypes.POINTER(ctypes.c_uint16)
_f32p = ctypes.POINTER(ctypes.c_float)


class _AdamCfg(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("weight_decay", ctypes.c_double),
                ("decoupled_wd", ctypes.c_int32), ("loss_scale", ctypes.c_double),
                ("weight_fmt", ctypes.c_int32), ("grad_fmt", ctypes.c_int32), ("res_bits", ctypes.c_int32),
                ("res_packed", ctypes.c_int32), ("round", ctypes.c_int32), ("seed", ctypes.c_uint64),
                ("grad_clip", ctypes.c_double)]


class _SgdCfg(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("momentum", ctypes.c_double),
                ("weight_decay", ctypes.c_double), ("loss_scale", ctypes.c_double),
                ("weight_fmt", ctypes.c_int32), ("grad_fmt", ctypes.c_int32), ("res_bits", ctypes.c_int32),
                ("res_packed", ctypes.c_int32), ("round", ctypes.c_int32), ("seed", ctypes.c_uint64),
                ("grad_clip", ctypes.c_double)]


def res_dtype(res_bits: int):
    """Storage type of the residual: one byte per element for 1..8 kept bits, else two."""
    return np.uint8 if 1 <= res_bits <= 8 else np.uint16


@dataclass
class AdamCfg:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0
    decoupled_wd: bool = True
    loss_scale: float = 1.0
    weight_fmt: int = BF16
    grad_fmt: int = BF16
    res_bits: int = 0
    round: int = TRUNC
    seed: int = 0
    grad_clip: float = 0.0
    res_packed: bool = False

    def _c(self):
        return _AdamCfg(self.lr, self.beta1, self.beta2, self.eps, self.weight_decay,
                        int(self.decoupled_wd), self.loss_scale, self.weight_fmt, self.grad_fmt, self.res_bits,
                        int(self.res_packed), self.round, self.seed, self.grad_clip)


@dataclass
class SgdCfg:
    lr: float = 1e-2
    momentum: float = 0.9
    weight_decay: float = 0.0
    loss_scale: float = 1.0
    weight_fmt: int = BF16
    grad_fmt: int = BF16
    res_bits: int = 0
    round: int = TRUNC
    seed: int = 0
    grad_clip: float = 0.0
    res_packed: bool = False

    def _c(self):
        return _SgdCfg(self.lr, self.momentum, self.weight_decay, self.loss_scale,
                       self.weight_fmt, self.grad_fmt, self.res_bits, int(self.res_packed), self.round, self.seed,
                       self.grad_clip)


def _chk(a, dtype, n=None):
    if not isinstance(a, np.ndarray) or a.dtype != dtype or a.ndim != 1 or not a.flags.c_contiguous:
        raise TypeError("expected a contiguous 1-d %s array" % np.dtype(dtype).name)
    if n is not None and a.shape[0] != n:
        raise ValueError("length mismatch")
    return a


def _p16(a):
    return a.ctypes.data_as(_u16p)


def _pv(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _p32(a):
    return a.ctypes.data_as(_f32p)


class Oracle:
    BF16 = BF16
    FP16 = FP16
    TRUNC = TRUNC
    NEAREST = NEAREST
    STOCHASTIC = STOCHASTIC
    AdamCfg = AdamCfg
    SgdCfg = SgdCfg

    def __init__(self, path):
        lib = ctypes.CDLL(path)
        lib.mpo_ref_split.argtypes = [_f32p, _u16p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64]
        lib.mpo_ref_res_bytes.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.mpo_ref_res_bytes.restype = ctypes.c_uint64
        lib.mpo_ref_split.restype = None
        lib.mpo_ref_merge.argtypes = [_u16p, ctypes.c_void_p, _f32p, ctypes.c_uint64, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_int]
        lib.mpo_ref_merge.restype = None
        lib.mpo_ref_adam_step.argtypes = [_u16p, ctypes.c_void_p, _u16p, _f32p, _f32p, ctypes.c_uint64,
                                          ctypes.POINTER(_AdamCfg), ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64]
        lib.mpo_ref_adam_step.restype = None
        lib.mpo_ref_sgd_step.argtypes = [_u16p, ctypes.c_void_p, _u16p, _f32p, ctypes.c_uint64,
                                         ctypes.POINTER(_SgdCfg), ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64]
        lib.mpo_ref_sgd_step.restype = None
        lib.mpo_ref_cvt16.argtypes = [ctypes.c_uint16, ctypes.c_int]
        lib.mpo_ref_cvt16.restype = ctypes.c_float
        lib.mpo_ref_philox4x32_10.argtypes = [ctypes.POINTER(ctypes.c_uint32)] * 3
        lib.mpo_ref_philox4x32_10.restype = None
        self._lib = lib

    def philox(self, counter, key):
        """One Philox4x32-10 block."""
        c = (ctypes.c_uint32 * 4)(*counter)
        k = (ctypes.c_uint32 * 2)(*key)
        o = (ctypes.c_uint32 * 4)()
        self._lib.mpo_ref_philox4x32_10(c, k, o)
        return list(o)

    def res_bytes(self, n, fmt=BF16, res_bits=0, packed=False):
        return int(self._lib.mpo_ref_res_bytes(n, fmt, res_bits, int(packed)))

    def _res_ok(self, res, n, fmt, res_bits, packed):
        if packed:
            _chk(res, np.uint8, self.res_bytes(n, fmt, res_bits, True))
        else:
            _chk(res, res_dtype(res_bits), n)

    def split(self, w32, fmt=BF16, res_bits=0, round=TRUNC, seed=0, tensor_id=0, packed=False, first_index=0):
        """fp32 array -> (hi uint16, res) arrays; res is uint16 or uint8 per value, or with
        packed=True the bit planes as one uint8 array (res_bits then counts the bits stored per
        value: with STOCHASTIC the leading one is the flag).  first_index: position, in its tensor,
        of the array's first element (selects the random numbers of STOCHASTIC; 0 when packed)."""
        _chk(w32, np.float32)
        n = w32.shape[0]
        hi = np.empty(n, np.uint16)
        res = np.zeros(self.res_bytes(n, fmt, res_bits, True), np.uint8) if packed else np.empty(n, res_dtype(res_bits))
        self._lib.mpo_ref_split(_p32(w32), _p16(hi), _pv(res), n, fmt, res_bits, int(packed), round, seed, tensor_id,
                                first_index)
        return hi, res

    def merge(self, hi, res, fmt=BF16, res_bits=0, round=TRUNC, packed=False):
        """(hi, res) arrays -> fp32 array."""
        n = _chk(hi, np.uint16).shape[0]
        self._res_ok(res, n, fmt, res_bits, packed)
        w32 = np.empty(n, np.float32)
        self._lib.mpo_ref_merge(_p16(hi), _pv(res), _p32(w32), n, fmt, res_bits, int(packed), round)
        return w32

    def adam_step(self, hi, res, grad, m, v, cfg: AdamCfg, step: int, tensor_id: int = 0, first_index: int = 0):
        """One Adam step on one tensor (or on the slice of it that starts at first_index), in place
        on hi, res, m, v."""
        n = _chk(hi, np.uint16).shape[0]
        self._res_ok(res, n, cfg.weight_fmt, cfg.res_bits, cfg.res_packed)
        _chk(grad, np.uint16, n)
        _chk(m, np.float32, n)
        _chk(v, np.float32, n)
        if step < 1:
            raise ValueError("step counts from 1")
        c = cfg._c()
        self._lib.mpo_ref_adam_step(_p16(hi), _pv(res), _p16(grad), _p32(m), _p32(v), n,
                                    ctypes.byref(c), step, tensor_id, first_index)

    def sgd_step(self, hi, res, grad, buf, cfg: SgdCfg, step: int, tensor_id: int = 0, first_index: int = 0):
        """One SGD(-momentum) step on one tensor (or on the slice of it that starts at first_index),
        in place on hi, res, buf."""
        n = _chk(hi, np.uint16).shape[0]
        self._res_ok(res, n, cfg.weight_fmt, cfg.res_bits, cfg.res_packed)
        _chk(grad, np.uint16, n)
        if cfg.momentum != 0.0:
            _chk(buf, np.float32, n)
        if step < 1:
            raise ValueError("step counts from 1")
        c = cfg._c()
        bp = _p32(buf) if buf is not None else ctypes.cast(None, _f32p)
        self._lib.mpo_ref_sgd_step(_p16(hi), _pv(res), _p16(grad), bp, n, ctypes.byref(c), step, tensor_id,
                                   first_index)

    def cvt16(self, x: int, fmt=BF16) -> float:
        """One 16-bit float pattern read as fp32."""
        return float(self._lib.mpo_ref_cvt16(int(x) & 0xFFFF, fmt))


    res_dtype = staticmethod(res_dtype)


_default = Oracle(_build.build())
split = _default.split
merge = _default.merge
adam_step = _default.adam_step
sgd_step = _default.sgd_step
cvt16 = _default.cvt16
philox = _default.philox
res_bytes = _default.res_bytes
