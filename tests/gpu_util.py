"""Helpers shared by the GPU parity tests: device state mirrored on the host for the oracle."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

import paper_2309_12381_amd as mpo
from oracle import ref

DEV = "cuda:0"
WORKERS = min(16, os.cpu_count() or 1)
FMT = {"bf16": (mpo.MPO_BF16, ref.BF16), "fp16": (mpo.MPO_FP16, ref.FP16)}


def say(msg):
    """Name the case before every GPU step, flushed, so that a fault can be attributed."""
    print("[gpu-case] " + msg, flush=True)


def dev_u16(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a.view(np.int16).copy()).to(DEV)


def host_u16(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().view(np.uint16).copy()


def dev_f32(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a.copy()).to(DEV)


def host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().copy()


def parallel_slices(n, fn, min_chunk=1 << 18):
    """Run fn(lo, hi) over slices of [0, n) on host threads (the oracle is elementwise)."""
    if n <= min_chunk:
        fn(0, n)
        return
    k = min(WORKERS, (n + min_chunk - 1) // min_chunk)
    bounds = np.linspace(0, n, k + 1).astype(np.int64)
    with ThreadPoolExecutor(k) as ex:
        list(ex.map(lambda i: fn(int(bounds[i]), int(bounds[i + 1])), range(k)))


def dev_res(a: np.ndarray) -> torch.Tensor:
    """Residual array (uint8 or uint16 on the host) as a device tensor of the same width."""
    if a.dtype == np.uint8:
        return torch.from_numpy(a.copy()).to(DEV)
    return dev_u16(a)


def host_res(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.uint8:
        return t.detach().cpu().numpy().copy()
    return host_u16(t)


def res_torch_dtype(res_bits: int):
    return torch.uint8 if 1 <= res_bits <= 8 else torch.int16


def ref_split(w32, rfmt, res_bits=0):
    hi = np.empty(w32.shape[0], np.uint16)
    res = np.empty(w32.shape[0], ref.res_dtype(res_bits))

    def f(lo, up):
        h, r = ref.split(w32[lo:up], rfmt, res_bits)
        hi[lo:up] = h
        res[lo:up] = r
    parallel_slices(w32.shape[0], f)
    return hi, res


def ref_adam(hi, res, g, m, v, cfg, step):
    parallel_slices(hi.shape[0], lambda lo, up: ref.adam_step(hi[lo:up], res[lo:up], g[lo:up], m[lo:up], v[lo:up],
                                                              cfg, step))


def ref_sgd(hi, res, g, buf, cfg, step):
    parallel_slices(hi.shape[0], lambda lo, up: ref.sgd_step(hi[lo:up], res[lo:up], g[lo:up],
                                                             None if buf is None else buf[lo:up], cfg, step))


ROUND = {"trunc": (mpo.MPO_ROUND_TRUNC, ref.TRUNC), "nearest": (mpo.MPO_ROUND_NEAREST, ref.NEAREST),
         "stochastic": (mpo.MPO_ROUND_STOCHASTIC, ref.STOCHASTIC)}


def cfg_pair(kind, fmt="bf16", gfmt=None, res_bits=0, round="trunc", seed=0, packed=False, **kw):
    """The same hyper-parameters for the library and for the oracle.  The number of extra bits
    kept is a property of each tensor in the library and of the step in the oracle."""
    gfmt = gfmt or fmt
    # remaining keywords (lr, betas, decay, loss_scale, grad_clip, ...) have the same names on both sides
    if kind == "adam":
        return (mpo.AdamCfg(weight_fmt=FMT[fmt][0], grad_fmt=FMT[gfmt][0], round=ROUND[round][0], seed=seed, **kw),
                ref.AdamCfg(weight_fmt=FMT[fmt][1], grad_fmt=FMT[gfmt][1], res_bits=res_bits, round=ROUND[round][1],
                            seed=seed, res_packed=packed, **kw))
    return (mpo.SgdCfg(weight_fmt=FMT[fmt][0], grad_fmt=FMT[gfmt][0], round=ROUND[round][0], seed=seed, **kw),
            ref.SgdCfg(weight_fmt=FMT[fmt][1], grad_fmt=FMT[gfmt][1], res_bits=res_bits, round=ROUND[round][1],
                       seed=seed, res_packed=packed, **kw))


class HostTensor:
    """Oracle-side state of one tensor."""

    def __init__(self, w32: np.ndarray, rfmt, with_v=True, res_bits=0, round="trunc", seed=0, tensor_id=0, packed=False):
        self.n = w32.shape[0]
        self.res_bits = res_bits
        self.tensor_id = tensor_id
        self.hi, self.res = ref.split(w32, rfmt, res_bits, ROUND[round][1], seed, tensor_id, packed)
        self.m = np.zeros(self.n, np.float32)
        self.v = np.zeros(self.n, np.float32) if with_v else None


class DevTensor:
    """GPU-side state of one tensor, split by the library itself."""

    def __init__(self, w32: np.ndarray, fmt, with_v=True, layer=0, grad=None, misalign=0, stream=None, res_bits=0,
                 round="trunc", seed=0, tensor_id=0, packed=False):
        n = w32.shape[0]
        self.n, self.layer, self.res_bits, self.packed = n, layer, res_bits, packed
        # optional misalignment: carve each array out of a larger one at an odd element offset
        def alloc(dtype):
            full = torch.zeros(n + misalign + 8, dtype=dtype, device=DEV)
            return full[misalign:misalign + n]
        self.hi = alloc(torch.int16)
        if packed:      # planes: one byte buffer, 16-byte aligned whatever the other arrays are
            self.res = torch.zeros(mpo.mpo_res_bytes(n, res_bits, True), dtype=torch.uint8, device=DEV)
        else:
            self.res = alloc(res_torch_dtype(res_bits))
        self.m = alloc(torch.float32)
        self.v = alloc(torch.float32) if with_v else None
        self.grad = grad if grad is not None else alloc(torch.int16)
        w = torch.zeros(n + misalign + 8, dtype=torch.float32, device=DEV)[misalign:misalign + n]
        w.copy_(torch.from_numpy(w32))
        mpo.mpo_split(w, self.hi, self.res, n, fmt=fmt, res_bits=res_bits, round=ROUND[round][0], seed=seed,
                      tensor_id=tensor_id, res_packed=packed, stream=stream)

    def spec(self):
        return mpo.Tensor(self.hi, self.res, self.grad, self.m, self.v, self.n, self.layer, self.res_bits, self.packed)


def assert_state_equal(d: DevTensor, h: HostTensor, what=""):
    torch.cuda.synchronize()
    ghi, gres = host_u16(d.hi), host_res(d.res)
    bad = np.flatnonzero(ghi != h.hi)
    assert bad.size == 0, "%s: %d of %d 16-bit weights differ, first at %d: gpu %04x oracle %04x" % (
        what, bad.size, h.n, bad[0], ghi[bad[0]], h.hi[bad[0]])
    # residual: one slot per parameter, or (packed) the plane bytes
    bad = np.flatnonzero(gres != h.res)
    assert bad.size == 0, "%s: %d of %d residual entries differ, first at %d: gpu %x oracle %x" % (
        what, bad.size, h.res.size, bad[0], gres[bad[0]], h.res[bad[0]])
    gm = host_f32(d.m)
    assert np.array_equal(gm.view(np.uint32), h.m.view(np.uint32)), what + ": m differs"
    if h.v is not None and d.v is not None:
        gv = host_f32(d.v)
        assert np.array_equal(gv.view(np.uint32), h.v.view(np.uint32)), what + ": v differs"
