"""Device-side state of a synthetic workload and the stepping loops around libmpo.

PyTorch is used for device memory, streams and seeded random numbers only; every
step of the method is a call into the library.  Shared by bench.py, the smoke
check and the full-size GPU tests.
"""
from dataclasses import dataclass
from typing import Dict, List

import torch

from . import binding as mpo
from . import placement
from . import synth

FMT = {"bf16": mpo.MPO_BF16, "fp16": mpo.MPO_FP16}
# Tensors start at multiples of 64 elements in the flat arrays: 128 bytes, one memory line, for the
# 16-bit arrays (256 for the fp32 ones).  The library only needs 16 bytes for its vector path, but a
# tensor that starts inside a line makes every row of its chunks straddle lines, and with streaming
# stores that costs 14 % on a list of many odd-length tensors (c1: 4.98 -> 5.69 TB/s).
ALIGN_ELEMS = 64


def _round_up(x: int, k: int) -> int:
    return (x + k - 1) // k * k


@dataclass
class TensorView:
    spec: synth.Spec
    off: int            # element offset into the flat state arrays (multiple of ALIGN_ELEMS)
    goff: int           # element offset into the reused gradient buffer, local to the tensor's layer


class ModelState:
    """hi, res, m, v for every tensor of a workload, each kind in ONE flat allocation (large
    blocks keep the driver on large page fragments), plus ONE gradient buffer sized for the
    largest layer and reused by every layer (Section 3.2: a gradient is consumed as soon as it
    exists and never kept).  For workloads stepped in one launch the buffer holds all gradients.
    With `place` (the default) a large state is laid out over two HBM regions: hi and m in one,
    res, v and the gradient buffer in another (see placement.py); `self.placement` is the report."""

    def __init__(self, wl: synth.Workload, device="cuda:0", seed: int = 2309, keep_w32_samples=None,
                 res_bits: int = 0, round: int = mpo.MPO_ROUND_TRUNC, rng_seed: int = 0x2309_12381,
                 res_packed: bool = False, place: bool = True, small_layer_params=None):
        self.wl = wl
        self.res_packed = res_packed        # extra bits stored in packed planes (Section 3.1, Figure 1)
        self.round = round                  # how hi is rounded (Section 3.1, last paragraph)
        self.rng_seed = rng_seed            # random stream of stochastic rounding
        self.res_bits = res_bits            # extra bits kept per weight, 0 = all (Section 3.1)
        self.res_bytes = 1 if 1 <= res_bits <= 8 else 2
        self.device = device
        self.fmt = FMT[wl.fmt]
        self.views: List[TensorView] = []
        off = 0
        layer_fill: Dict[int, int] = {}
        for s in wl.tensors:
            if wl.per_layer:
                g = layer_fill.get(s.layer, 0)
                layer_fill[s.layer] = g + _round_up(s.n, ALIGN_ELEMS)
            else:
                g = off
            self.views.append(TensorView(s, off, g))
            off += _round_up(s.n, ALIGN_ELEMS)
        self.total = off
        self.grad_len = max(layer_fill.values()) if wl.per_layer else off
        if res_packed:
            # one byte buffer; each tensor's planes start at a multiple of 16 bytes
            self.res_off, fill = [], 0
            for tv in self.views:
                self.res_off.append(fill)
                fill += mpo.mpo_res_bytes(tv.spec.n, res_bits, True)
            res_spec = (fill, torch.uint8)
        else:
            self.res_off = [tv.off for tv in self.views]
            res_spec = (self.total, torch.uint8 if self.res_bytes == 1 else torch.int16)
        self.gdtype = torch.bfloat16 if wl.fmt == "bf16" else torch.float16
        arrays, self.placement = placement.allocate_state(self.total, res_spec, (self.grad_len, self.gdtype), device,
                                                          zero_res=res_packed, place=place)
        self.hi, self.m = arrays["hi"], arrays["m"]
        self.res, self.v, self.grad = arrays["res"], arrays["v"], arrays["grad"]
        self.seed = seed
        self.w32_samples = {}
        # weights: fp32 ~ N(0, std^2), drawn per tensor on the device, then split by the library
        for i, tv in enumerate(self.views):
            n = tv.spec.n
            w = synth.gen_weights(n, synth.seed_for(seed, 1, i), device, wl.weight_std)
            if keep_w32_samples is not None:
                idx = keep_w32_samples(i, n)
                if idx is not None:
                    self.w32_samples[i] = (idx, w[idx].cpu())
            mpo.mpo_split(w, self.hi[tv.off:], self.res[self.res_off[i]:], n, fmt=self.fmt, res_bits=res_bits,
                          round=round, seed=rng_seed, tensor_id=i, res_packed=res_packed)
            del w
        torch.cuda.synchronize(device)
        self.plan = mpo.Plan([mpo.Tensor(self.hi[tv.off:], self.res[self.res_off[i]:], self.grad[tv.goff:],
                                         self.m[tv.off:], self.v[tv.off:], tv.spec.n, tv.spec.layer, res_bits,
                                         res_packed)
                              for i, tv in enumerate(self.views)], small_layer_params=small_layer_params)
        self.layers_backward = wl.layers_backward
        self.by_layer: Dict[int, List[int]] = {}
        for i, tv in enumerate(self.views):
            self.by_layer.setdefault(tv.spec.layer, []).append(i)

    @property
    def resident_bytes(self) -> int:
        return self.total * 10 + self.res.numel() * self.res.element_size() + self.grad_len * 2

    def adam_cfg(self) -> mpo.AdamCfg:
        wl = self.wl
        return mpo.AdamCfg(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=wl.weight_decay,
                           decoupled_wd=(wl.optimizer == "adamw"), loss_scale=wl.loss_scale,
                           weight_fmt=self.fmt, grad_fmt=self.fmt, round=self.round, seed=self.rng_seed)

    def sgd_cfg(self) -> mpo.SgdCfg:
        wl = self.wl
        return mpo.SgdCfg(lr=1e-2, momentum=0.9, weight_decay=wl.weight_decay, loss_scale=wl.loss_scale,
                          weight_fmt=self.fmt, grad_fmt=self.fmt, round=self.round, seed=self.rng_seed)

    def fill_grads(self, tensor_ids, step: int):
        """Stand-in for backward: fresh seeded gradients for these tensors, written into the buffer."""
        wl = self.wl
        for i in tensor_ids:
            tv = self.views[i]
            synth.gen_grads(tv.spec.n, synth.seed_for(self.seed, 2, i, step), self.device, wl.grad_std, wl.fmt,
                            wl.loss_scale, out=self.grad[tv.goff:])

    def step(self, step: int, cfg=None, stream=None, fresh_grads: bool = False, before_layer=None, streams=None) -> int:
        """One optimizer step over the whole model.  Per-layer workloads: one mpo_step_layer per
        layer in backward order; otherwise one mpo_adam_step.  Returns the number of launches.
        `before_layer(layer, tensor_ids)` runs after that layer's gradients are in the buffer."""
        assert not (streams and fresh_grads), "gradients are generated on one stream"
        cfg = cfg or self.adam_cfg()
        if not self.wl.per_layer:
            if fresh_grads:
                self.fill_grads(range(len(self.views)), step)
            if before_layer:
                before_layer(None, list(range(len(self.views))))
            if isinstance(cfg, mpo.SgdCfg):
                mpo.mpo_sgd_step(self.plan, cfg, step, stream=stream)
            else:
                mpo.mpo_adam_step(self.plan, cfg, step, stream=stream)
            return 1
        for k, layer in enumerate(self.layers_backward):
            ids = self.by_layer[layer]
            if fresh_grads:
                self.fill_grads(ids, step)
            if before_layer:
                before_layer(layer, ids)
            # `streams`: the layers' steps go round a set of streams (layers are independent of each other), so that
            # one launch fills the GPU while the one before it drains; the caller orders the streams around the step
            mpo.mpo_step_layer(self.plan, layer, cfg, step, stream=streams[k % len(streams)] if streams else stream)
        return len(self.layers_backward)

    def close(self):
        self.plan.destroy()
