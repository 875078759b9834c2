"""The optimizer step fused into PyTorch's backward pass (arXiv 2309.12381, Section 3.2).

Each parameter's step runs in a post-accumulate-grad hook, as soon as autograd has produced
that parameter's gradient, and the gradient is released right there: no gradient outlives
the backward of its own layer.  The 16-bit parameter tensor of the model IS the `hi` array of
the split weight (the library updates it in place); the extra bits and the moments are
optimizer state (Section 3.1).  Clipping and loss scaling happen inside the step (Section 4.1).

PyTorch provides memory, streams and autograd; every arithmetic step is `mpo_step_layer`.
"""
from typing import Callable, Iterable, Optional, Sequence

import torch

from . import binding as mpo
from . import placement

_FMT = {torch.bfloat16: mpo.MPO_BF16, torch.float16: mpo.MPO_FP16}


def _round_up(x: int, k: int) -> int:
    return (x + k - 1) // k * k


class FusedBackwardOptimizer:
    """Split-precision Adam / SGD whose step runs inside backward.

    params      bf16 or fp16 CUDA parameters (all of one dtype), contiguous.
    cfg         mpo.AdamCfg or mpo.SgdCfg; its weight_fmt / grad_fmt are set from the dtype.
    res_bits    extra bits kept per weight (0 = all); with res_packed the bits stored per weight.
    res_packed  store the extra bits in packed planes (Section 3.1, Figure 1) instead of slots.
    init_fp32   optional fp32 tensors to start from (else the 16-bit values, residual 0).
    fused       True: step in the hook and free the gradient (Section 3.2).  False: keep gradients
                and step them all in `step()`, the classical schedule, for comparison.
    observer    optional callable(index, grad) invoked just before a parameter is stepped.
    overlap     run the steps on a stream of their own, so that a layer's (memory-bound) step runs
                while backward computes the layers below it; each step waits for everything
                backward had enqueued when its gradient arrived, and `start_step()` makes the
                next forward wait for the last steps.  Results are the same; a gradient lives
                until its step has run instead of until it is enqueued.  (Measured on MI355X with
                2.4 B parameters: 29.4 against 29.5 ms per iteration; both the step and the matrix
                products of backward fill every compute unit, so they take turns anyway.)

    bucket_params  consecutive parameters are grouped into buckets of at least this many elements (at most 64 parameters
                each); a bucket is stepped in ONE launch when the last of its gradients has arrived, and its gradients
                are released then.  None (default): 2^16, which only makes a small parameter (a norm weight, a bias)
                wait for the next large one: a launch over a few thousand elements is all latency, and half of a
                transformer's launches are of that kind.  0: strictly one launch per parameter, as the paper steps.
                Larger values (say the size of a block) give fewer, larger launches, which run closer to the memory
                system's rate (a launch over one matrix spends 2-3 % of its time filling and draining the GPU); the
                price is that one bucket's gradients, not one parameter's, are alive at a time.  A bucket whose gradients
                do not all arrive in a backward is stepped for those that did by `start_step()` /
                `synchronize_buckets()`, parameter by parameter.
    place       divide the optimizer state between two regions of the device memory (placement.py): `m` is
                allocated first, next to the model's weights, and `res`, `v` where the bandwidth probe sees
                the gain of a second region relative to the largest parameter and `m`.  Only models with a
                parameter of at least 2^26 elements and 2e8 parameters in all are placed; the report is in
                `self.placement`.  The search holds up to `max_transient_bytes` (default: half of the free
                memory) beyond the state while it runs, so construct the optimizer before activations exist.

    Call `start_step()` before every backward: all parameters stepped during one backward share
    the step count.  With `overlap`, call `synchronize()` before reading parameters or state from
    another stream than the one `start_step()` is called on.
    """

    def __init__(self, params: Iterable[torch.nn.Parameter], cfg, res_bits: int = 0,
                 init_fp32: Optional[Sequence[torch.Tensor]] = None, fused: bool = True,
                 observer: Optional[Callable] = None, res_packed: bool = False, overlap: bool = False,
                 place: bool = True, max_transient_bytes: Optional[int] = None, bucket_params: Optional[int] = None):
        self.params = [p for p in params if p.requires_grad]
        if not self.params:
            raise ValueError("no parameters")
        dtype = self.params[0].dtype
        if dtype not in _FMT:
            raise TypeError("parameters must be bfloat16 or float16")
        for p in self.params:
            if p.dtype != dtype or not p.is_cuda or not p.is_contiguous():
                raise TypeError("parameters must be contiguous CUDA tensors of one 16-bit dtype")
        self.cfg = cfg
        self.cfg.weight_fmt = self.cfg.grad_fmt = _FMT[dtype]
        self.is_adam = isinstance(cfg, mpo.AdamCfg)
        self.res_bits = res_bits
        self.res_packed = res_packed
        self.fused = fused
        self.observer = observer
        self.step_no = 0
        self.side = torch.cuda.Stream(device=self.params[0].device) if (overlap and fused) else None
        dev = self.params[0].device
        offs, total = [], 0
        for p in self.params:
            offs.append(total)
            total += _round_up(p.numel(), 64)       # every parameter's state starts on a 128-byte line
        if res_packed:
            # one byte buffer; each parameter's planes start at a multiple of 16 bytes
            self.res_offs, fill = [], 0
            for p in self.params:
                self.res_offs.append(fill)
                fill += mpo.mpo_res_bytes(p.numel(), res_bits, True)
            res_spec = (fill, torch.uint8)
        else:
            self.res_offs = offs
            res_spec = (total, torch.uint8 if 1 <= res_bits <= 8 else torch.int16)
        # m first: right behind the model's weights in a fresh process, i.e. in their region
        self.m = torch.empty(total, dtype=torch.float32, device=dev)

        def second():
            out = {"res": torch.empty(res_spec[0], dtype=res_spec[1], device=dev)}
            if self.is_adam:
                out["v"] = torch.empty(total, dtype=torch.float32, device=dev)
            return out
        biggest = max(self.params, key=lambda p: p.numel())
        res_bytes = res_spec[0] * (1 if res_spec[1] == torch.uint8 else 2)
        if place and self.is_adam and biggest.numel() >= (1 << 26) and res_bytes >= (1 << 27):
            chosen, self.placement = placement.place_second(biggest.data.view(-1), self.m, second, res_bytes + 4 * total,
                                                            max_transient_bytes=max_transient_bytes, keep_hi=True)
        else:
            chosen = second()
            self.placement = {"split": False, "why": "placement switched off" if not place else
                              "not placed: needs Adam, a parameter of 2^26 elements and 16-bit weights of 2^27 bytes"}
        self.res = chosen["res"].zero_()
        self.m.zero_()
        self.v = chosen["v"].zero_() if self.is_adam else None
        self.offs = offs
        specs = []
        for i, (p, off) in enumerate(zip(self.params, offs)):
            n = p.numel()
            master = init_fp32[i].to(dev, torch.float32).reshape(-1).contiguous() if init_fp32 is not None \
                else p.detach().float().reshape(-1)
            res = self.res[self.res_offs[i]:]
            mpo.mpo_split(master, p.data, res, n, fmt=_FMT[dtype], res_bits=res_bits, round=cfg.round,
                          seed=cfg.seed, tensor_id=i, res_packed=res_packed)
            specs.append(mpo.Tensor(p.data, res, None, self.m[off:],
                                    self.v[off:] if self.is_adam else None, n, i, res_bits, res_packed))
        torch.cuda.synchronize(dev)
        self.plan = mpo.Plan(specs)          # one layer id per parameter: the paper steps per parameter
        # optional buckets: a second plan over the same tensors whose layers are runs of consecutive parameters
        self.bucket_of, self.buckets, self.bucket_plan = None, None, None
        if bucket_params is None:
            bucket_params = 1 << 16
        if bucket_params > 0 and fused:
            self.bucket_of, self.buckets, fill = [], [], 0
            for i, p in enumerate(self.params):
                if not self.buckets or fill >= bucket_params or len(self.buckets[-1]) == mpo.MPO_MAX_LAYER_GRADS:
                    self.buckets.append([])
                    fill = 0
                self.buckets[-1].append(i)
                self.bucket_of.append(len(self.buckets) - 1)
                fill += p.numel()
            self.bucket_plan = mpo.Plan([mpo.Tensor(t.hi, t.res, None, t.m, t.v, t.n, self.bucket_of[i], res_bits, res_packed)
                                         for i, t in enumerate(specs)])
            self._pending = [dict() for _ in self.buckets]      # bucket -> {parameter index: gradient}
        self._index = {id(p): i for i, p in enumerate(self.params)}
        self._handles = []
        if fused:
            for p in self.params:
                self._handles.append(p.register_post_accumulate_grad_hook(self._on_grad))

    def start_step(self):
        self.synchronize_buckets()
        self.synchronize()
        self.step_no += 1

    def synchronize_buckets(self):
        """Step, parameter by parameter, whatever gradients are still waiting in incomplete buckets (parameters
        that took no part in the last backward leave their bucket incomplete)."""
        if self.buckets is None:
            return
        for pending in self._pending:
            for i, g in sorted(pending.items()):
                self._launch(self.plan, i, [g])
            pending.clear()

    def synchronize(self):
        """Make the current stream wait for the steps enqueued so far (a no-op without `overlap`)."""
        if self.side is not None:
            torch.cuda.current_stream(self.params[0].device).wait_stream(self.side)

    def _launch(self, plan, layer: int, grads):
        stream = torch.cuda.current_stream(self.params[0].device)
        if self.side is not None:
            # after everything backward has enqueued so far (the kernels that read these weights and
            # wrote these gradients among it), and keep the gradients' memory until the step has run
            self.side.wait_stream(stream)
            for g in grads:
                g.record_stream(self.side)
            stream = self.side
        mpo.mpo_step_layer(plan, layer, self.cfg, self.step_no, grads=grads, stream=stream)

    def _step_param(self, i: int, p: torch.nn.Parameter):
        g = p.grad
        if g.dtype != p.dtype:
            raise TypeError("gradient dtype differs from the parameter's")
        if not g.is_contiguous():
            g = g.contiguous()
        if self.observer is not None:
            self.observer(i, g)
        if self.buckets is not None:
            b = self.bucket_of[i]
            pending = self._pending[b]
            pending[i] = g
            if len(pending) == len(self.buckets[b]):        # the bucket's last gradient: one launch for all of them
                self._launch(self.bucket_plan, b, [pending[k] for k in self.buckets[b]])
                pending.clear()
            return
        self._launch(self.plan, i, [g])

    def _on_grad(self, p: torch.nn.Parameter):
        if self.step_no == 0:
            raise RuntimeError("call start_step() before backward")
        self._step_param(self._index[id(p)], p)
        p.grad = None                       # the gradient is consumed: never kept (Section 3.2)

    def step(self):
        """Classical schedule (fused=False): step every parameter after backward has finished."""
        if self.fused:
            raise RuntimeError("steps already ran inside backward")
        for i, p in enumerate(self.params):
            if p.grad is not None:
                self._step_param(i, p)
                p.grad = None

    def master_fp32(self, i: int) -> torch.Tensor:
        """The fp32 value of parameter i held by (hi, res)."""
        self.synchronize_buckets()
        self.synchronize()
        p = self.params[i]
        out = torch.empty(p.numel(), dtype=torch.float32, device=p.device)
        mpo.mpo_merge(p.data, self.res[self.res_offs[i]:], out, p.numel(), fmt=_FMT[p.dtype], res_bits=self.res_bits,
                      round=self.cfg.round, res_packed=self.res_packed)
        return out.view_as(p)

    def state_of(self, i: int):
        self.synchronize_buckets()
        self.synchronize()
        n, off, roff = self.params[i].numel(), self.offs[i], self.res_offs[i]
        rlen = mpo.mpo_res_bytes(n, self.res_bits, True) if self.res_packed else n
        return self.res[roff:roff + rlen], self.m[off:off + n], (self.v[off:off + n] if self.is_adam else None)

    def close(self):
        self.synchronize_buckets()
        self.synchronize()
        for h in self._handles:
            h.remove()
        self._handles = []
        self.plan.destroy()
        if self.bucket_plan is not None:
            self.bucket_plan.destroy()
