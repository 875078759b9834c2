"""Seeded synthetic workloads: tensor lists shaped like the paper's models, and
weight / gradient generators.

This module holds none of the method's arithmetic (no split, merge or update):
it only names shapes and draws random numbers with torch's seeded generators
and library casts.  Both the GPU path and the CPU oracle are fed the bytes it
produces.

The paper trains ResNet-18, T5/BERT, DLRM and DCGAN on public datasets
(Section 4, appendix); those are not reproduced.  The optimizer step does not
depend on the data beyond the value distributions of weights and gradients, so
parameter lists of the same shape with normal weights (std 0.02) and normal
gradients stand in for them.
"""
import math
from dataclasses import dataclass
from typing import List

import numpy as np
import torch


@dataclass(frozen=True)
class Spec:
    name: str
    n: int
    layer: int


@dataclass(frozen=True)
class Workload:
    key: str
    description: str
    tensors: List[Spec]
    weight_std: float
    grad_std: float
    fmt: str            # "bf16" or "fp16": format of hi and of grad
    loss_scale: float
    optimizer: str      # "adam" | "adamw"
    weight_decay: float
    steps: int
    per_layer: bool     # stepped layer by layer in reverse order (fused into backward)

    @property
    def num_params(self) -> int:
        return sum(t.n for t in self.tensors)

    @property
    def layers_backward(self) -> List[int]:
        """Layer ids in the order their gradients appear in a backward pass."""
        return sorted({t.layer for t in self.tensors}, reverse=True)


def _single() -> List[Spec]:
    return [Spec("w", 1 << 20, 0)]


def _resnet50_like(seed: int = 50) -> List[Spec]:
    """161 tensors, sizes log-uniform in [64, 2.4M], rescaled to 25.6M in total; odd lengths on purpose."""
    rng = np.random.default_rng(seed)
    s = np.exp(rng.uniform(math.log(64.0), math.log(2.4e6), size=161))
    sizes = np.maximum(1, np.rint(s * (25.6e6 / s.sum()))).astype(np.int64)
    sizes[-1] += 25_600_000 - int(sizes.sum())
    assert sizes.min() >= 1 and int(sizes.sum()) == 25_600_000
    return [Spec("t%03d" % i, int(n), i // 3) for i, n in enumerate(sizes)]


def _gpt2_medium() -> List[Spec]:
    h, L, vocab, ctx = 1024, 24, 50257, 1024
    out = [Spec("wte", vocab * h, 0), Spec("wpe", ctx * h, 0)]
    for i in range(L):
        ly = i + 1
        p = "h%d." % i
        out += [Spec(p + "ln_1.w", h, ly), Spec(p + "ln_1.b", h, ly),
                Spec(p + "attn.qkv.w", h * 3 * h, ly), Spec(p + "attn.qkv.b", 3 * h, ly),
                Spec(p + "attn.proj.w", h * h, ly), Spec(p + "attn.proj.b", h, ly),
                Spec(p + "ln_2.w", h, ly), Spec(p + "ln_2.b", h, ly),
                Spec(p + "mlp.fc.w", h * 4 * h, ly), Spec(p + "mlp.fc.b", 4 * h, ly),
                Spec(p + "mlp.proj.w", 4 * h * h, ly), Spec(p + "mlp.proj.b", h, ly)]
    out += [Spec("ln_f.w", h, L + 1), Spec("ln_f.b", h, L + 1)]
    return out


def _llama(h: int, inter: int, L: int, vocab: int) -> List[Spec]:
    out = [Spec("embed", vocab * h, 0)]
    for i in range(L):
        ly = i + 1
        p = "l%d." % i
        out += [Spec(p + "attn_norm", h, ly),
                Spec(p + "q", h * h, ly), Spec(p + "k", h * h, ly), Spec(p + "v", h * h, ly), Spec(p + "o", h * h, ly),
                Spec(p + "mlp_norm", h, ly),
                Spec(p + "gate", h * inter, ly), Spec(p + "up", h * inter, ly), Spec(p + "down", inter * h, ly)]
    out += [Spec("norm", h, L + 1), Spec("lm_head", vocab * h, L + 2)]
    return out


def workload(key: str) -> Workload:
    if key == "c0":
        return Workload("c0", "single tensor, 1,048,576 params", _single(), 0.02, 1e-3, "bf16", 1.0,
                        "adam", 0.0, 10, False)
    if key == "c1":
        return Workload("c1", "ResNet-50-like list, 161 tensors, 25.6M params", _resnet50_like(), 0.02, 1e-3,
                        "bf16", 1.0, "adamw", 1e-4, 100, False)
    if key == "c2":
        return Workload("c2", "GPT-2-medium-shaped list, 292 tensors, 354.8M params", _gpt2_medium(), 0.02, 1e-4,
                        "bf16", 1.0, "adam", 0.0, 20, False)
    if key == "c3":
        return Workload("c3", "Llama-7B-shaped list, 291 tensors, 6.74B params, stepped per layer in backward order",
                        _llama(4096, 11008, 32, 32000), 0.02, 1e-4, "bf16", 1.0, "adam", 0.0, 5, True)
    if key == "c4":
        return Workload("c4", "Llama-13B-shaped list, 363 tensors, 13.0B params, fp16 + loss scale 1024, per layer",
                        _llama(5120, 13824, 40, 32000), 0.02, 1e-4, "fp16", 1024.0, "adam", 0.0, 3, True)
    raise KeyError(key)


# ---- random values ----------------------------------------------------------

def generator(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def gen_weights(n: int, seed: int, device="cpu", std: float = 0.02) -> torch.Tensor:
    """fp32 weights ~ N(0, std^2)."""
    w = torch.empty(n, dtype=torch.float32, device=device)
    w.normal_(0.0, std, generator=generator(seed, device))
    return w


def gen_grads(n: int, seed: int, device="cpu", std: float = 1e-3, fmt: str = "bf16",
              loss_scale: float = 1.0, out: torch.Tensor = None) -> torch.Tensor:
    """16-bit gradients: fp32 ~ N(0, std^2) times loss_scale, cast to `fmt` by the library's
    round-to-nearest cast.  Returned (or written into `out`) as a tensor of that dtype."""
    dtype = torch.bfloat16 if fmt == "bf16" else torch.float16
    g32 = torch.empty(n, dtype=torch.float32, device=device)
    g32.normal_(0.0, std * loss_scale, generator=generator(seed, device))
    if out is None:
        return g32.to(dtype)
    out[:n].copy_(g32)
    return out[:n]


def bits16(t: torch.Tensor) -> np.ndarray:
    """Bit patterns of a bf16 / fp16 / int16 tensor as a host uint16 array."""
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16).copy()


def seed_for(base: int, *ids: int) -> int:
    """A distinct deterministic seed per (tensor, step, ...)."""
    s = base & 0xFFFFFFFF
    for i in ids:
        s = (s * 1000003 + 0x9E3779B1 + int(i)) & 0x7FFFFFFFFFFFFFFF
    return s
