"""Pins for the oracle's Adam and SGD steps (arXiv 2309.12381, Section 3.1:
the classic optimizers, run on a 16-bit weight plus its extra bits, as precise
as an fp32 training; Section 4.1: gradient scaling happens inside the step).

Pins used, each against something other than the oracle itself:
  * torch.optim.Adam / AdamW / SGD on fp32 master weights (library routine);
  * an ordinary fp32-master optimizer whose 16-bit copy is the truncation of
    the master (Section 3.1: the stored value is as precise as in fp32 training), in numpy float32;
  * an exact-rational model of binary32 arithmetic (tests/exact_fp32.py);
  * closed forms in real arithmetic: first Adam step, constant-gradient Adam,
    momentum as a geometric series, decay-only steps;
  * invariants: power-of-two loss scale, zero gradient, residual carries
    updates the 16-bit weight alone would lose.
`pins_*` functions take the oracle as an argument so that
tests/test_oracle_pins_bite.py can run them against deliberately broken builds.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import exact_fp32 as ex


# ---- helpers ---------------------------------------------------------------

def to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns by the library's round-to-nearest cast."""
    return torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()


def to_fp16_bits(x32: np.ndarray) -> np.ndarray:
    return x32.astype(np.float16).view(np.uint16).copy()


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).float().numpy()


def fp16_to_f32(bits: np.ndarray) -> np.ndarray:
    return bits.view(np.float16).astype(np.float32)


def make_state(rng, n, wstd=0.02, gstd=1e-3):
    w = (rng.standard_normal(n) * wstd).astype(np.float32)
    g = (rng.standard_normal(n) * gstd).astype(np.float32)
    return w, g


def ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """Distance in fp32 steps between same-sign-or-near-zero patterns."""
    def key(b):
        b = b.astype(np.int64)
        return np.where(b & 0x80000000, -(b & 0x7FFFFFFF), b)
    return np.abs(key(a_bits) - key(b_bits))


# ---- pin: torch.optim on fp32 masters --------------------------------------

def _torch_run(opt_name, w0, grads, **kw):
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    cls = {"adam": torch.optim.Adam, "adamw": torch.optim.AdamW, "sgd": torch.optim.SGD}[opt_name]
    opt = cls([p], foreach=False, **kw)
    for g in grads:
        p.grad = torch.from_numpy(g.copy())
        opt.step()
    return p.detach().numpy().copy()


def pins_torch_optim(ref):
    rng = np.random.default_rng(7)
    n, steps = 4096, 25
    w0, _ = make_state(rng, n)
    gbits = [to_bf16_bits(make_state(rng, n)[1]) for _ in range(steps)]
    g32 = [bf16_to_f32(b) for b in gbits]
    cases = [
        ("adam", dict(lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.0),
         ref.AdamCfg(lr=1e-3)),
        ("adam", dict(lr=3e-4, betas=(0.64, 0.95), eps=1e-6, weight_decay=0.1),
         ref.AdamCfg(lr=3e-4, beta1=0.64, beta2=0.95, eps=1e-6, weight_decay=0.1, decoupled_wd=False)),
        ("adamw", dict(lr=2e-3, betas=(0.9, 0.99), eps=1e-8, weight_decay=0.05),
         ref.AdamCfg(lr=2e-3, beta2=0.99, weight_decay=0.05, decoupled_wd=True)),
    ]
    for name, kw, cfg in cases:
        want = _torch_run(name, w0, g32, **kw)
        hi, res = ref.split(w0)
        m = np.zeros(n, np.float32)
        v = np.zeros(n, np.float32)
        for t, gb in enumerate(gbits, 1):
            ref.adam_step(hi, res, gb, m, v, cfg, t)
        got = ref.merge(hi, res)
        # total movement is about steps*lr; both sides round differently per op, so allow
        # 2e-5 of the movement plus a few ulp of the weight; a wrong formula is off by
        # orders of magnitude more (see test_oracle_pins_bite.py)
        tol = 2e-5 * steps * cfg.lr + steps * np.spacing(np.maximum(np.abs(want), np.abs(w0)))
        assert np.all(np.abs(got.astype(np.float64) - want) <= tol), (name, kw)
    sgd_cases = [
        (dict(lr=1e-2, momentum=0.9, weight_decay=0.0), ref.SgdCfg(lr=1e-2, momentum=0.9)),
        (dict(lr=0.3, momentum=0.9, weight_decay=2e-4), ref.SgdCfg(lr=0.3, momentum=0.9, weight_decay=2e-4)),
        (dict(lr=0.1, momentum=0.0, weight_decay=0.0), ref.SgdCfg(lr=0.1, momentum=0.0)),
    ]
    for kw, cfg in sgd_cases:
        want = _torch_run("sgd", w0, g32, **kw)
        hi, res = ref.split(w0)
        buf = np.zeros(n, np.float32)
        for t, gb in enumerate(gbits, 1):
            ref.sgd_step(hi, res, gb, buf, cfg, t)
        got = ref.merge(hi, res)
        move = np.abs(want - w0)
        # each side rounds the weight once per step: at most one ulp apart per step
        tol = 1e-5 * move + steps * np.spacing(np.maximum(np.abs(want), np.abs(w0)))
        assert np.all(np.abs(got.astype(np.float64) - want) <= tol), kw


def test_matches_torch_optim(ref):
    pins_torch_optim(ref)


# ---- pin: ordinary fp32-master optimizer, 16-bit copy = truncated master ---

def _master_adam(w, g, m, v, lr, b1, b2, eps, wd, decoupled, t, inv_scale):
    """Textbook Adam on an fp32 master, numpy float32, one rounded op at a time."""
    f = np.float32
    g = g * f(inv_scale)
    if wd != 0.0:
        if decoupled:
            w = w * f(1.0 - lr * wd)
        else:
            g = g + f(wd) * w
    m[:] = f(b1) * m + f(1.0 - b1) * g
    v[:] = f(b2) * v + (f(1.0 - b2) * g) * g
    denom = np.sqrt(v) / f(np.sqrt(1.0 - b2 ** t)) + f(eps)
    return w - f(lr / (1.0 - b1 ** t)) * (m / denom)


def pins_fp32_master_equivalence(ref):
    rng = np.random.default_rng(11)
    n = 4096
    for fmt, tobits, tof32, scale in ((ref.BF16, to_bf16_bits, bf16_to_f32, 1.0),
                                      (ref.FP16, to_fp16_bits, fp16_to_f32, 1024.0)):
        w0, _ = make_state(rng, n)
        # adversarial values: zeros, tiny, exact powers of two, values next to a 16-bit boundary
        w0[:8] = [0.0, -0.0, 1.0, -1.0, 0.99999994, 1.0000001, 6.1035156e-05, -2.5e-4]
        crossed = 0
        if fmt == ref.FP16:
            # start inside the range where the fp16 pair is exact
            w0 = np.where(np.abs(w0) < 2.0 ** -13, np.float32(2.0 ** -13), w0).astype(np.float32)
        cfg = ref.AdamCfg(lr=1e-3, weight_decay=1e-2, decoupled_wd=True, loss_scale=scale,
                          weight_fmt=fmt, grad_fmt=fmt)
        hi, res = ref.split(w0, fmt)
        master = ref.merge(hi, res, fmt).copy()
        assert np.array_equal(master.view(np.uint32), w0.view(np.uint32))
        m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
        mm = np.zeros(n, np.float32); mv = np.zeros(n, np.float32)
        for t in range(1, 41):
            gb = tobits((make_state(rng, n)[1] * np.float32(scale)).astype(np.float32))
            ref.adam_step(hi, res, gb, m, v, cfg, t)
            master = _master_adam(master, tof32(gb), mm, mv, 1e-3, 0.9, 0.999, 1e-8, 1e-2, True, t,
                                  1.0 / scale)
            got = ref.merge(hi, res, fmt)
            if fmt == ref.FP16:
                # below 2^-14 the fp16 pair holds multiples of 2^-37 only: the master is cut
                # toward zero to that grid (exact in binary64); weights do cross zero here
                tiny = np.abs(master) < np.float32(2.0 ** -14)
                crossed += int(tiny.sum())
                cut = (np.trunc(master.astype(np.float64) * 2.0 ** 37) / 2.0 ** 37).astype(np.float32)
                master = np.where(tiny, cut, master)
            assert np.array_equal(got.view(np.uint32), master.view(np.uint32)), (fmt, t)
            assert np.array_equal(m.view(np.uint32), mm.view(np.uint32)), (fmt, t)
            assert np.array_equal(v.view(np.uint32), mv.view(np.uint32)), (fmt, t)
            # the 16-bit weight is the master rounded toward zero
            h16 = tof32(hi)
            assert np.all(np.abs(h16) <= np.abs(master)) and np.all(np.signbit(h16) == np.signbit(master))
            ulp16 = np.spacing(np.abs(h16).astype(np.float16 if fmt == ref.FP16 else np.float32))
            if fmt == ref.BF16:
                ulp16 = ulp16.astype(np.float64) * 65536.0
            assert np.all(np.abs(master).astype(np.float64) - np.abs(h16) < ulp16.astype(np.float64))
        if fmt == ref.FP16:
            assert crossed > 20            # the subnormal branch was exercised


def test_equals_fp32_master_training(ref):
    pins_fp32_master_equivalence(ref)


def pins_fp32_master_sgd(ref):
    rng = np.random.default_rng(13)
    n = 2048
    f = np.float32
    w0, _ = make_state(rng, n)
    for lr, mu, wd in ((1e-2, 0.9, 0.0), (0.3, 0.9, 2e-4), (0.1, 0.0, 1e-3)):
        cfg = ref.SgdCfg(lr=lr, momentum=mu, weight_decay=wd)
        hi, res = ref.split(w0)
        master = w0.copy()
        buf = np.zeros(n, f); mb = np.zeros(n, f)
        for t in range(1, 31):
            gb = to_bf16_bits(make_state(rng, n)[1])
            ref.sgd_step(hi, res, gb, buf, cfg, t)
            g = bf16_to_f32(gb)
            if wd:
                g = g + f(wd) * master
            if mu:
                mb = f(mu) * mb + g
                upd = mb
            else:
                upd = g
            master = master - f(lr) * upd
            assert np.array_equal(ref.merge(hi, res).view(np.uint32), master.view(np.uint32)), (lr, mu, wd, t)
            if mu:
                assert np.array_equal(buf.view(np.uint32), mb.view(np.uint32))


def test_sgd_equals_fp32_master_training(ref):
    pins_fp32_master_sgd(ref)


# ---- pin: exact-rational binary32 model ------------------------------------

def _exact_adam_element(w, g, m, v, cfg, t):
    F = Fraction
    rn = ex.rn
    B1 = rn(F(np.float32(cfg.beta1).item())); B2 = rn(F(np.float32(cfg.beta2).item()))
    O1 = rn(1 - F(cfg.beta1)); O2 = rn(1 - F(cfg.beta2))
    # lr/(1-beta1^t) and sqrt(1-beta2^t): exact rationals rounded once (the oracle goes
    # through binary64 first; for these magnitudes the two roundings agree, checked below)
    SS = rn(F(cfg.lr) / (1 - F(cfg.beta1) ** t))
    SQ = ex.sqrt_rn(1 - F(cfg.beta2) ** t)
    EPS = rn(F(cfg.eps)); IS = rn(1 / F(cfg.loss_scale))
    g = rn(g * IS)
    if cfg.weight_decay != 0.0:
        if cfg.decoupled_wd:
            w = rn(w * rn(1 - F(cfg.lr) * F(cfg.weight_decay)))
        else:
            g = rn(g + rn(rn(F(cfg.weight_decay)) * w))
    m1 = rn(rn(B1 * m) + rn(O1 * g))
    v1 = rn(rn(B2 * v) + rn(rn(O2 * g) * g))
    d = rn(rn(ex.sqrt_rn(v1) / SQ) + EPS)
    w1 = rn(w - rn(SS * rn(m1 / d)))
    return w1, m1, v1


def pins_exact_rational_adam(ref):
    rng = np.random.default_rng(17)
    n = 96
    for cfg, t in ((ref.AdamCfg(), 1), (ref.AdamCfg(weight_decay=1e-4), 3),
                   (ref.AdamCfg(lr=7e-5, beta1=0.64, weight_decay=0.01, decoupled_wd=False), 7),
                   (ref.AdamCfg(loss_scale=1024.0), 12)):
        w0, g0 = make_state(rng, n)
        g0 = g0 * np.float32(cfg.loss_scale)
        g0[:6] = [0.0, 1e-30, -1e-22, 3e-39, 1.0, -6e4]          # denormal products, big values
        w0[:3] = [0.0, 1e-38, -3e-39]
        gb = to_bf16_bits(g0)
        m0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        v0 = (rng.standard_normal(n) * 1e-3).astype(np.float32) ** 2
        m0[:2] = 0; v0[:2] = 0
        hi, res = ref.split(w0)
        m = m0.copy(); v = v0.copy()
        ref.adam_step(hi, res, gb, m, v, cfg, t)
        got = ref.merge(hi, res)
        g32 = bf16_to_f32(gb)
        for i in range(n):
            w1, m1, v1 = _exact_adam_element(Fraction(float(w0[i])), Fraction(float(g32[i])),
                                             Fraction(float(m0[i])), Fraction(float(v0[i])), cfg, t)
            assert Fraction(float(got[i])) == w1, (cfg, t, i)
            assert Fraction(float(m[i])) == m1 and Fraction(float(v[i])) == v1, (cfg, t, i)


def test_exact_rational_adam(ref):
    pins_exact_rational_adam(ref)


def pins_exact_rational_sgd(ref):
    rng = np.random.default_rng(19)
    n = 96
    F = Fraction
    rn = ex.rn
    for cfg in (ref.SgdCfg(), ref.SgdCfg(lr=0.3, weight_decay=2e-4), ref.SgdCfg(lr=0.1, momentum=0.0),
                ref.SgdCfg(loss_scale=256.0)):
        w0, g0 = make_state(rng, n)
        gb = to_bf16_bits(g0 * np.float32(cfg.loss_scale))
        b0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        hi, res = ref.split(w0)
        b = b0.copy()
        ref.sgd_step(hi, res, gb, b, cfg, 5)
        got = ref.merge(hi, res)
        g32 = bf16_to_f32(gb)
        for i in range(n):
            g = rn(F(float(g32[i])) * rn(1 / F(cfg.loss_scale)))
            w = F(float(w0[i]))
            if cfg.weight_decay:
                g = rn(g + rn(rn(F(cfg.weight_decay)) * w))
            if cfg.momentum:
                nb = rn(rn(rn(F(cfg.momentum)) * F(float(b0[i]))) + g)
                assert F(float(b[i])) == nb
            else:
                nb = g
                assert b[i] == b0[i]
            assert F(float(got[i])) == rn(w - rn(rn(F(cfg.lr)) * nb)), (cfg, i)


def test_exact_rational_sgd(ref):
    pins_exact_rational_sgd(ref)


# ---- pin: closed forms in real arithmetic ----------------------------------

def pins_adam_first_step_closed_form(ref):
    """From m = v = 0 the bias-corrected moments are g and g^2, so the first step moves
    every weight by -lr * g / (|g| + eps), whatever beta1 and beta2 are."""
    rng = np.random.default_rng(23)
    n = 2048
    for b1, b2, lr, eps in ((0.9, 0.999, 1e-3, 1e-8), (0.64, 0.95, 7e-5, 1e-6), (0.5, 0.9, 1e-2, 1e-3)):
        w0, g0 = make_state(rng, n)
        gb = to_bf16_bits(g0)
        g = bf16_to_f32(gb).astype(np.float64)
        hi, res = ref.split(w0)
        m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
        ref.adam_step(hi, res, gb, m, v, ref.AdamCfg(lr=lr, beta1=b1, beta2=b2, eps=eps), 1)
        want = w0.astype(np.float64) - lr * g / (np.abs(g) + eps)
        got = ref.merge(hi, res).astype(np.float64)
        assert np.all(np.abs(got - want) <= 1e-6 * lr + np.spacing(np.abs(w0)).astype(np.float64))
        assert np.allclose(m, (1 - b1) * g, rtol=1e-6, atol=0)
        assert np.allclose(v, (1 - b2) * g * g, rtol=1e-6, atol=0)


def test_adam_first_step_closed_form(ref):
    pins_adam_first_step_closed_form(ref)


def pins_adam_constant_gradient(ref):
    """With the same gradient every step, bias correction makes m_hat = g and v_hat = g^2
    at every t, so after T steps w = w0 - T * lr * g / (|g| + eps).  Sensitive to how the
    step count enters both corrections."""
    rng = np.random.default_rng(29)
    n, T, lr, eps = 1024, 60, 1e-3, 1e-8
    w0, g0 = make_state(rng, n)
    gb = to_bf16_bits(g0)
    g = bf16_to_f32(gb).astype(np.float64)
    hi, res = ref.split(w0)
    m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
    for t in range(1, T + 1):
        ref.adam_step(hi, res, gb, m, v, ref.AdamCfg(lr=lr, eps=eps), t)
        want = w0.astype(np.float64) - t * lr * g / (np.abs(g) + eps)
        got = ref.merge(hi, res).astype(np.float64)
        # fp32 rounding in m, v and w: about 1e-6 of the movement; a wrong correction is off by O(1)
        assert np.all(np.abs(got - want) <= 1e-5 * t * lr + 2e-7 * np.abs(want)), t
    assert np.allclose(m, (1 - 0.9 ** T) * g, rtol=2e-6, atol=0)
    assert np.allclose(v, (1 - 0.999 ** T) * g * g, rtol=2e-5, atol=0)


def test_adam_constant_gradient(ref):
    pins_adam_constant_gradient(ref)


def pins_sgd_geometric_series(ref):
    """Constant g: buf_n = g (1 - mu^n)/(1 - mu), w_n = w0 - lr * sum_k buf_k."""
    rng = np.random.default_rng(31)
    n, T, lr, mu = 1024, 40, 1e-2, 0.9
    w0, g0 = make_state(rng, n)
    gb = to_bf16_bits(g0)
    g = bf16_to_f32(gb).astype(np.float64)
    hi, res = ref.split(w0)
    buf = np.zeros(n, np.float32)
    ref.sgd_step(hi, res, gb, buf, ref.SgdCfg(lr=lr, momentum=mu), 1)
    assert np.array_equal(buf.view(np.uint32), bf16_to_f32(gb).view(np.uint32))   # first step: buf = g
    total = g.copy()
    for t in range(2, T + 1):
        ref.sgd_step(hi, res, gb, buf, ref.SgdCfg(lr=lr, momentum=mu), t)
        bn = g * (1 - mu ** t) / (1 - mu)
        total += bn
        assert np.allclose(buf, bn, rtol=1e-5, atol=0), t
    want = w0.astype(np.float64) - lr * total
    # the weight is rounded once per step: at most half an ulp each
    slack = T * np.spacing(np.maximum(np.abs(w0), np.abs(want)).astype(np.float32)).astype(np.float64)
    assert np.all(np.abs(ref.merge(hi, res) - want) <= 1e-5 * np.abs(lr * total) + slack)


def test_sgd_geometric_series(ref):
    pins_sgd_geometric_series(ref)


def pins_decay_only_steps(ref):
    """Zero gradient: AdamW only shrinks the weight by (1 - lr*wd); plain Adam leaves it
    alone and keeps m = v = 0; L2-Adam's first step moves by about lr toward zero;
    SGD with L2 shrinks by (1 - lr*wd)."""
    rng = np.random.default_rng(37)
    n = 512
    w0, _ = make_state(rng, n)
    w0[0] = 0.0
    z = np.zeros(n, np.uint16)
    hi, res = ref.split(w0)
    m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
    ref.adam_step(hi, res, z, m, v, ref.AdamCfg(), 1)
    assert np.array_equal(ref.merge(hi, res).view(np.uint32), w0.view(np.uint32))
    assert not m.any() and not v.any()

    ref.adam_step(hi, res, z, m, v, ref.AdamCfg(lr=1e-2, weight_decay=0.5, decoupled_wd=True), 1)
    assert np.array_equal(ref.merge(hi, res), w0 * np.float32(1 - 1e-2 * 0.5))
    assert not m.any() and not v.any()

    hi, res = ref.split(w0)
    ref.adam_step(hi, res, z, m, v, ref.AdamCfg(lr=1e-3, weight_decay=0.5, decoupled_wd=False), 1)
    g = 0.5 * w0.astype(np.float64)
    want = w0 - 1e-3 * g / (np.abs(g) + 1e-8)
    assert np.allclose(ref.merge(hi, res), want, rtol=1e-5, atol=1e-9)

    hi, res = ref.split(w0)
    ref.sgd_step(hi, res, z, np.zeros(n, np.float32), ref.SgdCfg(lr=0.1, momentum=0.0, weight_decay=0.25), 1)
    assert np.allclose(ref.merge(hi, res), w0.astype(np.float64) * (1 - 0.025), rtol=3e-7, atol=0)


def test_decay_only_steps(ref):
    pins_decay_only_steps(ref)


# ---- pin: invariants ---------------------------------------------------------

def pins_loss_scale_power_of_two(ref):
    """Scaling a 16-bit gradient by 2^k is exact, and so is the un-scaling inside the
    step: the trajectory does not depend on the loss scale (Section 4.1)."""
    rng = np.random.default_rng(41)
    n = 2048
    w0, _ = make_state(rng, n)
    for fmt, tobits in ((ref.BF16, to_bf16_bits), (ref.FP16, to_fp16_bits)):
        g32 = [(rng.standard_normal(n) * 1e-2).astype(np.float32) for _ in range(6)]
        # round to the 16-bit grid first so that multiplying by 1024 stays on it
        g16 = [tobits(g) for g in g32]
        back = bf16_to_f32 if fmt == ref.BF16 else fp16_to_f32
        g16s = [tobits(back(g) * np.float32(1024.0)) for g in g16]
        for a, b in zip(g16, g16s):
            assert np.array_equal(back(b), back(a) * np.float32(1024.0))
        out = []
        for scale, gs in ((1.0, g16), (1024.0, g16s)):
            hi, res = ref.split(w0)
            m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
            for t, g in enumerate(gs, 1):
                ref.adam_step(hi, res, g, m, v, ref.AdamCfg(loss_scale=scale, grad_fmt=fmt), t)
            out.append((hi.copy(), res.copy(), m.copy(), v.copy()))
        for a, b in zip(*out):
            assert np.array_equal(a.view(np.uint8), b.view(np.uint8))
        out = []
        for scale, gs in ((1.0, g16), (1024.0, g16s)):
            hi, res = ref.split(w0)
            buf = np.zeros(n, np.float32)
            for t, g in enumerate(gs, 1):
                ref.sgd_step(hi, res, g, buf, ref.SgdCfg(loss_scale=scale, grad_fmt=fmt), t)
            out.append((hi.copy(), res.copy(), buf.copy()))
        for a, b in zip(*out):
            assert np.array_equal(a.view(np.uint8), b.view(np.uint8))


def test_loss_scale_power_of_two(ref):
    pins_loss_scale_power_of_two(ref)


def pins_residual_carries_small_updates(ref):
    """Section 2 / 3.1: an update below half a bf16 ulp vanishes on a bf16-only weight;
    with the residual it accumulates exactly as in fp32 and hi moves once the sum
    crosses a bf16 step (2^-7 at 1.0)."""
    n = 1
    lr = 2.0 ** -10
    g = np.array([0x3F80], np.uint16)                      # bf16 1.0
    hi, res = ref.split(np.array([1.0], np.float32))
    w32 = np.float32(1.0)
    moved_at = None
    for t in range(1, 17):
        ref.sgd_step(hi, res, g, None, ref.SgdCfg(lr=lr, momentum=0.0), t)
        w32 = np.float32(w32 - np.float32(lr))
        assert ref.merge(hi, res)[0] == w32
        assert ref.merge(hi, res)[0] == np.float32(1.0 - t * lr)   # exact: multiples of 2^-10
        if moved_at is None and hi[0] != 0x3F80:
            moved_at = t
    # below 1.0 the bf16 step is 2^-8: the truncated weight drops at once, then every 4 steps
    assert moved_at == 1 and hi[0] == bf16_rtz_bits(1.0 - 16 * lr)
    # going up from 1.0 (bf16 step 2^-7 = 8 updates): hi stays until the sum crosses it
    hi, res = ref.split(np.array([1.0], np.float32))
    gneg = np.array([0xBF80], np.uint16)
    seen = []
    for t in range(1, 10):
        ref.sgd_step(hi, res, gneg, None, ref.SgdCfg(lr=lr, momentum=0.0), t)
        seen.append(int(hi[0]))
    assert seen[:7] == [0x3F80] * 7 and seen[7] == 0x3F81 and seen[8] == 0x3F81
    # a bf16-only weight with round-to-nearest never moves under the same update
    wb = torch.tensor([1.0], dtype=torch.bfloat16)
    for _ in range(9):
        wb = (wb.float() + lr).to(torch.bfloat16)
    assert float(wb) == 1.0


def bf16_rtz_bits(x: float) -> int:
    b = ex.bits_of(float(np.float32(x)))
    v = ex.decode(b >> 16, 8, 7)
    assert abs(v) <= abs(Fraction(float(np.float32(x))))
    return b >> 16


def test_residual_carries_small_updates(ref):
    pins_residual_carries_small_updates(ref)


def pins_mixed_formats(ref):
    """fp16 weights with bf16 gradients and the other way round give the same fp32
    trajectory as long as the weights stay where the fp16 pair is exact."""
    rng = np.random.default_rng(43)
    n = 1024
    w0 = (0.5 + rng.random(n)).astype(np.float32)              # in [0.5, 1.5): exact in both
    # gradients on the intersection of the two 16-bit grids: 8 significant bits, moderate range
    g = to_bf16_bits((rng.standard_normal(n) * 0.01).astype(np.float32))
    g = np.where(np.abs(bf16_to_f32(g)) < 1e-4, to_bf16_bits(np.full(n, 1e-3, np.float32)), g)
    g_as_fp16 = to_fp16_bits(bf16_to_f32(g))
    assert np.array_equal(fp16_to_f32(g_as_fp16), bf16_to_f32(g))
    outs = []
    for wf, gf, gb in ((ref.BF16, ref.BF16, g), (ref.FP16, ref.BF16, g), (ref.BF16, ref.FP16, g_as_fp16),
                       (ref.FP16, ref.FP16, g_as_fp16)):
        hi, res = ref.split(w0, wf)
        m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
        for t in range(1, 6):
            ref.adam_step(hi, res, gb, m, v, ref.AdamCfg(weight_fmt=wf, grad_fmt=gf), t)
        outs.append(ref.merge(hi, res, wf).view(np.uint32).copy())
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])


def test_mixed_formats(ref):
    pins_mixed_formats(ref)


def test_printed_single_element_values(ref):
    """Single-element values worked out with the exact-rational model (not stored from
    any implementation): Adam step 1 and two SGD steps from the same inputs."""
    cfg = ref.AdamCfg()
    for w, gbits in ((1.0, 0x3A80), (0.1, 0xBA83), (-0.02, 0x3A83)):
        w32 = np.array([w], np.float32)
        hi, res = ref.split(w32)
        m = np.zeros(1, np.float32); v = np.zeros(1, np.float32)
        ref.adam_step(hi, res, np.array([gbits], np.uint16), m, v, cfg, 1)
        g = Fraction(ref.cvt16(gbits))
        w1, m1, v1 = _exact_adam_element(Fraction(float(w32[0])), g, Fraction(0), Fraction(0), cfg, 1)
        assert Fraction(float(ref.merge(hi, res)[0])) == w1
        assert Fraction(float(m[0])) == m1 and Fraction(float(v[0])) == v1
        # real-arithmetic value: w - lr * g / (|g| + eps)
        real = Fraction(float(w32[0])) - Fraction(cfg.lr) * g / (abs(g) + Fraction(cfg.eps))
        assert abs(w1 - real) <= Fraction(float(np.spacing(np.float32(abs(w)))))


@pytest.mark.parametrize("n", [0, 1, 7])
def test_tiny_lengths(ref, n):
    w0 = np.linspace(-1, 1, n).astype(np.float32)
    hi, res = ref.split(w0)
    m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
    ref.adam_step(hi, res, np.zeros(n, np.uint16), m, v, ref.AdamCfg(), 1)
    assert np.array_equal(ref.merge(hi, res), w0)


# ---- keeping only E extra bits (Section 3.1; the paper's fp16+8 / bf16+8) ---------------

def _cut(x, sig_bits, emin):
    a = np.abs(x.astype(np.float64))
    m, e = np.frexp(a)
    e = np.maximum(e, emin + 1)
    ulp = np.ldexp(1.0, e - sig_bits)
    return np.copysign(np.trunc(a / ulp) * ulp, x.astype(np.float64)).astype(np.float32)


def pins_partial_bits_master_equivalence(ref):
    """With E extra bits the weights follow an fp32-master optimizer whose master is cut toward
    zero to 16+E bits after every step (numpy float32, library frexp/trunc for the cut)."""
    rng = np.random.default_rng(47)
    n = 4096
    for fmt, tobits, tof32, sig, emin, scale in ((ref.BF16, to_bf16_bits, bf16_to_f32, 8, -126, 1.0),
                                                 (ref.FP16, to_fp16_bits, fp16_to_f32, 11, -14, 512.0)):
        for E in (8, 4, 12):
            w0 = (0.05 + 0.5 * rng.random(n)).astype(np.float32) * np.where(rng.random(n) < 0.5, -1, 1).astype(np.float32)
            cfg = ref.AdamCfg(lr=1e-3, weight_decay=1e-2, decoupled_wd=True, loss_scale=scale,
                              weight_fmt=fmt, grad_fmt=fmt, res_bits=E)
            hi, res = ref.split(w0, fmt, E)
            master = _cut(w0, sig + E, emin)
            assert np.array_equal(ref.merge(hi, res, fmt, E).view(np.uint32), master.view(np.uint32))
            m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
            mm = np.zeros(n, np.float32); mv = np.zeros(n, np.float32)
            for t in range(1, 21):
                gb = tobits((make_state(rng, n)[1] * np.float32(scale)).astype(np.float32))
                ref.adam_step(hi, res, gb, m, v, cfg, t)
                master = _cut(_master_adam(master, tof32(gb), mm, mv, 1e-3, 0.9, 0.999, 1e-8, 1e-2, True, t,
                                           1.0 / scale), sig + E, emin)
                assert np.array_equal(ref.merge(hi, res, fmt, E).view(np.uint32), master.view(np.uint32)), (fmt, E, t)
                assert np.array_equal(m.view(np.uint32), mm.view(np.uint32))
                assert np.array_equal(v.view(np.uint32), mv.view(np.uint32))
            # SGD, same idea
            scfg = ref.SgdCfg(lr=1e-2, momentum=0.9, weight_fmt=fmt, grad_fmt=fmt, res_bits=E, loss_scale=scale)
            hi, res = ref.split(w0, fmt, E)
            master = _cut(w0, sig + E, emin)
            buf = np.zeros(n, np.float32); mb = np.zeros(n, np.float32)
            f = np.float32
            for t in range(1, 11):
                gb = tobits((make_state(rng, n)[1] * np.float32(scale)).astype(np.float32))
                ref.sgd_step(hi, res, gb, buf, scfg, t)
                mb = f(0.9) * mb + tof32(gb) * f(1.0 / scale)
                master = _cut(master - f(1e-2) * mb, sig + E, emin)
                assert np.array_equal(ref.merge(hi, res, fmt, E).view(np.uint32), master.view(np.uint32)), (fmt, E, t)


def test_partial_bits_master_equivalence(ref):
    pins_partial_bits_master_equivalence(ref)


def pins_partial_bits_torch_optim(ref):
    """bf16+8 against torch.optim.AdamW on fp32 masters: the only difference is the cut of at
    most 2^-16 of the weight per step, always toward zero."""
    rng = np.random.default_rng(53)
    n, steps = 2048, 20
    w0, _ = make_state(rng, n)
    gbits = [to_bf16_bits(make_state(rng, n)[1]) for _ in range(steps)]
    want = _torch_run("adamw", w0, [bf16_to_f32(b) for b in gbits], lr=1e-3, betas=(0.9, 0.999), eps=1e-8,
                      weight_decay=0.01)
    cfg = ref.AdamCfg(lr=1e-3, weight_decay=0.01, decoupled_wd=True, res_bits=8)
    hi, res = ref.split(w0, ref.BF16, 8)
    m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
    for t, gb in enumerate(gbits, 1):
        ref.adam_step(hi, res, gb, m, v, cfg, t)
    got = ref.merge(hi, res, ref.BF16, 8).astype(np.float64)
    bound = 2 * (steps + 1) * 2.0 ** -16 * (np.maximum(np.abs(want), np.abs(w0)) + steps * 1e-3) + 2e-5 * steps * 1e-3
    assert np.all(np.abs(got - want) <= bound)
    # the cut is toward zero: nearly all weights (those that did not change sign) end up smaller in magnitude
    assert np.mean(np.abs(got) < np.abs(want)) > 0.8


def test_partial_bits_torch_optim(ref):
    pins_partial_bits_torch_optim(ref)


# ---- element-wise gradient clipping inside the step (Section 4.1) ---------------------------------

def pins_grad_clip(ref):
    """Clipping the gradient in the step equals clamping it beforehand (torch.clamp on the un-scaled
    gradient, then an unclipped step), bit for bit; a huge bound changes nothing."""
    rng = np.random.default_rng(59)
    n = 4096
    w0, _ = make_state(rng, n)
    for scale in (1.0, 128.0):
        for clip in (5e-4, 2.0 ** -12):
            out = []
            for fused in (True, False):
                hi, res = ref.split(w0)
                m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
                buf = np.zeros(n, np.float32)
                hs, rs = ref.split(w0)
                r2 = np.random.default_rng(61)
                for t in range(1, 8):
                    g32 = (r2.standard_normal(n) * 1e-3).astype(np.float32)
                    g32[:4] = [clip, -clip, np.float32(clip) * 2, -1.0]
                    gb = to_bf16_bits(g32 * np.float32(scale))
                    if fused:
                        ref.adam_step(hi, res, gb, m, v, ref.AdamCfg(loss_scale=scale, grad_clip=clip), t)
                        ref.sgd_step(hs, rs, gb, buf, ref.SgdCfg(loss_scale=scale, grad_clip=clip), t)
                    else:
                        # clamp outside: un-scale exactly (power of two), clamp with the library, hand over unscaled
                        g = torch.clamp(torch.from_numpy(bf16_to_f32(gb) / np.float32(scale)), -np.float32(clip), np.float32(clip))
                        gb2 = to_bf16_bits(g.numpy())
                        exact = np.array_equal(bf16_to_f32(gb2), g.numpy())
                        assert exact or clip != 2.0 ** -12          # a power-of-two bound stays on the bf16 grid
                        if not exact:
                            break
                        ref.adam_step(hi, res, gb2, m, v, ref.AdamCfg(), t)
                        ref.sgd_step(hs, rs, gb2, buf, ref.SgdCfg(), t)
                else:
                    out.append([a.copy() for a in (hi, res, m, v, hs, rs, buf)])
            if len(out) == 2:
                for a, b in zip(*out):
                    assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), (scale, clip)
    # clipped gradients bound the first Adam step's moments: |m| <= (1-b1)*clip
    hi, res = ref.split(w0)
    m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
    gb = to_bf16_bits((rng.standard_normal(n)).astype(np.float32))
    ref.adam_step(hi, res, gb, m, v, ref.AdamCfg(grad_clip=0.25), 1)
    assert np.all(np.abs(m) <= np.float32(0.1) * np.float32(0.25) * (1 + 1e-6)) and np.mean(np.abs(m) > 0.02) > 0.5
    # a bound nothing reaches leaves the step unchanged
    a = ref.split(w0); b = ref.split(w0)
    ma = np.zeros(n, np.float32); va = np.zeros(n, np.float32); mb = np.zeros(n, np.float32); vb = np.zeros(n, np.float32)
    ref.adam_step(a[0], a[1], gb, ma, va, ref.AdamCfg(grad_clip=1e30), 1)
    ref.adam_step(b[0], b[1], gb, mb, vb, ref.AdamCfg(), 1)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and np.array_equal(ma, mb)


def test_grad_clip(ref):
    pins_grad_clip(ref)
