"""Pins for the oracle's rounding modes of the 16-bit value (arXiv 2309.12381, Section 3.1,
last paragraph: stochastic rounding at split, with one more stored bit that says whether the
value was rounded up so that it can be un-rounded before the update; round-to-nearest is the
deterministic counterpart, undone from the leading dropped bit).

What pins them:
  * Philox4x32-10 against the known answers of the published generator, and against a second
    implementation written here in plain Python;
  * merge(split(x, mode)) is the same fp32 value in every mode (only hi differs);
  * NEAREST: hi equals the library's round-to-nearest cast except at exact ties;
  * STOCHASTIC: hi is one of the two neighbours, P(up) = dropped bits / 2^full (binomial bound),
    the mean of hi is x, never up from an exact value or out of the finite range, the flag sits
    just above the kept bits, draws depend on seed, step, tensor and element exactly as stated;
  * a slice handled with `first_index` draws what the stated stream gives at those positions;
  * NEAREST never turns a NaN into something else (the all-ones pattern does not wrap to zero);
  * steps: the fp32 trajectory (merged weights, m, v) does not depend on the rounding mode.
`pins_*` take the oracle as argument (tests/test_oracle_pins_bite.py runs them on broken builds).
"""
import numpy as np
import torch

from test_oracle_steps import bf16_to_f32, fp16_to_f32, make_state, to_bf16_bits, to_fp16_bits

FULL = {0: 16, 1: 13}
MAXFIN = {0: 0x7F7F, 1: 0x7BFF}


# ---- Philox4x32-10 ------------------------------------------------------------------------

def philox_py(counter, key):
    """Second implementation, straight from the published description: 10 rounds; each round
    multiplies words 0 and 2 by two constants, keeps the low halves and xors the high halves
    with the other two words and the key; the key advances by Weyl constants between rounds."""
    c = list(counter)
    k = list(key)
    for r in range(10):
        if r:
            k[0] = (k[0] + 0x9E3779B9) & 0xFFFFFFFF
            k[1] = (k[1] + 0xBB67AE85) & 0xFFFFFFFF
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
    return c


KNOWN = [  # counter, key, output: test vectors published with the generator
    ([0, 0, 0, 0], [0, 0], [0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8]),
    ([0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344], [0xA4093822, 0x299F31D0],
     [0xD16CFE09, 0x94FDCCEB, 0x5001E420, 0x24126EA1]),
]


def pins_philox(ref):
    for c, k, want in KNOWN:
        assert ref.philox(c, k) == want
        assert philox_py(c, k) == want
    rng = np.random.default_rng(1)
    for _ in range(200):
        c = [int(x) for x in rng.integers(0, 1 << 32, 4)]
        k = [int(x) for x in rng.integers(0, 1 << 32, 2)]
        assert ref.philox(c, k) == philox_py(c, k)


def test_philox(ref):
    pins_philox(ref)


# ---- split / merge in the three modes ---------------------------------------------------------

def _patterns(rng, n):
    x = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)
    k = n // 2
    x[:k] = (rng.standard_normal(k) * 0.02).astype(np.float32).view(np.uint32)
    edge = np.array([0.0, -0.0, 1.0, -1.0, 1.00390625, 1.001953125, 0.99609375, 65504.0, 65519.99, 65520.0, 70000.0,
                     3.3895314e38, 3.4028235e38, 6.1e-5, 3e-5, 2.0 ** -37, 1e-45], np.float32)
    x[-edge.size:] = edge.view(np.uint32)
    x = x.view(np.float32)
    return x[np.isfinite(x)]


def pins_value_is_mode_independent(ref):
    rng = np.random.default_rng(3)
    x = _patterns(rng, 1 << 18)
    for fmt in (ref.BF16, ref.FP16):
        for E in (0, 12, 7, 3):
            h0, r0 = ref.split(x, fmt, E, ref.TRUNC)
            base = ref.merge(h0, r0, fmt, E, ref.TRUNC)
            h1, r1 = ref.split(x, fmt, E, ref.NEAREST)
            assert np.array_equal(ref.merge(h1, r1, fmt, E, ref.NEAREST).view(np.uint32), base.view(np.uint32))
            assert np.array_equal(r1, r0)                       # NEAREST stores nothing extra
            d = (h1.astype(np.int32) - h0.astype(np.int32)) & 0xFFFF
            assert np.all((d == 0) | (d == 1))
            # STOCHASTIC: with all bits asked for, bf16 keeps 15 (the flag takes the 16th)
            Es = E
            Et = 15 if (E == 0 and fmt == ref.BF16) else E
            ht, rt = ref.split(x, fmt, Et, ref.TRUNC)
            base_s = ref.merge(ht, rt, fmt, Et, ref.TRUNC)
            h2, r2 = ref.split(x, fmt, Es, ref.STOCHASTIC, seed=77, tensor_id=5)
            assert np.array_equal(ref.merge(h2, r2, fmt, Es, ref.STOCHASTIC).view(np.uint32), base_s.view(np.uint32))
            d = (h2.astype(np.int32) - ht.astype(np.int32)) & 0xFFFF
            assert np.all((d == 0) | (d == 1))
            kept = Et if Et else FULL[fmt]
            assert np.array_equal((r2.astype(np.uint32) >> kept), d.astype(np.uint32))       # the flag
            assert np.array_equal(r2.astype(np.uint32) & ((1 << kept) - 1), rt.astype(np.uint32))
            assert np.all((ht[d == 1] & 0x7FFF) < MAXFIN[fmt])                                # stays finite


def test_value_is_mode_independent(ref):
    pins_value_is_mode_independent(ref)


def pins_nearest_matches_library_cast(ref):
    rng = np.random.default_rng(5)
    x = _patterns(rng, 1 << 20)
    # bf16
    hi, res = ref.split(x, ref.BF16, 0, ref.NEAREST)
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    tie = (x.view(np.uint32) & 0xFFFF) == 0x8000
    assert np.array_equal(hi[~tie], lib[~tie])
    # at a tie the library goes to even, this mode away from zero: the two differ by at most one step
    assert np.all(np.abs(hi[tie].astype(np.int32) - lib[tie].astype(np.int32)) <= 1)
    up = bf16_to_f32(hi)
    fin = np.isfinite(up)
    err = np.abs(up[fin].astype(np.float64) - x[fin])
    ulp = np.spacing(np.abs(up[fin])).astype(np.float64) * 65536.0
    assert np.all(err <= ulp / 2)
    # fp16, inside its normal range
    y = x[(np.abs(x) >= 2.0 ** -14) & (np.abs(x) < 65519.0)]
    hi, res = ref.split(y, ref.FP16, 0, ref.NEAREST)
    lib = y.astype(np.float16).view(np.uint16)
    tie = (y.view(np.uint32) & 0x1FFF) == 0x1000
    assert np.array_equal(hi[~tie], lib[~tie])
    # a finite value within half a step of overflow becomes infinity, as in IEEE rounding, and merge undoes it
    big = np.array([65520.0, -65530.0, 3.3961775e38], np.float32)
    h, r = ref.split(big[:2], ref.FP16, 0, ref.NEAREST)
    assert list(h) == [0x7C00, 0xFC00]
    assert np.array_equal(ref.merge(h, r, ref.FP16, 0, ref.NEAREST), big[:2])
    h, r = ref.split(big[2:], ref.BF16, 0, ref.NEAREST)
    assert list(h) == [0x7F80] and ref.merge(h, r, ref.BF16, 0, ref.NEAREST)[0] == big[2]


def test_nearest_matches_library_cast(ref):
    pins_nearest_matches_library_cast(ref)


def pins_stochastic_statistics(ref):
    """P(up) = dropped bits / 2^full, checked per value with a 5.5-sigma binomial bound over
    2^16 elements holding the same value; mean of hi is the value; exact values never move."""
    n = 1 << 16
    for fmt, tof32, cases in ((ref.BF16, bf16_to_f32, [1.001, 1.0039, -0.0200001, 0.3330001, 1.0078124]),
                              (ref.FP16, fp16_to_f32, [1.0001, -0.02000001, 0.3330001, 1.0009764, 6.0e-5])):
        full = FULL[fmt]
        for val in cases:
            x = np.full(n, val, np.float32)
            ht, rt = ref.split(x[:1], fmt, 0, ref.TRUNC)
            p = int(rt[0]) / float(1 << full)
            hi, res = ref.split(x, fmt, 0, ref.STOCHASTIC, seed=12345, tensor_id=3)
            ups = int(np.count_nonzero(hi != ht[0]))
            sigma = (n * p * (1 - p)) ** 0.5
            assert abs(ups - n * p) <= 5.5 * sigma + 1, (fmt, val, ups, n * p)
            lo, up = float(tof32(ht)[0]), float(tof32(ht + np.uint16(1))[0])
            mean = (lo * (n - ups) + up * ups) / n
            assert abs(mean - float(np.float32(val))) <= 5.5 * abs(up - lo) * sigma / n + abs(up - lo) * 2.0 ** -full
        exact = np.full(n, 0.5, np.float32)
        hi, res = ref.split(exact, fmt, 0, ref.STOCHASTIC, seed=9)
        assert np.all(hi == hi[0]) and not res.any()
        # the largest finite 16-bit value is never pushed to infinity
        top = np.full(1024, 65519.0 if fmt == ref.FP16 else 3.4e38, np.float32)
        hi, res = ref.split(top, fmt, 0, ref.STOCHASTIC, seed=9)
        assert np.all(hi == MAXFIN[fmt])


def test_stochastic_statistics(ref):
    pins_stochastic_statistics(ref)


def _expected_up(x_res_full, full, seed, step, tensor, n, first=0):
    """Which elements round up, from the stated stream: Philox4x32-10 with key = seed and counter
    = (i/4 low, i/4 high, step low 32 bits, tensor); element i takes word i%4, its top bits.
    `first`: position in the tensor of element 0 of the array."""
    key = [seed & 0xFFFFFFFF, seed >> 32]
    out = np.zeros(n, bool)
    for b in range(first // 4, (first + n + 3) // 4):
        w = philox_py([b & 0xFFFFFFFF, b >> 32, step & 0xFFFFFFFF, tensor], key)
        for j in range(4):
            i = 4 * b + j - first
            if 0 <= i < n:
                out[i] = (w[j] >> (32 - full)) < int(x_res_full[i])
    return out


def pins_stochastic_stream(ref):
    rng = np.random.default_rng(7)
    n = 1001
    x = (0.5 + rng.random(n)).astype(np.float32)
    for fmt in (ref.BF16, ref.FP16):
        full = FULL[fmt]
        _, rfull = ref.split(x, fmt, 0, ref.TRUNC)
        ht, _ = ref.split(x, fmt, 0, ref.TRUNC)
        seen = []
        for seed, tensor in ((1, 0), (1, 1), (2, 0), ((1 << 40) + 1, 0)):
            hi, res = ref.split(x, fmt, 0, ref.STOCHASTIC, seed=seed, tensor_id=tensor)
            up = hi != ht
            assert np.array_equal(up, _expected_up(rfull, full, seed, 0, tensor, n)), (fmt, seed, tensor)
            seen.append(up)
        assert not np.array_equal(seen[0], seen[1]) and not np.array_equal(seen[0], seen[2])
        assert not np.array_equal(seen[0], seen[3])
        # inside a step the step number selects the draws, and the weights that result are rounded with them
        for step in (1, 2, (1 << 32) + 1):
            cfg = ref.SgdCfg(lr=0.0, momentum=0.0, weight_fmt=fmt, round=ref.STOCHASTIC, seed=99)
            hi, res = ref.split(x, fmt, 0, ref.STOCHASTIC, seed=99, tensor_id=4)
            ref.sgd_step(hi, res, np.zeros(n, np.uint16), None, cfg, step, tensor_id=4)
            # lr = 0: the fp32 value is unchanged, only re-rounded with this step's draws
            keep = 15 if fmt == ref.BF16 else 13
            _, r15 = ref.split(x, fmt, keep, ref.TRUNC)
            rf = r15.astype(np.uint32) << (full - keep)
            assert np.array_equal(hi != ht, _expected_up(rf, full, 99, step, 4, n)), (fmt, step)


def test_stochastic_stream(ref):
    pins_stochastic_stream(ref)


def pins_first_index(ref):
    """A slice of a tensor, handled with the position of its first element, gets the draws of
    those positions: checked against the stated stream (second Philox implementation) for starts
    of every residue modulo 4 and beyond 2^34 elements, where the counter's second word is in
    use, and against the same elements handled as part of a whole array."""
    rng = np.random.default_rng(17)
    n = 203
    x = (0.5 + rng.random(n)).astype(np.float32)
    for fmt in (ref.BF16, ref.FP16):
        full = FULL[fmt]
        ht, rfull = ref.split(x, fmt, 0, ref.TRUNC)
        whole_hi, whole_res = ref.split(x, fmt, 0, ref.STOCHASTIC, seed=5, tensor_id=2)
        for first in (0, 1, 2, 3, 4, 77, (1 << 34) - 2, (1 << 34) + 5, (3 << 34) + 1):
            hi, res = ref.split(x, fmt, 0, ref.STOCHASTIC, seed=5, tensor_id=2, first_index=first)
            assert np.array_equal(hi != ht, _expected_up(rfull, full, 5, 0, 2, n, first)), (fmt, first)
            if first < n:           # the tail of the whole array is the slice that starts there
                h2, r2 = ref.split(x[first:].copy(), fmt, 0, ref.STOCHASTIC, seed=5, tensor_id=2, first_index=first)
                assert np.array_equal(h2, whole_hi[first:]) and np.array_equal(r2, whole_res[first:])
        # the steps take it the same way (lr = 0: the value is only re-rounded with this step's draws)
        keep = 15 if fmt == ref.BF16 else 13
        _, rk = ref.split(x, fmt, keep, ref.TRUNC)
        rf = rk.astype(np.uint32) << (full - keep)
        for first in (0, 3, (1 << 34) + 6):
            hi, res = ref.split(x, fmt, 0, ref.STOCHASTIC, seed=5, tensor_id=2, first_index=first)
            cfg = ref.SgdCfg(lr=0.0, momentum=0.0, weight_fmt=fmt, round=ref.STOCHASTIC, seed=5)
            ref.sgd_step(hi, res, np.zeros(n, np.uint16), None, cfg, 3, tensor_id=2, first_index=first)
            assert np.array_equal(hi != ht, _expected_up(rf, full, 5, 3, 2, n, first)), (fmt, first)
            hi, res = ref.split(x, fmt, 0, ref.STOCHASTIC, seed=5, tensor_id=2, first_index=first)
            acfg = ref.AdamCfg(lr=0.0, weight_fmt=fmt, grad_fmt=fmt, round=ref.STOCHASTIC, seed=5)
            ref.adam_step(hi, res, np.zeros(n, np.uint16), np.zeros(n, np.float32), np.zeros(n, np.float32), acfg, 3,
                          tensor_id=2, first_index=first)
            assert np.array_equal(hi != ht, _expected_up(rf, full, 5, 3, 2, n, first)), (fmt, first)


def test_first_index(ref):
    pins_first_index(ref)


def pins_nearest_keeps_nan(ref):
    """Round-to-nearest adds one to the 16-bit pattern; on a NaN pattern that could wrap around to a
    zero.  A NaN must stay a NaN in hi and in the merged value, in split and through a step, and
    every pattern that is not a NaN must still come back bit for bit."""
    for fmt, tof32, inf in ((ref.BF16, bf16_to_f32, 0x7F80), (ref.FP16, fp16_to_f32, 0x7C00)):
        full = FULL[fmt]
        # every fp32 NaN whose 16-bit part is all ones, with the leading dropped bit set or not, both signs
        if fmt == ref.BF16:
            nan_bits = np.array([0x7FFF8000, 0x7FFFFFFF, 0xFFFF8000, 0xFFFFFFFF, 0x7FFF0001, 0x7F808000, 0x7FC08000,
                                 0x7F800001, 0xFF80FFFF], np.uint32)
        else:
            nan_bits = np.array([0x7FFFF000, 0x7FFFFFFF, 0xFFFFF000, 0x7FC01000, 0xFF801000, 0x7F800001], np.uint32)
        x = nan_bits.view(np.float32)
        hi, res = ref.split(x, fmt, 0, ref.NEAREST)
        assert np.all((hi & 0x7FFF) >= inf), [hex(h) for h in hi]
        back = ref.merge(hi, res, fmt, 0, ref.NEAREST)
        assert np.all(np.isnan(back)), back
        # what forward sees is a NaN whenever the 16-bit pattern of the truncated value is one
        ht, _ = ref.split(x, fmt, 0, ref.TRUNC)
        was_nan16 = (ht & 0x7FFF) > inf
        assert np.all(np.isnan(tof32(hi))[was_nan16])
        # such a pattern is left alone in both directions: it comes back as TRUNC would give it
        t_back = ref.merge(*ref.split(x, fmt, 0, ref.TRUNC), fmt, 0, ref.TRUNC)
        assert np.array_equal(back.view(np.uint32)[was_nan16], t_back.view(np.uint32)[was_nan16])
        assert np.array_equal(hi[was_nan16], ht[was_nan16])
        # through a step: a NaN gradient makes the weight a NaN and it stays one
        w = np.full(8, 0.5, np.float32)
        hi, res = ref.split(w, fmt, 0, ref.NEAREST)
        g = np.full(8, 0x7FFF, np.uint16)
        cfg = ref.SgdCfg(lr=0.1, momentum=0.0, weight_fmt=fmt, grad_fmt=fmt, round=ref.NEAREST)
        for t in (1, 2, 3):
            ref.sgd_step(hi, res, g if t == 1 else np.zeros(8, np.uint16), None, cfg, t)
            assert np.all(np.isnan(tof32(hi))) and np.all(np.isnan(ref.merge(hi, res, fmt, 0, ref.NEAREST)))
        # everything that is not a NaN still round-trips exactly (all 16-bit values x a few residuals)
        h_all = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
        h_all = h_all[(h_all & 0x7FFF) <= inf]
        for r in (0, 1, (1 << (full - 1)) - 1, 1 << (full - 1), (1 << full) - 1):
            rr = np.full(h_all.size, r, np.uint16)
            val = ref.merge(h_all, rr, fmt, 0, ref.TRUNC)
            keep = ~np.isnan(val)
            h1, r1 = ref.split(val[keep], fmt, 0, ref.NEAREST)
            again = ref.merge(h1, r1, fmt, 0, ref.NEAREST)
            assert np.array_equal(again.view(np.uint32), val[keep].view(np.uint32)), (fmt, r)


def test_nearest_keeps_nan(ref):
    pins_nearest_keeps_nan(ref)


# ---- steps: the fp32 trajectory does not depend on how hi is rounded ---------------------------

def pins_trajectory_is_mode_independent(ref):
    rng = np.random.default_rng(11)
    n = 3000
    for fmt, tobits, scale in ((ref.BF16, to_bf16_bits, 1.0), (ref.FP16, to_fp16_bits, 256.0)):
        w0, _ = make_state(rng, n)
        if fmt == ref.FP16:
            w0 = np.where(np.abs(w0) < 2.0 ** -10, np.float32(2.0 ** -10), w0).astype(np.float32)
        grads = [tobits((make_state(rng, n)[1] * np.float32(scale)).astype(np.float32)) for _ in range(12)]
        for E in (0, 8):
            runs = {}
            for mode in (ref.TRUNC, ref.NEAREST, ref.STOCHASTIC):
                Em = E
                if mode != ref.STOCHASTIC and E == 0 and fmt == ref.BF16:
                    Em = 15                          # what STOCHASTIC keeps for bf16 when asked for all
                if mode == ref.STOCHASTIC and E == 8:
                    continue                         # 8 bits + flag do not fit a byte
                cfg = ref.AdamCfg(lr=1e-3, weight_decay=1e-2, loss_scale=scale, weight_fmt=fmt, grad_fmt=fmt,
                                  res_bits=Em if mode != ref.STOCHASTIC else E, round=mode, seed=4242)
                hi, res = ref.split(w0, fmt, cfg.res_bits, mode, 4242, 9)
                m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
                his = []
                for t, g in enumerate(grads, 1):
                    ref.adam_step(hi, res, g, m, v, cfg, t, tensor_id=9)
                    his.append(hi.copy())
                runs[mode] = (ref.merge(hi, res, fmt, cfg.res_bits, mode).copy(), m, v, his)
            base = runs[ref.TRUNC]
            for mode, r in runs.items():
                assert np.array_equal(r[0].view(np.uint32), base[0].view(np.uint32)), (fmt, E, mode)
                assert np.array_equal(r[1].view(np.uint32), base[1].view(np.uint32))
                assert np.array_equal(r[2].view(np.uint32), base[2].view(np.uint32))
                if mode != ref.TRUNC:
                    d = (r[3][-1].astype(np.int32) - base[3][-1].astype(np.int32)) & 0xFFFF
                    assert np.all((d == 0) | (d == 1)) and 0.2 < d.mean() < 0.8
            if ref.STOCHASTIC in runs:
                # stochastic draws change from step to step
                a, b = runs[ref.STOCHASTIC][3][-1] != base[3][-1], runs[ref.STOCHASTIC][3][-2] != base[3][-2]
                assert not np.array_equal(a, b)


def test_trajectory_is_mode_independent(ref):
    pins_trajectory_is_mode_independent(ref)
