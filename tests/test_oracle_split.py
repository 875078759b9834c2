"""Pins for the oracle's split / merge (arXiv 2309.12381, Table 1 and Section 3.1).

None of these re-type the oracle's bit formulas.  They pin it to
  * hand-worked patterns (tests/golden/split_patterns.txt),
  * the value definition: hi is the 16-bit float obtained by rounding x toward
    zero, and res counts how many units of the fp32 grid lie between hi and x
    (checked in exact rational arithmetic with a decoder that knows only the
    field widths of Table 1),
  * library casts (torch bfloat16, numpy float16) turned into round-toward-zero,
  * the lossless round trip over every fp32 bit pattern, and over every pair.
"""
import os
from concurrent.futures import ThreadPoolExecutor
from fractions import Fraction

import numpy as np
import pytest
import torch

from exact_fp32 import decode, float_of

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "split_patterns.txt")
WORKERS = min(8, os.cpu_count() or 1)
CHUNK = 1 << 21


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            fmt, b, hi, res, mb = line.split()[:5]
            rows.append((fmt, int(b, 16), int(hi, 16), int(res, 16), int(mb, 16)))
    return rows


def test_golden_patterns(ref):
    pins_golden_patterns(ref)


def pins_golden_patterns(ref):
    rows = _golden_rows()
    assert len(rows) >= 18
    for fmt, b, hi, res, mb in rows:
        f = ref.FP16 if fmt == "fp16" else ref.BF16
        x = np.array([b], np.uint32).view(np.float32)
        h, r = ref.split(x, f)
        assert (int(h[0]), int(r[0])) == (hi, res), (fmt, hex(b), hex(int(h[0])), hex(int(r[0])))
        w = ref.merge(h, r, f)
        assert int(w.view(np.uint32)[0]) == mb, (fmt, hex(b))


# ---- value definition, exact rational arithmetic -------------------------

FIELDS = {"bf16": (8, 7), "fp16": (5, 10)}   # exponent, stored significand bits (Table 1)


def _expected_split_value(x: Fraction, fmt: str):
    """(|hi| as a rational, res as an integer) from the value definition alone."""
    ebits, mbits = FIELDS[fmt]
    bias = (1 << (ebits - 1)) - 1
    emin = 1 - bias
    a = abs(x)
    if a == 0:
        return Fraction(0), 0
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    max16 = (2 - Fraction(1, 1 << mbits)) * Fraction(2) ** bias
    if a >= Fraction(2) ** (bias + 1):
        # beyond the 16-bit format's range: largest finite pair (only fp16 can get here)
        return max16, (1 << (23 - mbits)) - 1
    e16 = max(e, emin)                        # exponent of the 16-bit float's grid
    ulp16 = Fraction(2) ** (e16 - mbits)
    hi = (a / ulp16).__floor__() * ulp16      # round toward zero
    # the residual counts units of 2^(23-mbits) per ulp16; in the 16-bit
    # subnormal range x may lie below that grid and is cut
    unit = ulp16 / (1 << (23 - mbits))
    if fmt == "bf16":
        # bf16 shares fp32's exponent range: fp32 subnormals sit on 2^-149 = unit
        assert unit == Fraction(2) ** (max(e, -126) - 23)
    res = ((a - hi) / unit).__floor__()
    return hi, res


def _sample_patterns(rng, n):
    pats = list(rng.integers(0, 1 << 32, size=n, dtype=np.uint64))
    # edges: every exponent with all-zero, all-one and single-bit fractions
    for E in range(0, 255):
        for M in (0, 1, 0x7FFFFF, 0x400000, 0x1FFF, 0x2000, 0xFFFF, 0x10000, 0x7FE000):
            pats.append((E << 23) | M)
            pats.append((1 << 31) | (E << 23) | M)
    return [int(p) for p in pats]


@pytest.mark.parametrize("fmt", ["bf16", "fp16"])
def test_split_is_round_toward_zero_plus_grid_count(ref, fmt):
    pins_split_value_definition(ref, fmt)


def pins_split_value_definition(ref, fmt):
    f = ref.FP16 if fmt == "fp16" else ref.BF16
    ebits, mbits = FIELDS[fmt]
    rng = np.random.default_rng(12381)
    pats = [p for p in _sample_patterns(rng, 6000) if ((p >> 23) & 0xFF) != 255]
    x = np.array(pats, np.uint32).view(np.float32)
    hi, res = ref.split(x, f)
    w = ref.merge(hi, res, f)
    for i, p in enumerate(pats):
        xv = Fraction(float_of(p))
        exp_hi, exp_res = _expected_split_value(xv, fmt)
        got_hi = decode(int(hi[i]), ebits, mbits)
        assert not isinstance(got_hi, str), hex(p)
        assert abs(got_hi) == exp_hi, (fmt, hex(p))
        assert (int(hi[i]) >> 15) == (p >> 31), (fmt, hex(p))        # sign kept, also on zero
        assert int(res[i]) == exp_res, (fmt, hex(p), int(res[i]), exp_res)
        # merge puts back exactly what the pair holds
        e16 = max((int(hi[i]) >> mbits) & ((1 << ebits) - 1), 1) - ((1 << (ebits - 1)) - 1)
        unit = Fraction(2) ** (e16 - 23)
        sign = -1 if p >> 31 else 1
        assert Fraction(float(w[i])) == sign * (exp_hi + exp_res * unit), (fmt, hex(p))


# ---- exhaustive sweeps ---------------------------------------------------

def _rtz_bf16(x):
    """Library cast (round-to-nearest) stepped back toward zero where it overshot."""
    t = torch.from_numpy(x)
    h = t.to(torch.bfloat16)
    over = (h.float().abs() > t.abs()).numpy()
    hb = h.view(torch.int16).numpy().view(np.uint16)
    return hb - over.astype(np.uint16)


def _rtz_fp16(x):
    with np.errstate(over="ignore"):
        h = x.astype(np.float16)
    over = np.abs(h.astype(np.float32)) > np.abs(x)
    return h.view(np.uint16) - over.astype(np.uint16)


def _check_bf16_chunk(ref, c):
    b = np.arange(c * CHUNK, (c + 1) * CHUNK, dtype=np.uint64).astype(np.uint32)
    x = b.view(np.float32)
    hi, res = ref.split(x, ref.BF16)
    w = ref.merge(hi, res, ref.BF16)
    assert np.array_equal(w.view(np.uint32), b), "round trip, chunk %d" % c
    fin = np.isfinite(x)
    assert np.array_equal(hi[fin], _rtz_bf16(x)[fin]), "hi is not the RTZ cast, chunk %d" % c
    # every (hi, res) pair, enumerated directly, survives merge then split
    ph = (b >> 16).astype(np.uint16)
    pr = (b & 0xFFFF).astype(np.uint16)
    h2, r2 = ref.split(ref.merge(ph, pr, ref.BF16), ref.BF16)
    assert np.array_equal(h2, ph) and np.array_equal(r2, pr), "pair round trip, chunk %d" % c
    return True


def test_bf16_exhaustive_all_fp32_patterns(ref):
    with ThreadPoolExecutor(WORKERS) as ex:
        assert all(ex.map(lambda c: _check_bf16_chunk(ref, c), range((1 << 32) // CHUNK)))


def _check_fp16_chunk(ref, c):
    b = np.arange(c * CHUNK, (c + 1) * CHUNK, dtype=np.uint64).astype(np.uint32)
    x = b.view(np.float32)
    sign = b & np.uint32(0x80000000)
    hi, res = ref.split(x, ref.FP16)
    w = ref.merge(hi, res, ref.FP16)
    wb = w.view(np.uint32)
    a = np.abs(x)
    fin = np.isfinite(x)
    nan = np.isnan(x)
    assert np.all(res < 0x2000)
    # hi is the round-toward-zero cast of x (library cast, corrected)
    assert np.array_equal(hi[fin], _rtz_fp16(x)[fin]), "hi is not the RTZ cast, chunk %d" % c
    # exact where the pair can hold x
    normal = fin & (a >= np.float32(2.0 ** -14)) & (a < np.float32(65536.0))
    assert np.array_equal(wb[normal], b[normal]), "normal range round trip, chunk %d" % c
    # too large: largest finite pair
    big = fin & (a >= np.float32(65536.0))
    assert np.all(wb[big] == (sign[big] | np.uint32(0x477FFFFF)))
    # below 2^-14: cut to a multiple of 2^-37 (exact in binary64)
    small = a < np.float32(2.0 ** -14)
    cut = (np.trunc(x[small].astype(np.float64) * 2.0 ** 37) / 2.0 ** 37).astype(np.float32)
    assert np.array_equal(wb[small], cut.view(np.uint32)), "subnormal range, chunk %d" % c
    # infinities and NaN
    inf = np.isinf(x)
    assert np.array_equal(wb[inf], b[inf])
    assert np.all(np.isnan(w[nan])) and np.all((wb[nan] & np.uint32(0x80000000)) == sign[nan])
    # what split keeps is stable: split(merge(split(x))) == split(x)
    h2, r2 = ref.split(w, ref.FP16)
    assert np.array_equal(h2, hi) and np.array_equal(r2, res), "idempotence, chunk %d" % c
    return True


def test_fp16_exhaustive_all_fp32_patterns(ref):
    with ThreadPoolExecutor(WORKERS) as ex:
        assert all(ex.map(lambda c: _check_fp16_chunk(ref, c), range((1 << 32) // CHUNK)))


def _check_fp16_pairs_chunk(ref, c):
    idx = np.arange(c * CHUNK, (c + 1) * CHUNK, dtype=np.uint64)
    ph = (idx >> 13).astype(np.uint16)            # all 2^16 hi patterns
    pr = (idx & 0x1FFF).astype(np.uint16)         # all 2^13 residuals
    w = ref.merge(ph, pr, ref.FP16)
    h2, r2 = ref.split(w, ref.FP16)
    nonfin = (ph & 0x7C00) == 0x7C00
    isnan = nonfin & ((ph & 0x3FF) != 0)
    ok = ~nonfin | (~isnan & (pr == 0))           # finite pairs, and the two infinities
    assert np.array_equal(h2[ok], ph[ok]) and np.array_equal(r2[ok], pr[ok]), "chunk %d" % c
    assert np.all(np.isnan(w[isnan])) and np.all(np.isinf(w[nonfin & ~isnan]))
    # the three spare residual bits are ignored by merge
    w_spare = ref.merge(ph, pr | np.uint16(0xE000), ref.FP16)
    assert np.array_equal(w_spare.view(np.uint32)[ok], w.view(np.uint32)[ok])
    return True


def test_fp16_every_pair_round_trips(ref):
    with ThreadPoolExecutor(WORKERS) as ex:
        assert all(ex.map(lambda c: _check_fp16_pairs_chunk(ref, c), range((1 << 29) // CHUNK)))


@pytest.mark.parametrize("fmt", ["bf16", "fp16"])
def test_cvt16_matches_library_cast(ref, fmt):
    """The gradient conversion reads every 16-bit pattern as the library does."""
    pats = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    if fmt == "bf16":
        lib = torch.from_numpy(pats.view(np.int16)).view(torch.bfloat16).float().numpy()
        f = ref.BF16
    else:
        lib = pats.view(np.float16).astype(np.float32)
        f = ref.FP16
    got = ref.merge(pats, np.zeros(1 << 16, np.uint16), f)
    nan = np.isnan(lib)
    assert np.array_equal(got.view(np.uint32)[~nan], lib.view(np.uint32)[~nan])
    assert np.all(np.isnan(got[nan]))
    for p in (0x0001, 0x03FF, 0x0400, 0x3C00, 0x7BFF, 0x8001, 0xBA83, 0x3A80):
        assert ref.cvt16(p, f) == float(lib[p])


# ---- keeping only E of the extra bits (Section 3.1 allows keeping only some of them) ----

FULL = {"bf16": 16, "fp16": 13}


def pins_partial_bits_value_definition(ref, fmt):
    """res_bits = E keeps the E leading extra bits: hi is unchanged, the residual is the full
    one divided by 2^(full-E) rounded down, and merge gives hi + res * 2^(full-E) grid units."""
    f = ref.FP16 if fmt == "fp16" else ref.BF16
    ebits, mbits = FIELDS[fmt]
    full = FULL[fmt]
    rng = np.random.default_rng(8)
    pats = [p for p in _sample_patterns(rng, 300)[::7] if ((p >> 23) & 0xFF) != 255]
    x = np.array(pats, np.uint32).view(np.float32)
    for E in (1, 4, 8, 9, 12, full):
        hi, res = ref.split(x, f, E)
        assert res.dtype == (np.uint8 if E <= 8 else np.uint16)
        w = ref.merge(hi, res, f, E)
        for i, p in enumerate(pats):
            xv = Fraction(float_of(p))
            exp_hi, exp_res = _expected_split_value(xv, fmt)
            kept = exp_res >> (full - E)
            assert abs(decode(int(hi[i]), ebits, mbits)) == exp_hi, (fmt, E, hex(p))
            assert int(res[i]) == kept, (fmt, E, hex(p), int(res[i]), kept)
            e16 = max((int(hi[i]) >> mbits) & ((1 << ebits) - 1), 1) - ((1 << (ebits - 1)) - 1)
            unit = Fraction(2) ** (e16 - 23)
            sign = -1 if p >> 31 else 1
            assert Fraction(float(w[i])) == sign * (exp_hi + (kept << (full - E)) * unit), (fmt, E, hex(p))
    # E = 0 and E = full are the same thing
    h0, r0 = ref.split(x, f, 0)
    h1, r1 = ref.split(x, f, full)
    assert np.array_equal(h0, h1) and np.array_equal(r0, r1)


@pytest.mark.parametrize("fmt", ["bf16", "fp16"])
def test_partial_bits_value_definition(ref, fmt):
    pins_partial_bits_value_definition(ref, fmt)


def _trunc_to_bits(x, sig_bits, emin):
    """|x| cut toward zero to `sig_bits` significant bits (grid fixed below 2^emin): library
    frexp / trunc in binary64, exact for binary32 inputs."""
    a = np.abs(x.astype(np.float64))
    m, e = np.frexp(a)                                  # a = m * 2^e, m in [0.5, 1)
    e = np.maximum(e, emin + 1)
    ulp = np.ldexp(1.0, e - sig_bits)
    return np.copysign(np.trunc(a / ulp) * ulp, x.astype(np.float64)).astype(np.float32)


def pins_partial_bits_is_truncation(ref):
    """merge(split(x, E)) is x cut toward zero to 8+E (bf16) or 11+E (fp16) significant bits."""
    rng = np.random.default_rng(9)
    x = rng.integers(0, 1 << 32, size=1 << 22, dtype=np.uint64).astype(np.uint32).view(np.float32)
    x = x[np.isfinite(x)]
    for E in (8, 3, 12):
        hi, res = ref.split(x, ref.BF16, E)
        got = ref.merge(hi, res, ref.BF16, E)
        want = _trunc_to_bits(x, 8 + E, -126)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), E
    inr = x[(np.abs(x) >= 2.0 ** -14) & (np.abs(x) < 65536.0)]
    for E in (8, 5, 12):
        hi, res = ref.split(inr, ref.FP16, E)
        got = ref.merge(hi, res, ref.FP16, E)
        want = _trunc_to_bits(inr, 11 + E, -14)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), E
        # what is kept is stable
        h2, r2 = ref.split(got, ref.FP16, E)
        assert np.array_equal(h2, hi) and np.array_equal(r2, res)


def test_partial_bits_is_truncation(ref):
    pins_partial_bits_is_truncation(ref)


# ---- packed storage of the extra bits (Section 3.1, Figure 1) -----------------------------------

def unpack_planes(buf: np.ndarray, n: int, E: int) -> np.ndarray:
    """Independent decoder of the packed layout, from its description: an 8-, a 4-, a 2- and a
    1-bit plane (those the binary form of E contains), in that order, each starting at a multiple of
    16 bytes, value i at bits [w*i, w*i+w) of its plane, little-endian; the 8-bit piece holds the
    leading bits."""
    bits = np.unpackbits(buf, bitorder="little")
    out = np.zeros(n, np.uint32)
    pos = 0                                             # byte offset of the current plane
    for w in (8, 4, 2, 1):
        if not E & w:
            continue
        plane = bits[8 * pos: 8 * pos + w * n].reshape(n, w)
        val = (plane.astype(np.uint32) << np.arange(w, dtype=np.uint32)).sum(axis=1)
        out = (out << w) | val
        pos += (((n * w + 7) // 8) + 15) // 16 * 16
    assert pos == buf.size
    return out


def pins_packed_storage(ref):
    rng = np.random.default_rng(71)
    for fmt, full in ((ref.BF16, 16), (ref.FP16, 13)):
        for n in (1, 2, 3, 5, 16, 31, 33, 4099):
            x = (rng.standard_normal(n) * 0.02).astype(np.float32)
            for E in range(1, min(full, 15) + 1):
                hi_s, res_s = ref.split(x, fmt, E)                       # one slot per value
                hi_p, buf = ref.split(x, fmt, E, packed=True)
                assert buf.dtype == np.uint8 and buf.size == ref.res_bytes(n, fmt, E, True)
                # E bits per value and nothing more (up to the 16-byte rounding of each plane)
                assert buf.size <= (n * E + 7) // 8 + 4 * 16
                assert np.array_equal(hi_p, hi_s)
                assert np.array_equal(unpack_planes(buf, n, E), res_s.astype(np.uint32)), (fmt, n, E)
                assert np.array_equal(ref.merge(hi_p, buf, fmt, E, packed=True).view(np.uint32),
                                      ref.merge(hi_s, res_s, fmt, E).view(np.uint32))
    # rounded modes: NEAREST stores the same E bits; STOCHASTIC stores E + 1, the flag leading,
    # which is exactly the content of the slot (kept bits, flag just above them)
    for fmt, full in ((ref.BF16, 16), (ref.FP16, 13)):
        for n in (1, 7, 64, 1001):
            x = (rng.standard_normal(n) * 0.02).astype(np.float32)
            for E in (1, 2, 6, 7, 12, 13):
                hi_s, res_s = ref.split(x, fmt, E, ref.NEAREST)
                hi_p, buf = ref.split(x, fmt, E, ref.NEAREST, packed=True)
                assert np.array_equal(hi_p, hi_s) and np.array_equal(unpack_planes(buf, n, E), res_s.astype(np.uint32))
                assert np.array_equal(ref.merge(hi_p, buf, fmt, E, ref.NEAREST, packed=True).view(np.uint32),
                                      ref.merge(hi_s, res_s, fmt, E, ref.NEAREST).view(np.uint32))
                hi_s, res_s = ref.split(x, fmt, E, ref.STOCHASTIC, 99, 3)
                hi_p, buf = ref.split(x, fmt, E + 1, ref.STOCHASTIC, 99, 3, packed=True)
                assert buf.size == ref.res_bytes(n, fmt, E + 1, True)
                assert np.array_equal(hi_p, hi_s) and np.array_equal(unpack_planes(buf, n, E + 1), res_s.astype(np.uint32))
                assert np.array_equal(ref.merge(hi_p, buf, fmt, E + 1, ref.STOCHASTIC, packed=True).view(np.uint32),
                                      ref.merge(hi_s, res_s, fmt, E, ref.STOCHASTIC).view(np.uint32))
    # steps on packed storage hold the same values as steps on slots
    n = 1003
    x = (rng.standard_normal(n) * 0.02).astype(np.float32)
    for E in (12, 4, 10, 13, 7, 1):
        a_hi, a_res = ref.split(x, ref.BF16, E)
        b_hi, b_buf = ref.split(x, ref.BF16, E, packed=True)
        ma = np.zeros(n, np.float32); va = np.zeros(n, np.float32); mb = np.zeros(n, np.float32); vb = np.zeros(n, np.float32)
        sa_hi, sa_res = ref.split(x, ref.BF16, E)
        sb_hi, sb_buf = ref.split(x, ref.BF16, E, packed=True)
        ba = np.zeros(n, np.float32); bb = np.zeros(n, np.float32)
        for t in range(1, 6):
            g = rng.integers(0x3800, 0x3A00, n).astype(np.uint16)
            ref.adam_step(a_hi, a_res, g, ma, va, ref.AdamCfg(res_bits=E), t)
            ref.adam_step(b_hi, b_buf, g, mb, vb, ref.AdamCfg(res_bits=E, res_packed=True), t)
            ref.sgd_step(sa_hi, sa_res, g, ba, ref.SgdCfg(res_bits=E), t)
            ref.sgd_step(sb_hi, sb_buf, g, bb, ref.SgdCfg(res_bits=E, res_packed=True), t)
        assert np.array_equal(a_hi, b_hi) and np.array_equal(ma, mb) and np.array_equal(va, vb)
        assert np.array_equal(unpack_planes(b_buf, n, E), a_res.astype(np.uint32))
        assert np.array_equal(sa_hi, sb_hi) and np.array_equal(ba, bb)
        assert np.array_equal(unpack_planes(sb_buf, n, E), sa_res.astype(np.uint32))
    for E, rnd in ((13, ref.STOCHASTIC), (6, ref.STOCHASTIC), (11, ref.NEAREST)):
        S = E + (1 if rnd == ref.STOCHASTIC else 0)
        a_hi, a_res = ref.split(x, ref.FP16, E, rnd, 5, 9)
        b_hi, b_buf = ref.split(x, ref.FP16, S, rnd, 5, 9, packed=True)
        ma = np.zeros(n, np.float32); va = np.zeros(n, np.float32); mb = np.zeros(n, np.float32); vb = np.zeros(n, np.float32)
        for t in range(1, 5):
            g = rng.integers(0x1400, 0x1800, n).astype(np.uint16)
            ref.adam_step(a_hi, a_res, g, ma, va, ref.AdamCfg(weight_fmt=ref.FP16, grad_fmt=ref.FP16, res_bits=E, round=rnd, seed=5), t, tensor_id=9)
            ref.adam_step(b_hi, b_buf, g, mb, vb, ref.AdamCfg(weight_fmt=ref.FP16, grad_fmt=ref.FP16, res_bits=S, res_packed=True, round=rnd, seed=5), t, tensor_id=9)
        assert np.array_equal(a_hi, b_hi) and np.array_equal(ma, mb) and np.array_equal(va, vb)
        assert np.array_equal(unpack_planes(b_buf, n, S), a_res.astype(np.uint32))


def test_packed_storage(ref):
    pins_packed_storage(ref)
