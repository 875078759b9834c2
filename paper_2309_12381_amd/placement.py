"""Where the state arrays of a large model sit in HBM.

Measured on MI355X (288 GiB; profiles/stream_probe_placements_shapes_and_memory_counters.txt):
the memory behaves as three regions of 96 GiB.  A kernel that reads and writes several arrays
in lock step, as the optimizer step does with hi, res, m and v (Section 3.1 of arXiv
2309.12381: 26 bytes per parameter for Adam), runs at about 5.75 TB/s when every array it
WRITES lies in one region and at 6.45-6.5 TB/s when the written arrays are divided between
two regions (write-only traffic: 5.8-5.9 TB/s into one region, 7.1 TB/s into two); which
arrays share a region matters little otherwise (balanced writes are best by 1 %), a third
region is slower again (6.3), and moving only the gradients (read-only) changes nothing.
Allocations made one after the other in a fresh process fill the memory in order, so a model
whose state is below 96 GiB lands in one region unless its arrays are placed on purpose.
Once a process (or an earlier one on the same GPU) has freed large blocks, the driver no
longer hands memory out in order and large arrays tend to be spread over the regions anyway.

`place_second` takes the arrays that are already there (hi: the 16-bit weights, m) and a
function that allocates the others (res, v, grad); it allocates up to `max_tries` candidates
one after the other (at least 16 GiB apart, with filler blocks between small ones), all kept
until the choice is made (memory that is freed comes back in any order, so the only way to
reach another region is to hold what lies before it).  Each candidate is timed with the
bandwidth probe (csrc/stream_probe.hip) on windows at several matching positions of the
arrays, the way the step walks them; the search stops at the first candidate that shows the
gain of a second region (7 % on average over the positions, at least 4 % at each: a candidate that
straddles two regions shows the gain at one end only; one in the same region measures within 4 % of the reference); the fastest
candidate seen is kept and the others are freed.  What the search may hold on top of the
arrays it returns is bounded by `max_transient_bytes`.  Nothing here knows physical addresses:
every decision is a measurement, and the outcome is reported to the caller.
"""
from typing import Callable, Dict, Optional, Sequence, Tuple

import torch

from . import probe

GIB = 1 << 30
_TEST_PARAMS = 1 << 26              # parameters per probe launch: 1.75 GB of traffic, about 0.3 ms
_N2 = _TEST_PARAMS * 2              # bytes of a window of a 16-bit array
_N4 = _TEST_PARAMS * 4              # bytes of a window of an fp32 array
MIN_PARAMS = 1 << 28                # allocate_state: below this the state is not placed
_STRIDE = 16 * GIB                  # successive candidates start at least this far apart
_RESERVE = 4 * GIB                  # never take the last of the device memory


def _window(t: torch.Tensor, q: float, nbytes: int) -> torch.Tensor:
    """`nbytes` bytes of `t` at relative position q in [0, 1], 4 KiB aligned."""
    b = t.view(torch.uint8)
    off = int(q * (b.numel() - nbytes)) & ~4095
    return b[off:off + nbytes]


def _rate(hi, res, grad, m, v, stream) -> float:
    """GB/s of the probe over these five windows: median of 3 timed launches after one untimed."""
    probe.stream_probe(hi, res, grad, m, v, _TEST_PARAMS, stream)
    rates = []
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        probe.stream_probe(hi, res, grad, m, v, _TEST_PARAMS, stream)
        e1.record(stream)
        e1.synchronize()
        rates.append(26.0 * _TEST_PARAMS / e0.elapsed_time(e1) / 1e6)
    return sorted(rates)[1]


def _nbytes(t: torch.Tensor) -> int:
    return t.numel() * t.element_size()


def place_second(hi: torch.Tensor, m: torch.Tensor, make_second: Callable[[], Dict[str, torch.Tensor]], need: int,
                 gain: float = 1.07, floor: float = 1.04, max_tries: int = 8,
                 positions: Sequence[float] = (0.0, 1.0 / 3, 2.0 / 3, 1.0), max_transient_bytes: Optional[int] = None,
                 keep_hi: bool = False) -> Tuple[Dict[str, torch.Tensor], dict]:
    """Choose where res, v (and grad) go, given hi and m.

    hi            16-bit weights (any dtype of 2 bytes), at least 2^26 elements; the probe overwrites the
                  windows it uses unless `keep_hi` (then they are saved and restored: a model's weights).
    m             fp32, at least 6 * 2^25 elements (the one-region reference takes four of its five windows from it);
                  overwritten (clear it afterwards).
    make_second   allocates and returns {"res": ..., "v": ..., and optionally "grad": ...}; res at least 2^27 bytes
                  (a 16-bit window), v fp32 of at least 2^26 elements.  Called once per candidate.
    need          bytes one call of make_second allocates.
    max_transient_bytes  most the search may hold beyond one candidate (default: half of the free memory at entry).
    Returns (the chosen candidate, report); report["split"] says whether the probe saw the gain of a second
    region (`gain` on average over the tested positions, `floor` at each of them) for the candidate kept;
    report["peak_transient_bytes"] what the search held at most beyond the candidate it returns."""
    dev = m.device
    if _nbytes(hi) < _N2 or _nbytes(m) < 6 * _N2:
        return make_second(), {"split": False, "why": "arrays too small to probe", "peak_transient_bytes": 0}
    stream = torch.cuda.current_stream(dev)
    free0, _ = torch.cuda.mem_get_info(dev)
    if max_transient_bytes is None:
        max_transient_bytes = free0 // 2

    saved = {}

    def hi_window(q):
        w = _window(hi, q, _N2)
        if keep_hi and q not in saved:
            saved[q] = (w, w.clone())
        return w

    try:
        # reference: the same hi windows the candidates are measured with, everything else inside m, i.e.
        # certainly close together (hi and m are taken to lie in one region: m is allocated right after hi)
        one_region = []
        for q in positions:
            w = _window(m, q, 6 * _N2)
            one_region.append(_rate(hi_window(q), w[:_N2], w[_N2:2 * _N2], w[2 * _N2:2 * _N2 + _N4], w[2 * _N2 + _N4:], stream))

        def measure(c):
            out = []
            for q in positions:
                g = c.get("grad")
                if g is not None and _nbytes(g) >= _N2:
                    grad_w = _window(g, 0.0, _N2)
                else:
                    # no gradient array to read from: a part of m away from the m window (where read-only data
                    # lie does not matter; reading the res window twice would save a sixth of the reads and
                    # make every candidate look better than it is)
                    grad_w = _window(m, q + 0.5 if q <= 0.5 else q - 0.5, _N2)
                out.append(_rate(hi_window(q), _window(c["res"], q, _N2), grad_w, _window(m, q, _N4), _window(c["v"], q, _N4),
                                 stream))
            return out

        def good(r):
            """The gain of a second region: `gain` on average over the positions, `floor` at each."""
            return sum(r) >= gain * sum(one_region) and all(s >= floor * p for s, p in zip(r, one_region))

        cands, rates, fillers = [], [], []
        held = 0                                            # bytes of candidates and fillers held so far
        while len(cands) < max_tries:
            step = need + (max(0, _STRIDE - need) if cands else 0)
            free, _ = torch.cuda.mem_get_info(dev)
            if free < step + _RESERVE:
                break
            if cands and held + step - need > max_transient_bytes:
                break                                       # one more candidate would hold too much
            # nothing is freed during the search: freed memory comes back in any order
            if cands and need < _STRIDE:
                fillers.append(torch.empty(_STRIDE - need, dtype=torch.uint8, device=dev))
            cands.append(make_second())
            held += step
            rates.append(measure(cands[-1]))
            if good(rates[-1]):
                break
        if not cands:
            return make_second(), {"split": False, "why": "no memory to search with", "peak_transient_bytes": 0}
        best = max(range(len(cands)), key=lambda i: sum(rates[i]))
        chosen = cands[best]
        del cands, fillers
        torch.cuda.empty_cache()            # the candidates not chosen go back to the driver
        split = good(rates[best])
        report = {"split": split, "candidates": len(rates), "chosen": best,
                  "probe_GBps_one_region": [round(x) for x in one_region],
                  "probe_GBps_per_candidate": [[round(x) for x in r] for r in rates],
                  "peak_transient_bytes": held - need, "max_transient_bytes": max_transient_bytes}
        if not split:
            report["why"] = "no candidate with the gain of a second region at every position; fastest kept"
        return chosen, report
    finally:
        for w, copy in saved.values():
            w.copy_(copy)
        saved.clear()


def allocate_state(n: int, res_spec: Tuple[int, torch.dtype], grad_spec: Tuple[int, torch.dtype], device="cuda:0",
                   zero_res: bool = False, place: bool = True, gain: float = 1.07, floor: float = 1.04, max_tries: int = 8,
                   positions: Sequence[float] = (0.0, 1.0 / 3, 2.0 / 3, 1.0),
                   max_transient_bytes: Optional[int] = None) -> Tuple[Dict[str, torch.Tensor], dict]:
    """Allocate hi (int16) and m, v (fp32, cleared) of n elements, res and grad as specified
    ((elements, dtype); grad cleared, res cleared if `zero_res`).  With `place`, and n at least
    2^28, (res, v, grad) are placed in another HBM region than (hi, m) when the probe can find one
    (see place_second, which the remaining arguments go to).
    Returns ({"hi","res","grad","m","v"}, report)."""
    dev = torch.device(device)

    def second():
        return {"res": torch.empty(res_spec[0], dtype=res_spec[1], device=dev),
                "v": torch.empty(n, dtype=torch.float32, device=dev),
                "grad": torch.empty(grad_spec[0], dtype=grad_spec[1], device=dev)}

    def finish(arrays, report):
        for name in ("m", "v", "grad") + (("res",) if zero_res else ()):
            arrays[name].zero_()
        return arrays, report

    arrays = {"hi": torch.empty(n, dtype=torch.int16, device=dev), "m": torch.empty(n, dtype=torch.float32, device=dev)}
    res_bytes = res_spec[0] * torch.empty((), dtype=res_spec[1]).element_size()
    grad_bytes = grad_spec[0] * torch.empty((), dtype=grad_spec[1]).element_size()
    if not place or n < MIN_PARAMS or res_bytes < _N2:
        arrays.update(second())
        return finish(arrays, {"split": False, "why": "placement switched off" if not place else "state too small to place"})
    chosen, report = place_second(arrays["hi"], arrays["m"], second, res_bytes + 4 * n + grad_bytes, gain=gain, floor=floor,
                                  max_tries=max_tries, positions=positions, max_transient_bytes=max_transient_bytes)
    arrays.update(chosen)
    return finish(arrays, report)
