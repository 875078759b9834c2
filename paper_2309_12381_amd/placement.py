"""Where the state arrays of a large model sit in HBM.

Measured on MI355X (288 GiB): the memory behaves as three regions of 96 GiB.  A kernel
that reads and writes several arrays in lock step, as the optimizer step does with hi,
res, m and v (Section 3.1 of arXiv 2309.12381: 26 bytes per parameter for Adam), runs at
about 5.6 TB/s when every array it WRITES lies in one region and at 6.4-6.5 TB/s when
the written arrays are divided between two regions; which arrays share a region does not
matter otherwise, a third region adds nothing, and moving only the gradients (read-only)
changes nothing.  Allocations made one after the other in a fresh process fill the
memory in order, so a model whose state is below 96 GiB lands in one region unless its
arrays are placed on purpose.  Once a process (or an earlier one on the same GPU) has
freed large blocks, the driver no longer hands memory out in order and large arrays tend
to be spread over the regions anyway.

`allocate_state` allocates hi and m first, then up to `max_tries` candidates for
(res, v, grad) one after the other (at least 16 GiB apart, with filler blocks between
small ones), all kept until the choice is made.  Each candidate
is timed with the bandwidth probe (csrc/stream_probe.hip) on windows at several matching
positions of the arrays, the way the step walks them; the search stops at the first
candidate that shows the gain of a second region (8 % on average over the positions, at
least 4 % at each); the fastest candidate seen is kept and the others are freed.  Nothing here knows physical addresses:
every decision is a measurement, and the outcome is reported to the caller.
"""
from typing import Dict, Sequence, Tuple

import torch

from . import probe

GIB = 1 << 30
_TEST_PARAMS = 1 << 26              # parameters per probe launch: 1.75 GB of traffic, about 0.3 ms
_N2 = _TEST_PARAMS * 2              # bytes of a window of a 16-bit array
_N4 = _TEST_PARAMS * 4              # bytes of a window of an fp32 array
MIN_PARAMS = 1 << 28                # below this the state is not placed (the windows must fit)
_STRIDE = 16 * GIB                  # successive candidates start at least this far apart


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


def allocate_state(n: int, res_spec: Tuple[int, torch.dtype], grad_spec: Tuple[int, torch.dtype], device="cuda:0",
                   zero_res: bool = False, place: bool = True, gain: float = 1.08, floor: float = 1.04, max_tries: int = 8,
                   positions: Sequence[float] = (0.0, 1.0 / 3, 2.0 / 3, 1.0)) -> Tuple[Dict[str, torch.Tensor], dict]:
    """Allocate hi (int16) and m, v (fp32, cleared) of n elements, res and grad as specified
    ((elements, dtype); grad cleared, res cleared if `zero_res`).  With `place`, and n at least
    2^28, (res, v, grad) are placed in another HBM region than (hi, m) when the probe can find one.
    Returns ({"hi","res","grad","m","v"}, report): report["split"] says whether the probe saw the
    gain of a second region (`gain` on average over the tested positions, `floor` at each of them)
    for the arrays it kept, with the rates it measured."""
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

    stream = torch.cuda.current_stream(dev)
    hi, m = arrays["hi"], arrays["m"]
    # reference: all five windows inside m, i.e. certainly close together
    one_region = []
    for q in positions:
        w = _window(m, q, 7 * _N2)
        one_region.append(_rate(w[:_N2], w[_N2 + _N4:2 * _N2 + _N4], w[2 * _N2 + _N4:3 * _N2 + _N4],
                                w[_N2:_N2 + _N4], w[3 * _N2 + _N4:], stream))

    def measure(c):
        out = []
        for q in positions:
            res_w = _window(c["res"], q, _N2)
            grad_w = _window(c["grad"], 0.0, _N2) if grad_bytes >= _N2 else res_w   # read-only: may alias
            out.append(_rate(_window(hi, q, _N2), res_w, grad_w, _window(m, q, _N4), _window(c["v"], q, _N4), stream))
        return out

    def good(r):
        """The gain of a second region: `gain` on average over the positions, `floor` at each."""
        return sum(r) >= gain * sum(one_region) and all(s >= floor * p for s, p in zip(r, one_region))

    need = res_bytes + 4 * n + grad_bytes
    cands, rates, fillers = [], [], []
    found = False
    while len(cands) < max_tries:
        free, _ = torch.cuda.mem_get_info(dev)
        if free < max(need, _STRIDE) + (4 << 30):
            break
        # nothing is freed during the search: freed memory comes back in any order
        if cands and need < _STRIDE:
            fillers.append(torch.empty(_STRIDE - need, dtype=torch.uint8, device=dev))
        cands.append(second())
        rates.append(measure(cands[-1]))
        if good(rates[-1]):
            found = True
            break
    if not cands:
        arrays.update(second())
        return finish(arrays, {"split": False, "why": "no memory to search with"})
    best = max(range(len(cands)), key=lambda i: sum(rates[i]))
    chosen = cands[best]
    del cands, fillers
    torch.cuda.empty_cache()            # the candidates not chosen go back to the driver
    arrays.update(chosen)
    split = good(rates[best])
    report = {"split": split, "candidates": len(rates), "chosen": best,
              "probe_GBps_one_region": [round(x) for x in one_region],
              "probe_GBps_per_candidate": [[round(x) for x in r] for r in rates]}
    if not split:
        report["why"] = "no candidate with the gain of a second region at every position; fastest kept"
    return finish(arrays, report)
