"""The bandwidth probe and the placement of the state arrays over HBM regions.

The probe is a measuring aid, not part of the method: what is checked here is that it touches
exactly the elements it says it touches, and that `allocate_state` hands out clean, disjoint
arrays whatever its search did."""
import pytest
import torch

from paper_2309_12381_amd import placement, probe

from gpu_util import DEV, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [0, 100, 4096, 3 * 4096 + 5, 64 * 4096])
@pytest.mark.parametrize("with_v", [True, False])
def test_probe_touches_whole_chunks_only(n, with_v):
    say("probe n=%d with_v=%s" % (n, with_v))
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    size = n + 4096                                   # room to see that nothing past the end moves
    hi = torch.randint(-30000, 30000, (size,), dtype=torch.int16, device=DEV, generator=g)
    res = torch.randint(-30000, 30000, (size,), dtype=torch.int16, device=DEV, generator=g)
    grad = torch.randint(-30000, 30000, (size,), dtype=torch.int16, device=DEV, generator=g)
    m = torch.randn(size, device=DEV, generator=g)
    v = torch.randn(size, device=DEV, generator=g)
    before = [t.clone() for t in (hi, res, grad, m, v)]
    probe.stream_probe(hi, res, grad, m, v if with_v else None, n, torch.cuda.current_stream())
    torch.cuda.synchronize()
    k = n - n % 4096
    assert torch.equal(hi[:k], before[0][:k] ^ before[2][:k]) and torch.equal(hi[k:], before[0][k:])
    assert torch.equal(res[:k], ~(before[1][:k] ^ before[2][:k])) and torch.equal(res[k:], before[1][k:])
    assert torch.equal(grad, before[2])
    assert torch.equal(m[:k], before[3][:k] + 1.0) and torch.equal(m[k:], before[3][k:])
    if with_v:
        assert torch.equal(v[:k], before[4][:k] + 2.0) and torch.equal(v[k:], before[4][k:])
    else:
        assert torch.equal(v, before[4])


def test_probe_rejects_bad_arguments():
    a = torch.zeros(8192, dtype=torch.int16, device=DEV)
    f = torch.zeros(8192, dtype=torch.float32, device=DEV)
    with pytest.raises(RuntimeError):
        probe.stream_probe(a[1:], a, a, f, f, 4096)          # not 16-byte aligned
    with pytest.raises(RuntimeError):
        probe.stream_probe(a, a, a, f, f, -1)


def _disjoint(arrays):
    spans = sorted((t.data_ptr(), t.data_ptr() + t.numel() * t.element_size()) for t in arrays.values())
    return all(spans[i][1] <= spans[i + 1][0] for i in range(len(spans) - 1))


def test_small_state_is_allocated_plainly():
    arrays, report = placement.allocate_state(1000, (1000, torch.int16), (1000, torch.bfloat16), DEV)
    assert report["split"] is False and "small" in report["why"]
    assert set(arrays) == {"hi", "res", "grad", "m", "v"} and _disjoint(arrays)
    assert not arrays["m"].any() and not arrays["v"].any() and not arrays["grad"].view(torch.int16).any()


@pytest.mark.parametrize("res_dtype,zero_res", [(torch.int16, False), (torch.uint8, True)])
def test_placed_state_is_clean_and_disjoint(res_dtype, zero_res):
    """2^28 parameters (3.2 GB of state): large enough for the search to run.  Whatever it found,
    the arrays are the right size, do not overlap, and those that must start at zero do."""
    n = 1 << 28
    say("allocate_state n=2^28 res=%s" % res_dtype)
    free0, _ = torch.cuda.mem_get_info()
    arrays, report = placement.allocate_state(n, (n, res_dtype), (1 << 26, torch.bfloat16), DEV, zero_res=zero_res)
    print(report)
    assert report["candidates"] >= 1 and 0 <= report["chosen"] < report["candidates"]
    assert len(report["probe_GBps_one_region"]) == 4 and all(len(r) == 4 for r in report["probe_GBps_per_candidate"])
    assert arrays["hi"].numel() == n and arrays["hi"].dtype == torch.int16
    assert arrays["res"].numel() == n and arrays["res"].dtype == res_dtype
    assert arrays["m"].numel() == n and arrays["v"].numel() == n and arrays["grad"].numel() == 1 << 26
    assert _disjoint(arrays)
    assert not arrays["m"].any() and not arrays["v"].any() and not arrays["grad"].view(torch.int16).any()
    if zero_res:
        assert not arrays["res"].any()
    # the candidates that were not chosen went back to the driver
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    held = sum(t.numel() * t.element_size() for t in arrays.values())
    assert free0 - free1 < held + (1 << 30)
    del arrays
    torch.cuda.empty_cache()


def test_search_holds_no_more_than_it_is_allowed():
    """The search reaches another region only by holding the memory before it; what it holds beyond the
    arrays it returns is bounded by max_transient_bytes (here: room for one more candidate)."""
    n = 1 << 28
    need = 2 * n + 4 * n + 2 * (1 << 26)                      # res + v + grad of one candidate
    say("allocate_state n=2^28 with a bound on transient memory")
    torch.cuda.empty_cache()
    torch.cuda.synchronize()
    base = torch.cuda.memory_allocated()
    torch.cuda.reset_peak_memory_stats()
    bound = 17 << 30                                          # one stride: a filler and a second candidate
    arrays, report = placement.allocate_state(n, (n, torch.int16), (1 << 26, torch.bfloat16), DEV, max_transient_bytes=bound)
    print(report)
    final = sum(t.numel() * t.element_size() for t in arrays.values())
    peak = torch.cuda.max_memory_allocated() - base
    assert report["peak_transient_bytes"] <= bound and report["candidates"] <= 2
    assert peak <= final + bound + (1 << 30), (peak, final, bound)        # 1 GiB: the probe's own event and window slack
    assert _disjoint(arrays) and not arrays["m"].any() and not arrays["v"].any()
    del arrays
    torch.cuda.empty_cache()
    # and with no room at all it still allocates, plainly
    arrays, report = placement.allocate_state(n, (n, torch.int16), (1 << 26, torch.bfloat16), DEV, max_transient_bytes=0)
    assert report["candidates"] == 1 and report["peak_transient_bytes"] == 0 and _disjoint(arrays)
    del arrays
    torch.cuda.empty_cache()


def test_placement_can_be_switched_off():
    n = 1 << 28
    arrays, report = placement.allocate_state(n, (n, torch.int16), (4096, torch.float16), DEV, place=False)
    assert report == {"split": False, "why": "placement switched off"} and _disjoint(arrays)
    assert not arrays["m"].any() and not arrays["v"].any()
    del arrays
    torch.cuda.empty_cache()


def test_native_search_returns_a_block_restores_the_weights_and_keeps_its_bound():
    """mpo_place_second (the same search behind the C interface, on hipMalloc'ed blocks): whatever it finds, it
    returns one block of the size asked for, frees the rest, leaves hi as it was, and holds no more than allowed."""
    n = 1 << 28
    need = 2 * n + 4 * n + 2 * (1 << 26)
    say("mpo_place_second n=2^28")
    g = torch.Generator(device=DEV)
    g.manual_seed(11)
    hi = torch.randint(-30000, 30000, (n,), dtype=torch.int16, device=DEV, generator=g)
    m = torch.empty(n, dtype=torch.float32, device=DEV)
    before = hi.clone()
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    bound = 17 << 30
    block, report = probe.place_second_native(hi, m, 2 * n, 4 * n, 2 * (1 << 26), max_transient_bytes=bound, keep_hi=True)
    print(report)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert block and block % 256 == 0
    assert report["v_offset"] == 2 * n and report["grad_offset"] == 6 * n and report["block_bytes"] == need
    assert 1 <= report["candidates"] <= 2 and 0 <= report["chosen"] < report["candidates"]
    assert report["peak_transient_bytes"] <= bound and report["max_transient_bytes"] == bound
    assert all(3000.0 < r < 8000.0 for r in report["one_region_GBps"] + report["chosen_GBps"])
    assert torch.equal(hi, before)
    assert need - (64 << 20) <= free0 - free1 < need + (1 << 30)            # only the returned block is still held
    probe.place_free(block)
    free2, _ = torch.cuda.mem_get_info()
    assert free0 - free2 < (1 << 30)
    # arrays too small to probe: a plain allocation
    block, report = probe.place_second_native(hi[:4096], m, 2 * n, 4 * n, 1000)
    assert block and report["split"] is False and report["candidates"] == 1 and report["peak_transient_bytes"] == 0
    probe.place_free(block)
    with pytest.raises(RuntimeError):
        probe.place_second_native(hi, m, 0, 4 * n, 0)
