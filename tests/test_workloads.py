"""The synthetic parameter sets (shapes stated by the benchmark configurations) and the plan the
library builds over them, on the CPU: counts, layer structure, chunk tables."""
import numpy as np
import pytest

import paper_2309_12381_amd as mpo
from paper_2309_12381_amd import synth

EXPECT = {                      # key: (tensors, parameters, layers)
    "c0": (1, 1_048_576, 1),
    "c1": (161, 25_600_000, 54),
    "c2": (292, 354_823_168, 26),
    "c3": (291, 6_738_415_616, 35),
    "c4": (363, 13_015_864_320, 43),
}


@pytest.mark.parametrize("key", sorted(EXPECT))
def test_shapes_and_counts(key):
    wl = synth.workload(key)
    nt, params, layers = EXPECT[key]
    assert len(wl.tensors) == nt and wl.num_params == params
    assert len(wl.layers_backward) == layers and wl.layers_backward == sorted(wl.layers_backward, reverse=True)
    assert all(t.n >= 1 for t in wl.tensors)
    assert wl.fmt == ("fp16" if key == "c4" else "bf16") and wl.loss_scale == (1024.0 if key == "c4" else 1.0)
    assert wl.per_layer == (key in ("c3", "c4"))


def test_c1_sizes_are_seeded_log_uniform_and_odd():
    a = [t.n for t in synth.workload("c1").tensors]
    b = [t.n for t in synth.workload("c1").tensors]
    assert a == b                                               # seeded
    assert min(a) >= 1 and max(a) < 4_000_000
    assert sum(1 for n in a if n % 8) > 100                     # ragged ends and odd lengths on purpose
    logs = np.log(np.array(a[:-1], float))
    assert logs.std() > 2.0                                      # spread over several orders of magnitude


def test_llama_layers_hold_what_a_block_holds():
    wl = synth.workload("c3")
    h, inter = 4096, 11008
    block = [t.n for t in wl.tensors if t.layer == 7]
    assert sorted(block) == sorted([h, h, h * h, h * h, h * h, h * h, h * inter, h * inter, inter * h])
    assert [t.n for t in wl.tensors if t.layer == 0] == [32000 * h]              # embedding: last in backward
    assert [t.n for t in wl.tensors if t.layer == 34] == [32000 * h]             # head: first in backward
    assert [t.n for t in wl.tensors if t.layer == 33] == [h]                     # final norm


@pytest.mark.parametrize("key", ["c1", "c3"])
def test_host_plan_over_a_workload(key):
    """Chunk table of the whole list (made-up, disjoint addresses: a host plan never touches them)."""
    wl = synth.workload(key)
    at = 1 << 24
    specs = []
    for t in wl.tensors:
        ptrs = []
        for width in (2, 2, 2, 4, 4):
            ptrs.append(at)
            at += (t.n * width + 255) // 256 * 256
        specs.append(mpo.Tensor(ptrs[0], ptrs[1], ptrs[2], ptrs[3], ptrs[4], t.n, t.layer))
    plan = mpo.Plan(specs, host_only=True)
    assert plan.num_params == wl.num_params
    total = 0
    for layer in wl.layers_backward:
        info = plan.layer_info(layer)
        mine = [t.n for t in wl.tensors if t.layer == layer]
        assert info["num_tensors"] == len(mine) and info["num_params"] == sum(mine)
        chunk = info["chunk_elems"]
        assert chunk == 1024                                  # the default cut: one row per workgroup
        assert info["num_chunks"] == sum((n + chunk - 1) // chunk for n in mine)
        total += info["num_chunks"]
    assert total == plan.num_chunks
    # the table goes layer by layer
    first = plan.chunk(0)
    assert wl.tensors[first[0]].layer == min(t.layer for t in wl.tensors)
    last = plan.chunk(plan.num_chunks - 1)
    assert wl.tensors[last[0]].layer == max(t.layer for t in wl.tensors)
    plan.destroy()
