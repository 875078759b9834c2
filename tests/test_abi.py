"""CPU-only checks of libmpo.so: it loads, exports everything include/mpo.h declares,
validates arguments before touching the GPU, and lays plans out as documented.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

import paper_2309_12381_amd as mpo
from paper_2309_12381_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "mpo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mpo_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    for required in ("mpo_split", "mpo_merge", "mpo_adam_step", "mpo_sgd_step", "mpo_step_layer",
                     "mpo_plan_create", "mpo_plan_destroy"):
        assert required in names
    for n in names:
        assert hasattr(mpo.lib, n), n
        assert n in binding.EXPORTS, "binding does not cover " + n


def test_probe_library_exports_what_its_header_declares():
    text = open(os.path.join(ROOT, "include", "mpo_probe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(mpo_[a-z_0-9]+)\s*\(", text)))
    assert "mpo_probe_stream" in names and "mpo_place_second" in names and len(names) == 7
    from paper_2309_12381_amd import probe
    lib = probe._load()
    for n in names:
        assert hasattr(lib, n), n
    # argument checks that need no GPU
    assert lib.mpo_probe_stream(None, None, None, None, None, 4096, None) == -1
    assert lib.mpo_place_second(None, 0, None, 0, 0, 0, 0, 0, 0, None, None, None) == -1
    assert lib.mpo_place_free(None) == 0


def test_status_strings():
    seen = set()
    for s in range(7):
        msg = mpo.lib.mpo_status_string(s).decode()
        assert msg and msg not in seen
        seen.add(msg)
    assert mpo.lib.mpo_status_string(99).decode() == "unknown status"


A = 0x10000000  # fake, well separated, 16-byte aligned device addresses: never dereferenced on the host


def T(i=0, n=1000, layer=0, **kw):
    base = A + i * 0x1000000
    d = dict(hi=base, res=base + 0x100000, grad=base + 0x200000, m=base + 0x300000, v=base + 0x400000, n=n, layer=layer)
    d.update(kw)
    return mpo.Tensor(**d)


def _status(fn, *a, **k):
    try:
        fn(*a, **k)
    except mpo.MpoError as e:
        return e.status
    return mpo.MPO_OK


def test_split_merge_argument_validation():
    # nothing is enqueued when validation fails, so fake addresses are fine
    assert _status(mpo.mpo_split, 0, A, A + 0x1000, 10) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_split, A, 0, A + 0x1000, 10) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x2000, 10, fmt=7) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x2000, 10, round=5) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_merge, A, A + 0x1000, A + 0x2000, 10, round=-1) == mpo.MPO_ERR_INVALID_ARG
    # stochastic rounding stores a flag above the kept bits: 8 + 1 do not fit a byte, 16 + 1 not 16 bits
    S = mpo.MPO_ROUND_STOCHASTIC
    assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x2000, 10, res_bits=8, round=S) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x2000, 10, res_bits=16, round=S) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_merge, A, A + 0x1000, A + 0x2000, 10, res_bits=8, round=S) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x2000, 1 << 60) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_split, A, A + 16, A + 0x2000, 10) == mpo.MPO_ERR_ALIAS       # hi inside w32
    assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x1000 + 10, 10) == mpo.MPO_ERR_ALIAS  # res inside hi
    assert _status(mpo.mpo_merge, A, A + 0x1000, A + 0x1000 + 8, 10) == mpo.MPO_ERR_ALIAS
    assert _status(mpo.mpo_merge, A, A + 0x1000, 0, 10) == mpo.MPO_ERR_INVALID_ARG
    # extra bits kept: 0 = all, else 1..16 (bf16) / 1..13 (fp16); a byte per element up to 8
    assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x2000, 10, res_bits=17) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x2000, 10, res_bits=-1) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x2000, 10, fmt=mpo.MPO_FP16, res_bits=14) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_merge, A, A + 0x1000, A + 0x2000, 10, fmt=mpo.MPO_FP16, res_bits=16) == mpo.MPO_ERR_INVALID_ARG
    # res [A+0x1000, +10 bytes) with 8 bits does not reach hi at A+0x100a; with 16 bits it does
    assert _status(mpo.mpo_split, A, A + 0x100a, A + 0x1000, 10, res_bits=9) == mpo.MPO_ERR_ALIAS
    # packed planes: 1 to 15 stored bits, 16-byte aligned buffer
    for bad in (0, 16, -2):
        assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x2000, 10, res_bits=bad, res_packed=True) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_merge, A, A + 0x1004, A + 0x2000, 10, res_bits=12, res_packed=True) == mpo.MPO_ERR_INVALID_ARG
    # ... of which at least one and at most the format's are kept bits; with stochastic rounding one is the flag
    assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x2000, 10, fmt=mpo.MPO_FP16, res_bits=14, res_packed=True) \
        == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x2000, 10, fmt=mpo.MPO_FP16, res_bits=14, res_packed=True,
                   round=mpo.MPO_ROUND_NEAREST) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_split, A, A + 0x1000, A + 0x2000, 10, fmt=mpo.MPO_FP16, res_bits=15, res_packed=True,
                   round=mpo.MPO_ROUND_STOCHASTIC) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_merge, A, A + 0x1000, A + 0x2000, 10, res_bits=1, res_packed=True,
                   round=mpo.MPO_ROUND_STOCHASTIC) == mpo.MPO_ERR_INVALID_ARG
    # zero elements: a legal no-op even with null pointers
    assert _status(mpo.mpo_split, 0, 0, 0, 0) == mpo.MPO_OK
    assert _status(mpo.mpo_merge, 0, 0, 0, 0, fmt=mpo.MPO_FP16) == mpo.MPO_OK


def _host_plan(ts):
    return mpo.Plan(ts, host_only=True)


def test_plan_validation():
    assert _status(_host_plan, [T(hi=0)]) == mpo.MPO_ERR_INVALID_ARG
    assert _status(_host_plan, [T(res=0)]) == mpo.MPO_ERR_INVALID_ARG
    assert _status(_host_plan, [T(layer=-1)]) == mpo.MPO_ERR_INVALID_ARG
    assert _status(_host_plan, [T(n=1 << 50)]) == mpo.MPO_ERR_INVALID_ARG
    # optional buffers may be absent at creation
    assert _status(_host_plan, [T(grad=0, v=0)]) == mpo.MPO_OK
    assert _status(_host_plan, [T(m=0, v=0)]) == mpo.MPO_OK
    assert _status(_host_plan, [T(res_bits=17)]) == mpo.MPO_ERR_INVALID_ARG
    assert _status(_host_plan, [T(res_bits=-2)]) == mpo.MPO_ERR_INVALID_ARG
    assert _status(_host_plan, [T(0, res_bits=8), T(1, res_bits=3)]) == mpo.MPO_OK          # both in bytes
    assert _status(_host_plan, [T(0, res_bits=12), T(1, res_bits=0)]) == mpo.MPO_OK         # both in 16 bits
    assert _status(_host_plan, [T(0, res_bits=8), T(1, res_bits=0)]) == mpo.MPO_ERR_UNSUPPORTED   # mixed widths
    # a zero-length tensor needs no pointers
    assert _status(_host_plan, [T(n=0, hi=0, res=0, grad=0, m=0, v=0)]) == mpo.MPO_OK
    assert _status(_host_plan, []) == mpo.MPO_OK


def test_res_bytes():
    assert mpo.mpo_res_bytes(1000) == 2000 and mpo.mpo_res_bytes(1000, 8) == 1000 and mpo.mpo_res_bytes(1000, 9) == 2000
    r16 = lambda x: (x + 15) // 16 * 16
    assert mpo.mpo_res_bytes(1000, 12, True) == r16(1000) + r16(500)             # 1.5 bytes per parameter
    assert mpo.mpo_res_bytes(1001, 14, True) == r16(1001) + r16(501) + r16(251)
    assert mpo.mpo_res_bytes(7, 2, True) == 16 and mpo.mpo_res_bytes(1 << 30, 4, True) == 1 << 29
    # a packed list: the next tensor may start right after the planes, not before
    a = T(0, n=1000, res_bits=12, res_packed=True)
    nb = mpo.mpo_res_bytes(1000, 12, True)
    assert _status(_host_plan, [a, T(1, res_bits=12, res_packed=True, hi=a.res + nb)]) == mpo.MPO_OK
    assert _status(_host_plan, [a, T(1, res_bits=12, res_packed=True, hi=a.res + nb - 2)]) == mpo.MPO_ERR_ALIAS
    assert _status(_host_plan, [a, T(1, res_bits=12)]) == mpo.MPO_ERR_UNSUPPORTED           # packed and slots mixed
    assert _status(_host_plan, [T(0, res_bits=0, res_packed=True)]) == mpo.MPO_ERR_INVALID_ARG
    assert _status(_host_plan, [T(0, res_bits=16, res_packed=True)]) == mpo.MPO_ERR_INVALID_ARG
    assert _status(_host_plan, [T(0, res_bits=5, res_packed=True)]) == mpo.MPO_OK
    assert _status(_host_plan, [T(0, res_bits=12, res_packed=True, res=A + 0x100008)]) == mpo.MPO_ERR_INVALID_ARG


def test_plan_alias_detection():
    a, b = T(0), T(1)
    assert _status(_host_plan, [a, b]) == mpo.MPO_OK
    assert _status(_host_plan, [a, a]) == mpo.MPO_ERR_ALIAS                       # tied weights listed twice
    assert _status(_host_plan, [a, T(1, hi=a.hi + 1998)]) == mpo.MPO_ERR_ALIAS    # last element of a.hi
    assert _status(_host_plan, [a, T(1, hi=a.hi + 2000)]) == mpo.MPO_OK           # just past it
    assert _status(_host_plan, [a, T(1, m=a.v + 3996)]) == mpo.MPO_ERR_ALIAS
    assert _status(_host_plan, [a, T(1, grad=a.m)]) == mpo.MPO_ERR_ALIAS          # gradient over written state
    assert _status(_host_plan, [T(0, grad=a.hi)]) == mpo.MPO_ERR_ALIAS
    # byte residuals take n bytes, not 2n: the next array may start right after them
    assert _status(_host_plan, [T(0, res_bits=8), T(1, res_bits=8, hi=a.res + 1000)]) == mpo.MPO_OK
    assert _status(_host_plan, [T(0, res_bits=9), T(1, res_bits=9, hi=a.res + 1000)]) == mpo.MPO_ERR_ALIAS
    # gradients may share one buffer (one layer's gradient alive at a time)
    assert _status(_host_plan, [a, T(1, grad=a.grad), T(2, grad=a.grad + 10)]) == mpo.MPO_OK
    # a written range nested inside a long read-only range that starts earlier
    assert _status(_host_plan, [T(0, grad=A - 0x100, n=1000), T(1, hi=A - 0x80, n=8)]) == mpo.MPO_ERR_ALIAS


def test_plan_layout_covers_every_element_once_in_layer_order():
    ce0 = _host_plan([]).chunk_elems
    small = 1024                                    # chunk length in layers below 2^26 parameters
    big = (1 << 26) + 5                             # one layer large enough for the long chunks
    sizes = [1, ce0 - 1, ce0, ce0 + 1, 3 * ce0 + 5, 0, 100000, 64, big, 4096 * 3 + 1]
    layers = [3, 0, 2, 0, 1, 1, 2, 0, 5, 5]
    ts = [T(i, n=n, layer=l) for i, (n, l) in enumerate(zip(sizes, layers))]
    far = 0x100000000000                            # the large tensor needs room: arrays 1 GiB apart
    ts[8] = T(8, n=big, layer=5, hi=far, res=far + (1 << 30), grad=far + (2 << 30), m=far + (3 << 30), v=far + (4 << 30))
    p = mpo.Plan(ts, host_only=True, small_layer_params=1 << 26)     # mixed: long chunks from 2^26 parameters on
    assert p.chunk_elems == ce0 == 4096
    assert p.num_params == sum(sizes)
    clen = {l: (ce0 if sum(n for n, l2 in zip(sizes, layers) if l2 == l) >= (1 << 26) else small) for l in set(layers)}
    assert p.num_chunks == sum((n + clen[l] - 1) // clen[l] for n, l in zip(sizes, layers))
    covered = {t: [] for t in range(len(sizes))}
    order = []
    for i in range(p.num_chunks):
        t, first, count = p.chunk(i)
        ce = clen[layers[t]]
        assert first % ce == 0 and 1 <= count <= ce and first + count <= sizes[t]
        assert count == ce or first + count == sizes[t]          # only a tensor's last chunk is shorter
        covered[t].append((first, count))
        order.append((layers[t], count != ce, t, first))
    for t, n in enumerate(sizes):                                 # every element exactly once
        at = 0
        for first, count in sorted(covered[t]):
            assert first == at
            at += count
        assert at == n
    # launch order: by layer; in a layer the ragged chunks first, then full chunks by tensor, ascending
    assert order == sorted(order, key=lambda k: (k[0], not k[1], k[2], k[3]))
    for layer in set(layers):
        info = p.layer_info(layer)
        members = [t for t in range(len(sizes)) if layers[t] == layer]
        assert info["num_tensors"] == len(members)
        assert info["num_params"] == sum(sizes[t] for t in members)
        assert info["chunk_elems"] == clen[layer]
        rng = [k[2] for k in order[info["first_chunk"]: info["first_chunk"] + info["num_chunks"]]]
        assert set(rng) <= set(members)
        assert info["num_chunks"] == sum((sizes[t] + clen[layer] - 1) // clen[layer] for t in members)
    assert _status(p.layer_info, 7) == mpo.MPO_ERR_INVALID_ARG
    assert _status(p.chunk, p.num_chunks) == mpo.MPO_ERR_INVALID_ARG
    p.destroy()
    p.destroy()   # idempotent
    # default: every layer in short chunks; 1: every layer in long ones
    for small, ce in ((None, 1024), (1, 4096)):
        q = mpo.Plan(ts, host_only=True, small_layer_params=small)
        assert q.num_chunks == sum((n + ce - 1) // ce for n in sizes)
        assert all(q.layer_info(l)["chunk_elems"] == ce for l in set(layers))
        q.destroy()


def test_step_calls_validate_before_touching_the_gpu():
    p = _host_plan([T(0)])
    # a host-only plan cannot be stepped
    assert _status(mpo.mpo_adam_step, p, mpo.AdamCfg(), 1) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_sgd_step, p, mpo.SgdCfg(), 1) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_step_layer, p, 0, mpo.AdamCfg(), 1) == mpo.MPO_ERR_INVALID_ARG
    # config errors are reported first
    assert _status(mpo.mpo_adam_step, p, mpo.AdamCfg(), 0) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_adam_step, p, mpo.AdamCfg(round=7), 1) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_adam_step, p, mpo.AdamCfg(weight_fmt=3), 1) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_adam_step, p, mpo.AdamCfg(beta1=1.0), 1) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_adam_step, p, mpo.AdamCfg(loss_scale=0.0), 1) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_adam_step, p, mpo.AdamCfg(lr=float("nan")), 1) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_adam_step, p, mpo.AdamCfg(grad_clip=-1.0), 1) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_sgd_step, p, mpo.SgdCfg(grad_clip=float("inf")), 1) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_sgd_step, p, mpo.SgdCfg(round=-3), 1) == mpo.MPO_ERR_INVALID_ARG
    assert _status(mpo.mpo_sgd_step, p, mpo.SgdCfg(loss_scale=float("inf")), 1) == mpo.MPO_ERR_INVALID_ARG
    # null plan / null cfg through the raw entry points
    cfg = mpo.AdamCfg().c()
    assert mpo.lib.mpo_adam_step(None, ctypes.byref(cfg), 1, None) == mpo.MPO_ERR_INVALID_ARG
    assert mpo.lib.mpo_adam_step(p._h, None, 1, None) == mpo.MPO_ERR_INVALID_ARG
    assert mpo.lib.mpo_step_layer(p._h, 0, None, 0, 9, ctypes.cast(ctypes.byref(cfg), ctypes.c_void_p), 1, None) \
        == mpo.MPO_ERR_INVALID_ARG
    assert mpo.lib.mpo_plan_destroy(None) == mpo.MPO_OK


def test_plan_create_without_a_gpu_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(mpo.MpoError) as e:
        mpo.Plan([T(0)])
    assert e.value.status == mpo.MPO_ERR_HIP and mpo.lib.mpo_last_hip_error() != 0


@pytest.mark.parametrize("order", ["package, torch", "torch, package", "probe, torch"])
def test_one_hip_runtime_whatever_the_import_order(order):
    """The library and PyTorch must share ONE copy of the HIP runtime: with two, the library's
    launches go to a runtime that knows nothing of torch's streams and allocations."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    first = {"package, torch": "import paper_2309_12381_amd, torch",
             "torch, package": "import torch, paper_2309_12381_amd",
             "probe, torch": "from paper_2309_12381_amd import probe; probe._load(); import torch, paper_2309_12381_amd"}[order]
    code = (first + "\n"
            "libs = sorted({l.split()[-1] for l in open('/proc/self/maps') if 'libamdhip64' in l})\n"
            "print('\\n'.join(libs))\n")
    out = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    libs = [l for l in out.stdout.split("\n") if l]
    assert len(libs) == 1, "more than one HIP runtime mapped: %s" % libs
