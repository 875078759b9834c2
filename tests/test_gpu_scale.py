"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (harness.ModelState: flat state arrays, one reused gradient buffer, one
mpo_step_layer per layer in backward order for the Llama-shaped sets).

c1 and c2 are compared in full.  c3 (6.7 B parameters) and c4 (13 B, fp16) do not fit in host
memory: whole tensors are compared for a few tensors and 4096-element blocks (first, last and
random ones) for every tensor.  The oracle starts from the fp32 weights and the gradient bytes
the generators produced, never from anything the library computed.
"""
import numpy as np
import pytest
import torch

import paper_2309_12381_amd as mpo
from paper_2309_12381_amd import harness, synth
from oracle import ref

from gpu_util import DEV, ref_adam, ref_split, say

pytestmark = pytest.mark.gpu

BLOCK = 4096


def _ref_cfg(st):
    c = st.adam_cfg()
    rf = ref.BF16 if st.wl.fmt == "bf16" else ref.FP16
    return ref.AdamCfg(lr=c.lr, beta1=c.beta1, beta2=c.beta2, eps=c.eps, weight_decay=c.weight_decay,
                       decoupled_wd=c.decoupled_wd, loss_scale=c.loss_scale, weight_fmt=rf, grad_fmt=rf,
                       res_bits=st.res_bits, round=st.round, seed=st.rng_seed, res_packed=st.res_packed), rf


def _run_and_compare(key, steps, sampler, res_bits=0, round=0, packed=False):
    """round: 0 truncation, 1 nearest, 2 stochastic.  With stochastic rounding the sampler must
    pick whole tensors only: the oracle numbers the elements of the array it is given, and the
    random stream is indexed by the element's position in its tensor."""
    wl = synth.workload(key)
    say("full-size %s: %d params, %d steps, res_bits %d, round %d" % (key, wl.num_params, steps, res_bits, round))
    st = harness.ModelState(wl, DEV, seed=2309, keep_w32_samples=sampler, res_bits=res_bits, round=round,
                            res_packed=packed)
    if packed:
        assert all(isinstance(st.w32_samples[i][0], slice) for i in st.w32_samples), "packed: whole tensors only"
    rcfg, rf = _ref_cfg(st)
    host = {}
    for i, (idx, w) in st.w32_samples.items():
        if packed:
            hi, res = ref.split(np.ascontiguousarray(w.numpy()), rf, res_bits, round, st.rng_seed, i, packed=True)
        elif round == 2:
            assert isinstance(idx, slice)
            hi, res = ref.split(np.ascontiguousarray(w.numpy()), rf, res_bits, round, st.rng_seed, i)
        else:
            hi, res = ref.split(np.ascontiguousarray(w.numpy()), rf, res_bits, round) if round else \
                ref_split(np.ascontiguousarray(w.numpy()), rf, res_bits)
        host[i] = [hi, res, np.zeros(hi.size, np.float32), np.zeros(hi.size, np.float32)]

    for t in range(1, steps + 1):
        def grab(layer, ids, t=t):
            # this layer's gradients are in the buffer now: take the sampled bytes for the oracle
            for i in ids:
                if i not in host:
                    continue
                tv = st.views[i]
                idx = st.w32_samples[i][0]
                g = st.grad[tv.goff:tv.goff + tv.spec.n][idx]
                gb = synth.bits16(g)
                h = host[i]
                if round == 2 or packed:
                    ref.adam_step(h[0], h[1], gb, h[2], h[3], rcfg, t, tensor_id=i)     # whole tensor, in order
                else:
                    ref_adam(h[0], h[1], gb, h[2], h[3], rcfg, t)
        st.step(t, fresh_grads=True, before_layer=grab)
    torch.cuda.synchronize()

    checked = 0
    for i, h in host.items():
        tv = st.views[i]
        idx = st.w32_samples[i][0]
        n = tv.spec.n
        got_hi = synth.bits16(st.hi[tv.off:tv.off + n][idx])
        if packed:
            got_res = st.res[st.res_off[i]:st.res_off[i] + mpo.mpo_res_bytes(n, res_bits, True)].cpu().numpy().copy()
        else:
            got_res = st.res[tv.off:tv.off + n][idx]
            got_res = got_res.cpu().numpy().copy() if got_res.dtype == torch.uint8 else synth.bits16(got_res)
        got_m = st.m[tv.off:tv.off + n][idx].cpu().numpy()
        got_v = st.v[tv.off:tv.off + n][idx].cpu().numpy()
        name = "%s tensor %d (%s)" % (key, i, tv.spec.name)
        assert np.array_equal(got_hi, h[0]) and np.array_equal(got_res, h[1]), name + ": stored weights differ"
        assert np.array_equal(got_m.view(np.uint32), h[2].view(np.uint32)), name + ": m differs"
        assert np.array_equal(got_v.view(np.uint32), h[3].view(np.uint32)), name + ": v differs"
        checked += h[0].size
    st.close()
    return checked, wl


def _everything(i, n):
    return slice(None)


def _blocks_sampler(whole_every=97, nblocks=6, seed=5):
    rng = np.random.default_rng(seed)

    def sampler(i, n):
        if n <= 4 * BLOCK or i % whole_every == 3:
            return slice(None)                                   # norm vectors, and a few whole matrices
        nb = (n + BLOCK - 1) // BLOCK
        pick = {0, nb - 1, nb // 2} | {int(b) for b in rng.integers(0, nb, size=nblocks)}
        idx = np.concatenate([np.arange(b * BLOCK, min(n, (b + 1) * BLOCK)) for b in sorted(pick)])
        return torch.from_numpy(idx).to(DEV)
    return sampler


def test_c1_resnet50_like_full():
    checked, wl = _run_and_compare("c1", 5, _everything)
    assert checked == wl.num_params == 25_600_000


def test_c2_gpt2_medium_full():
    checked, wl = _run_and_compare("c2", 2, _everything)
    assert checked == wl.num_params == 354_823_168


def test_c3_llama7b_per_layer_sampled():
    checked, wl = _run_and_compare("c3", 2, _blocks_sampler())
    assert wl.num_params == 6_738_415_616 and checked > 40_000_000


def test_c3_llama7b_bf16_plus_8_per_layer_sampled():
    """The paper's bf16+8: byte residuals, 11 B resident and 24 B moved per parameter."""
    checked, wl = _run_and_compare("c3", 2, _blocks_sampler(seed=6), res_bits=8)
    assert checked > 40_000_000


def test_c1_bf16_plus_8_full():
    checked, wl = _run_and_compare("c1", 3, _everything, res_bits=8)
    assert checked == wl.num_params


def _whole_tensors(i, n):
    return slice(None) if (n <= 4 * BLOCK or i % 89 == 2 or i == 0) else None


def test_c3_llama7b_nearest_per_layer_sampled():
    checked, wl = _run_and_compare("c3", 2, _blocks_sampler(seed=7), round=1)
    assert checked > 40_000_000


def test_c3_llama7b_packed_12_bits_whole_tensors():
    """The paper's Figure 1 example, 12 extra bits without padding: 3.5 B per weight, 25 B moved per Adam step."""
    checked, wl = _run_and_compare("c3", 2, _whole_tensors, res_bits=12, packed=True)
    assert checked > 100_000_000


def test_c3_llama7b_packed_13_bits_whole_tensors():
    """An odd width: 13 = 8 + 4 + 1 stored bits, so the 1-bit plane (two lanes per byte) is in play."""
    checked, wl = _run_and_compare("c3", 2, _whole_tensors, res_bits=13, packed=True)
    assert checked > 100_000_000


def test_c4_llama13b_fp16_packed_14_bits_stochastic_whole_tensors():
    """The paper's "fp16+13 rstoc" without padding: 13 extra bits and the un-round flag in 14 stored bits."""
    free, total = torch.cuda.mem_get_info()
    if total < 200e9:
        pytest.skip("needs about 160 GB of device memory")
    checked, wl = _run_and_compare("c4", 2, _whole_tensors, res_bits=14, round=2, packed=True)
    assert checked > 200_000_000


def test_c4_llama13b_fp16_stochastic_whole_tensors():
    """The paper's "fp16+13 rstoc": stochastic rounding with the un-round flag in bit 13."""
    free, total = torch.cuda.mem_get_info()
    if total < 200e9:
        pytest.skip("needs about 160 GB of device memory")
    checked, wl = _run_and_compare("c4", 2, _whole_tensors, round=2)
    assert checked > 200_000_000


def test_c4_llama13b_fp16_per_layer_sampled():
    free, total = torch.cuda.mem_get_info()
    if total < 200e9:
        pytest.skip("needs about 160 GB of device memory")
    checked, wl = _run_and_compare("c4", 1, _blocks_sampler(whole_every=131))
    assert wl.num_params == 13_015_864_320 and checked > 40_000_000


def test_one_tensor_longer_than_2_to_32():
    """Element offsets beyond 32 bits: one tensor of 2^32 + 3 chunks + 5 parameters (60 GB of state)
    through split, two Adam steps and merge; blocks at the start, across the 2^32 boundary, at the
    ragged end and at random places are replayed by the oracle."""
    torch.cuda.empty_cache()
    free, total = torch.cuda.mem_get_info()
    if free < 100e9:
        pytest.skip("needs about 80 GB of device memory")
    n = (1 << 32) + 3 * BLOCK + 5
    say("one tensor of %d parameters" % n)
    g = torch.Generator(device=DEV)
    g.manual_seed(11)
    w = torch.empty(n, dtype=torch.float32, device=DEV)
    w.normal_(0.0, 0.02, generator=g)
    hi = torch.empty(n, dtype=torch.int16, device=DEV)
    res = torch.empty(n, dtype=torch.int16, device=DEV)
    m = torch.zeros(n, dtype=torch.float32, device=DEV)
    v = torch.zeros(n, dtype=torch.float32, device=DEV)
    grad = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    rng = np.random.default_rng(12)
    spans = [(0, 2 * BLOCK), ((1 << 32) - 2 * BLOCK, (1 << 32) + 2 * BLOCK), (n - BLOCK - 9, n)]
    spans += [(int(b) * BLOCK, int(b) * BLOCK + BLOCK) for b in rng.integers(0, n // BLOCK, size=12)]
    host = []
    for lo, up in spans:
        h, r = ref.split(np.ascontiguousarray(w[lo:up].cpu().numpy()), ref.BF16)
        host.append([h, r, np.zeros(up - lo, np.float32), np.zeros(up - lo, np.float32)])
    mpo.mpo_split(w, hi, res, n, fmt=mpo.MPO_BF16)
    del w
    plan = mpo.Plan([mpo.Tensor(hi, res, grad, m, v, n, 0)])
    assert plan.num_params == n and plan.num_chunks == (n + 1023) // 1024           # the default cut: 1024 per workgroup
    cfg = mpo.AdamCfg(lr=1e-3, weight_decay=0.01)
    rcfg = ref.AdamCfg(lr=1e-3, weight_decay=0.01)
    for t in (1, 2):
        grad.normal_(0.0, 1e-3, generator=g)
        for (lo, up), h in zip(spans, host):
            ref.adam_step(h[0], h[1], synth.bits16(grad[lo:up]), h[2], h[3], rcfg, t)
        if t == 1:
            mpo.mpo_adam_step(plan, cfg, t)
        else:
            mpo.mpo_step_layer(plan, 0, cfg, t)
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    mpo.mpo_merge(hi, res, out, n, fmt=mpo.MPO_BF16)
    torch.cuda.synchronize()
    for (lo, up), h in zip(spans, host):
        what = "parameters [%d, %d)" % (lo, up)
        assert np.array_equal(synth.bits16(hi[lo:up]), h[0]) and np.array_equal(synth.bits16(res[lo:up]), h[1]), what
        assert np.array_equal(m[lo:up].cpu().numpy().view(np.uint32), h[2].view(np.uint32)), what + ": m"
        assert np.array_equal(v[lo:up].cpu().numpy().view(np.uint32), h[3].view(np.uint32)), what + ": v"
        assert np.array_equal(out[lo:up].cpu().numpy().view(np.uint32), ref.merge(h[0], h[1], ref.BF16).view(np.uint32)), what
    plan.destroy()


def test_stochastic_split_beyond_2_to_34_elements():
    """The random stream is indexed by (element / 4) as a 64-bit counter: with more than 2^34 elements
    its high word is in use.  Sampled runs of elements are split by the oracle itself, told where in
    the tensor each run starts."""
    torch.cuda.empty_cache()
    free, total = torch.cuda.mem_get_info()
    if free < 230e9:
        pytest.skip("needs about 210 GB of device memory")
    n = (1 << 34) + BLOCK + 3
    seed, tid = 0x1234_5678_9ABC, 5
    say("stochastic split of %d parameters" % n)
    g = torch.Generator(device=DEV)
    g.manual_seed(13)
    w = torch.empty(n, dtype=torch.float32, device=DEV)
    w.normal_(0.0, 0.02, generator=g)
    hi = torch.empty(n, dtype=torch.int16, device=DEV)
    res = torch.empty(n, dtype=torch.int16, device=DEV)
    mpo.mpo_split(w, hi, res, n, fmt=mpo.MPO_BF16, round=mpo.MPO_ROUND_STOCHASTIC, seed=seed, tensor_id=tid)
    torch.cuda.synchronize()
    rng = np.random.default_rng(14)
    # runs of 1 to 37 elements at the start, around 2^34 (where the counter's high word changes), at the
    # end, and at random places on both sides of 2^34; starts of every residue modulo 4
    starts = [0, 1, 2, 3, (1 << 34) - 19, (1 << 34) - 2, 1 << 34, (1 << 34) + 1, n - 37, n - 3, n - 1]
    starts += [int(x) for x in rng.integers(1 << 34, n - 40, size=60)] + [int(x) for x in rng.integers(0, n - 40, size=60)]
    ups = total_checked = 0
    for k, lo in enumerate(starts):
        cnt = min(n - lo, 1 + (k * 7) % 37)
        x = np.ascontiguousarray(w[lo:lo + cnt].cpu().numpy())
        want_hi, want_res = ref.split(x, ref.BF16, 0, ref.STOCHASTIC, seed, tid, first_index=lo)
        assert np.array_equal(synth.bits16(hi[lo:lo + cnt]), want_hi), "hi of elements [%d, %d)" % (lo, lo + cnt)
        assert np.array_equal(synth.bits16(res[lo:lo + cnt]), want_res), "15 kept bits and the flag of [%d, %d)" % (lo, lo + cnt)
        ups += int((want_res >> 15).sum())
        total_checked += cnt
    assert 0.3 * total_checked < ups < 0.7 * total_checked                  # about half of them round up
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    mpo.mpo_merge(hi, res, out, n, fmt=mpo.MPO_BF16, round=mpo.MPO_ROUND_STOCHASTIC)
    # merge undoes the rounding: the value cut to 16 + 15 bits
    w.view(torch.int32).bitwise_and_(-2)                                   # in place: no third 69 GB array
    assert torch.equal(out.view(torch.int32), w.view(torch.int32))
