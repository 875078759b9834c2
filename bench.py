#!/usr/bin/env python3
"""Throughput of the split-precision Adam step on one MI355X.

A "step" is one optimizer step over the whole synthetic model: for the default
workload (c3, Llama-7B-shaped, 6.74 B parameters) that is one mpo_step_layer call
per layer, last layer first, every layer reading its gradient from the one reused
gradient buffer.  All state and the gradients are resident in HBM before the
timed region; the timed region contains nothing but the library's launches.

Prints ONE JSON line: parameters updated per second, with a `roofline` object
(algorithmic bytes = 26 B per parameter for Adam, against 8 TB/s) and a
`cpu_baseline` object (the CPU oracle timed on this host on a bounded sample).

Other legs, each printing one JSON line of its own: --fused-backward (the step inside a real PyTorch backward),
--probe-streams and --split-merge (what the memory system gives, by placement and launch shape), --measure-traffic
(HBM-side bytes per parameter from hardware counters), --compare-lib
(two builds of the library in one process), --c-caller (the same steps from a C program, no Python in its process).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0            # MI355X HBM3E, published peak
SGD_BYTES_PER_PARAM = 18          # read hi, res, grad, momentum buffer; write hi, res, buffer
ADAM_BYTES_PER_PARAM = 26         # read hi, res, grad (2 B each), m, v (4 B each); write hi, res, m, v
# HBM-side bytes per parameter of the Adam step kernel measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# each scaled by what the same counter reads for a plain kernel of known size (FETCH_SIZE x 2.000, WRITE_SIZE
# x 1.000 on this GPU): 14.12 read + 12.00 written.  Source: profiles/step_kernel_adam_bf16_c3_pmc_traffic.txt.
# Counters cannot be collected inside a timed run, so the figure is carried here from that file and the JSON
# line says so (roofline.traffic_source); `python bench.py --measure-traffic` takes the measurement again.
MEASURED_TRAFFIC_BYTES_PER_PARAM = {"c3": 26.12}
TRAFFIC_SOURCE = ("carried from profiles/step_kernel_adam_bf16_c3_pmc_traffic.txt (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE), not measured "
                  "in this run; python bench.py --measure-traffic measures it")


def host_threads():
    """Host threads the oracle's timing may use: what the machine grants this job (OMP_NUM_THREADS where the
    job's CPU share is announced that way, else the CPUs this process may run on)."""
    env = os.environ.get("OMP_NUM_THREADS", "")
    if env.isdigit() and int(env) > 0:
        return int(env), "OMP_NUM_THREADS"
    try:
        return len(os.sched_getaffinity(0)), "sched_getaffinity"
    except AttributeError:
        return os.cpu_count() or 1, "cpu_count"


def _oracle_rate(wl, n: int, steps: int, threads: int):
    """params/s of the oracle's Adam step on n parameters of this workload's value distributions, the
    array sliced over `threads` host threads (elementwise work: a slice per thread, each calling the C routine)."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import ref
    from paper_2309_12381_amd import synth
    rfmt = ref.BF16 if wl.fmt == "bf16" else ref.FP16
    w = synth.gen_weights(n, 99, "cpu", wl.weight_std).numpy()
    g = synth.bits16(synth.gen_grads(n, 98, "cpu", wl.grad_std, wl.fmt, wl.loss_scale))
    cfg = ref.AdamCfg(lr=1e-3, weight_decay=wl.weight_decay, decoupled_wd=(wl.optimizer == "adamw"),
                      loss_scale=wl.loss_scale, weight_fmt=rfmt, grad_fmt=rfmt)
    hi, res = ref.split(w, rfmt)
    del w
    m = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32)
    bounds = np.linspace(0, n, threads + 1).astype(np.int64)

    def run(i, t):
        lo, up = int(bounds[i]), int(bounds[i + 1])
        ref.adam_step(hi[lo:up], res[lo:up], g[lo:up], m[lo:up], v[lo:up], cfg, t)
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda i: run(i, 1), range(threads)))          # warm the pages
        t0 = time.perf_counter()
        for t in range(2, 2 + steps):
            list(ex.map(lambda i: run(i, t), range(threads)))
        dt = time.perf_counter() - t0
    return n * steps / dt


def cpu_baseline(wl, sample_params: int, steps: int, others: bool):
    """The oracle as it stands, on host cores, on a slice of the same workload (elementwise work, so a
    slice of one tensor is a fair sample), once on one thread and once on every thread the job is granted.
    `others`: also the small configurations c0, c1 and c2 in full (their whole parameter count, same value
    distributions), so that every configuration the oracle can hold has a CPU figure."""
    from paper_2309_12381_amd import synth
    cores, source = host_threads()
    one = _oracle_rate(wl, sample_params, steps, 1)
    many = _oracle_rate(wl, sample_params, steps, cores)
    out = {"value": many, "unit": "params/s", "cores": cores, "cores_from": source, "kind": "oracle",
           "value_1core": one, "host_GBps": many * ADAM_BYTES_PER_PARAM / 1e9,
           "sample": "%d params of the same value distributions, %d Adam steps, oracle/mpo_ref.c as built for "
                     "the tests, slice-parallel over %d host threads" % (sample_params, steps, cores)}
    if others:
        full = {}
        for key, k in (("c0", 10), ("c1", 5), ("c2", 2)):
            w2 = synth.workload(key)
            full[key] = {"params": w2.num_params, "steps": k,
                         "params_per_s_1core": _oracle_rate(w2, w2.num_params, k, 1),
                         "params_per_s_all_cores": _oracle_rate(w2, w2.num_params, k, cores)}
        out["full_configs"] = full
    return out


def layer_breakdown(st, cfg, stream, step_no, bpp):
    """One more step with an event around every mpo_step_layer call: GB/s of the big launches
    (transformer blocks, embedding, head) and the time of the small one (a norm vector)."""
    import torch
    from paper_2309_12381_amd import binding as mpo
    rows = []
    for layer in st.layers_backward:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        mpo.mpo_step_layer(st.plan, layer, cfg, step_no, stream=stream)
        e1.record(stream)
        rows.append((layer, sum(st.views[i].spec.n for i in st.by_layer[layer]), e0, e1))
    torch.cuda.synchronize()
    big, small = [], []
    for layer, n, e0, e1 in rows:
        ms = e0.elapsed_time(e1)
        (big if n >= (1 << 24) else small).append((bpp * n / ms / 1e6, ms, n, layer))
    big.sort()
    out = {"what": "one extra step, an event pair around every per-layer launch (includes the gaps between launches)",
           "big_launches": len(big), "big_GBps_min": big[0][0], "big_GBps_median": big[len(big) // 2][0],
           "big_GBps_max": big[-1][0], "big_params_each": sorted({b[2] for b in big})}
    if small:
        out["small_launches"] = [{"layer": s[3], "params": s[2], "us": s[1] * 1e3} for s in small]
    return out


def graph_run(st, cfg, stream, step_no, steps, P, bpp):
    """The same `steps` optimizer steps captured once in a HIP graph (each with its own step number) and
    replayed: what is left when the host's launch latency is taken out.  Small lists only."""
    import torch
    from paper_2309_12381_amd import binding as mpo
    side = torch.cuda.Stream()
    side.wait_stream(stream)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for k in range(steps):
            if isinstance(cfg, mpo.SgdCfg):
                mpo.mpo_sgd_step(st.plan, cfg, step_no + 1 + k, stream=torch.cuda.current_stream())
            else:
                mpo.mpo_adam_step(st.plan, cfg, step_no + 1 + k, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    reps = 20
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        graph.replay()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / (reps * steps)
    return {"ms_per_step": dt * 1e3, "params_per_s": P / dt, "GBps": bpp * P / dt / 1e9,
            "frac_of_peak": bpp * P / dt / 1e9 / PEAK_HBM_GBPS,
            "what": "%d steps captured in one HIP graph, %d replays (the step numbers are fixed in the graph: a "
                    "measurement of launch cost, not a way to train)" % (steps, reps)}


def traffic_probe(st, stream, with_v, bpp, steps):
    """The same bytes over the same arrays in the same per-layer launches with the arithmetic
    taken out (csrc/stream_probe.hip): what this access pattern reaches on this GPU.  Runs after
    the timed region; it overwrites the state."""
    import torch
    from paper_2309_12381_amd import probe
    if st.wl.per_layer:
        spans = []
        for layer in st.layers_backward:
            ids = st.by_layer[layer]
            assert ids == list(range(ids[0], ids[-1] + 1)), "a layer's tensors are adjacent in the flat arrays"
            lo = st.views[ids[0]].off
            up = st.views[ids[-1]].off + st.views[ids[-1]].spec.n
            spans.append((lo, up - lo))
    else:
        spans = [(0, st.total)]

    def once():
        moved = 0
        for lo, n in spans:
            probe.stream_probe(st.hi[lo:], st.res[lo:], st.grad, st.m[lo:], st.v[lo:] if with_v else None, n, stream)
            moved += n - n % 4096
        return moved
    once()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    moved = sum(once() for _ in range(steps))
    e1.record(stream)
    torch.cuda.synchronize()
    gbps = bpp * moved / e0.elapsed_time(e1) / 1e6
    return {"achieved": gbps, "unit": "GB/s", "frac_of_peak": gbps / PEAK_HBM_GBPS,
            "what": "stream_probe: same arrays, same launches per step (%d), same bytes per parameter, no arithmetic; "
                    "%d steps after the timed region" % (len(spans), steps)}


def fused_backward_run(a):
    """Section 3.2 on a real PyTorch backward: a stack of pre-norm transformer blocks (causal self-attention
    through torch's scaled_dot_product_attention, then a GELU MLP; bf16, synthetic data) trained with the
    split-precision Adam step, once with the step fused into backward (each parameter stepped in its
    post-accumulate-grad hook, gradient freed there), once more without the placement of the optimizer state,
    once with the hook's steps on a stream of their own, and once with the classical schedule (all gradients
    kept, stepped after backward).  Each variant runs in this one process, one after the other.  Prints one JSON
    line with the time per iteration, the peak device memory and the rate of the step launches on their own."""
    import torch
    import paper_2309_12381_amd as mpo
    from paper_2309_12381_amd.fused_backward import FusedBackwardOptimizer
    dev = "cuda:0"
    torch.cuda.set_device(0)
    d, depth, tokens, seq = a.width, a.depth, a.tokens, a.seq
    heads = max(1, d // 128)
    if tokens % seq:
        print("bench.py: --tokens must be a multiple of --seq", file=sys.stderr)
        sys.exit(2)

    class Block(torch.nn.Module):
        def __init__(self):
            super().__init__()
            self.norm1 = torch.nn.LayerNorm(d)
            self.qkv = torch.nn.Linear(d, 3 * d, bias=False)
            self.proj = torch.nn.Linear(d, d, bias=False)
            self.norm2 = torch.nn.LayerNorm(d)
            self.up = torch.nn.Linear(d, 4 * d, bias=False)
            self.down = torch.nn.Linear(4 * d, d, bias=False)

        def forward(self, x):                                   # x: (batch, seq, d)
            b, s_, _ = x.shape
            q, k, v = self.qkv(self.norm1(x)).view(b, s_, 3, heads, d // heads).permute(2, 0, 3, 1, 4)
            att = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
            x = x + self.proj(att.transpose(1, 2).reshape(b, s_, d))
            return x + self.down(torch.nn.functional.gelu(self.up(self.norm2(x))))

    def run(fused, overlap=False, place=True, bucket=None):
        torch.manual_seed(0)
        model = torch.nn.Sequential(*[Block() for _ in range(depth)]).to(dev).to(torch.bfloat16)
        params = sum(p.numel() for p in model.parameters())
        opt = FusedBackwardOptimizer(model.parameters(), mpo.AdamCfg(lr=1e-4, weight_decay=0.01), fused=fused,
                                     overlap=overlap, place=place, bucket_params=bucket)
        x = torch.randn(tokens // seq, seq, d, device=dev, dtype=torch.bfloat16)
        y = torch.randn(tokens // seq, seq, d, device=dev, dtype=torch.bfloat16)

        def iteration():
            opt.start_step()
            loss = torch.nn.functional.mse_loss(model(x).float(), y.float())
            loss.backward()
            if not fused:
                opt.step()
        for _ in range(a.warmup):
            iteration()
        torch.cuda.synchronize()
        resident = torch.cuda.memory_allocated()
        torch.cuda.reset_peak_memory_stats()
        steps = a.steps or 5
        t0 = time.perf_counter()
        for _ in range(steps):
            iteration()
        opt.synchronize()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        peak = torch.cuda.max_memory_allocated()
        out = {"ms_per_iteration": dt * 1e3, "peak_GB": peak / 1e9, "resident_GB": resident / 1e9,
               "peak_above_resident_GB": (peak - resident) / 1e9, "placement": opt.placement}
        # the step launches of one iteration on their own: every parameter stepped from one reused gradient buffer,
        # as the hooks do it (one mpo_step_layer with a per-call gradient pointer per parameter)
        big = max(p.numel() for p in opt.params)
        gbuf = torch.randn(big, device=dev, dtype=torch.bfloat16) * 1e-4
        stream = torch.cuda.current_stream()

        def all_steps(t):
            if opt.buckets is not None:                          # one launch per bucket, as the hooks issue them
                for b, members in enumerate(opt.buckets):
                    mpo.mpo_step_layer(opt.bucket_plan, b, opt.cfg, t, grads=[gbufs[k][:opt.params[i].numel()]
                                                                               for k, i in enumerate(members)], stream=stream)
                return
            for i, p in enumerate(opt.params):
                mpo.mpo_step_layer(opt.plan, i, opt.cfg, t, grads=[gbuf[:p.numel()]], stream=stream)
        if opt.buckets is not None:
            gbufs = [torch.randn(big, device=dev, dtype=torch.bfloat16) * 1e-4 for _ in range(max(len(b) for b in opt.buckets))]
        all_steps(opt.step_no + 1)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for k in range(3):
            all_steps(opt.step_no + 2 + k)
        e1.record(stream)
        e1.synchronize()
        ms = e0.elapsed_time(e1) / 3
        out["step_launches"] = {"ms": ms, "GBps": ADAM_BYTES_PER_PARAM * params / ms / 1e6,
                                "frac_of_peak": ADAM_BYTES_PER_PARAM * params / ms / 1e6 / PEAK_HBM_GBPS,
                                "launches": len(opt.buckets) if opt.buckets is not None else len(opt.params)}
        opt.close()
        del model, opt, x, y, gbuf
        gbufs = None
        torch.cuda.empty_cache()
        return out, params

    variants = {"fused": dict(fused=True), "fused_one_launch_per_parameter": dict(fused=True, bucket=0),
                "fused_one_launch_per_block": dict(fused=True, bucket=12 * d * d),
                "fused_without_placement": dict(fused=True, place=False), "fused_overlapped": dict(fused=True, overlap=True),
                "classical": dict(fused=False)}
    if a.fb_variant:
        out, params = run(**variants[a.fb_variant])
        out["params"] = params
        print(json.dumps(out), flush=True)
        return
    # every variant in a process of its own: where its arrays land depends on what the process allocated before
    import subprocess
    res = {}
    for name in variants:
        cmd = [sys.executable, os.path.abspath(__file__), "--fused-backward", "--fb-variant", name, "--width", str(d),
               "--depth", str(depth), "--tokens", str(tokens), "--seq", str(seq), "--warmup", str(a.warmup)]
        if a.steps:
            cmd += ["--steps", str(a.steps)]
        r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
        if r.returncode != 0:
            print("bench.py --fused-backward: variant %s failed:\n%s" % (name, r.stderr[-2000:]), file=sys.stderr)
            sys.exit(1)
        res[name] = json.loads([l for l in r.stdout.split("\n") if l.startswith("{")][-1])
    params = res["fused"]["params"]
    print(json.dumps({
        "metric": "training iteration with the split-precision Adam step fused into backward vs stepped after it",
        "n_gpus": 1, "data": "synthetic", "dtype": "bf16 forward/backward, f32 update",
        "config": {"workload": "%d transformer blocks of width %d, %d heads (%.2f B parameters), %d tokens per iteration in "
                               "sequences of %d; every variant in a process of its own" % (depth, d, heads, params / 1e9, tokens, seq),
                   "optimizer": "adamw"},
        **res,
        "gradient_bytes_GB": params * 2 / 1e9,
        "peak_saved_GB": res["classical"]["peak_GB"] - res["fused"]["peak_GB"],
    }), flush=True)


def probe_streams_run(a):
    """What the memory system gives the step's kind of traffic, and why the step kernel has the shape it
    has: plain read-only / write-only / in-place streams and the arithmetic-free copy of the Adam step's
    traffic (csrc/stream_probe.hip), with the arrays placed on purpose in one, two or three thirds of the
    device memory, then every variant of the launch shape on the two-thirds placement.  Must be the first
    thing a fresh process does on the GPU: ONE allocation of (almost) the whole memory is taken, which in
    a fresh process is laid out in order, and arrays are carved out of its thirds.  Prints one JSON line."""
    import torch
    from paper_2309_12381_amd import probe
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    GiB = 1 << 30
    props = torch.cuda.get_device_properties(0)
    free, total_mem = torch.cuda.mem_get_info()
    third = 96 * GiB
    whole = None
    for gib in (272, 200):
        if free > (gib + 4) * GiB:
            whole = torch.empty(gib * GiB, dtype=torch.uint8, device=dev)
            break
    if whole is None:
        print("bench.py --probe-streams: needs 204 GiB of free device memory in a fresh process", file=sys.stderr)
        sys.exit(1)
    thirds = whole.numel() // third + (1 if whole.numel() % third >= 24 * GiB else 0)
    SLOT = 10 * GiB

    def at(region, slot, nbytes):
        """nbytes at slot `slot` (10 GiB apart, from 4 GiB on) of third `region` of the allocation."""
        off = region * third + 4 * GiB + slot * SLOT
        assert nbytes <= SLOT and off + nbytes <= whole.numel()
        return whole[off:off + nbytes]

    stream = torch.cuda.current_stream()
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    for r in range(min(thirds, 3)):
        for sl in range(5 if r < 2 else 2):
            at(r, sl, 8 * GiB).fill_(0x11)
    torch.cuda.synchronize()

    default_reps = a.steps or 10

    def timed(fn, nbytes, reps=None):
        reps = reps or default_reps
        fn(); fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        e1.synchronize()
        return nbytes * reps / e0.elapsed_time(e1) / 1e6          # GB/s

    out = {"metric": "achieved HBM GB/s of plain streams and of the Adam step's traffic without arithmetic, by placement "
                     "and by launch shape", "unit": "GB/s", "n_gpus": 1, "data": "synthetic",
           "device": "%s (%d CUs)" % (props.name, props.multi_processor_count),
           "allocation_GiB": whole.numel() // GiB, "thirds_GiB": 96, "rows": []}

    def row(kind, what, gbps):
        out["rows"].append({"kind": kind, "what": what, "GBps": round(gbps, 1), "frac_of_8TBps": round(gbps / PEAK_HBM_GBPS, 4)})
        print("%-10s %-100s %8.1f GB/s" % (kind, what, gbps), file=sys.stderr, flush=True)

    # ---- plain streams: k arrays of 2 GiB in lock step -------------------------------------------------
    nb = 2 * GiB
    modes = (("read", probe.PLAIN_READ, 1), ("write", probe.PLAIN_WRITE, 1), ("in-place", probe.PLAIN_INPLACE, 2))
    layouts = [("1 array in one third", [(0, 0)]), ("2 arrays in one third", [(0, 0), (0, 1)]),
               ("4 arrays in one third", [(0, 0), (0, 1), (0, 2), (0, 3)]),
               ("2 arrays, one in each of two thirds", [(0, 0), (1, 0)]),
               ("4 arrays, two in each of two thirds", [(0, 0), (0, 1), (1, 0), (1, 1)])]
    if thirds >= 3:
        layouts.append(("3 arrays, one in each of three thirds", [(0, 0), (1, 0), (2, 0)]))
    # a nearly idle memory system for comparison (for counter runs: what one read costs without queueing)
    row("read", "light load: 64 workgroups, 1 MiB", timed(lambda: probe.plain_streams(probe.PLAIN_READ, [at(0, 0, nb)], 1 << 20, sink, stream), 1 << 20))
    for name, mode, passes in modes:
        for what, where in layouts:
            arrs = [at(r, sl, nb) for r, sl in where]
            row(name, what, timed(lambda: probe.plain_streams(mode, arrs, nb, sink, stream), passes * nb * len(arrs)))

    # ---- the Adam step's traffic (26 B per parameter, in place), by placement --------------------------
    n = 1 << 28
    placements = [("all five arrays in one third", dict(hi=0, res=0, grad=0, m=0, v=0)),
                  ("hi, m | res, v, grad", dict(hi=0, res=1, grad=1, m=0, v=1)),
                  ("hi, m, grad | res, v", dict(hi=0, res=1, grad=0, m=0, v=1)),
                  ("hi, res, grad | m, v", dict(hi=0, res=0, grad=0, m=1, v=1)),
                  ("hi, res, m | v, grad", dict(hi=0, res=0, grad=1, m=0, v=1))]
    if thirds >= 3:
        placements.append(("hi, m | res, v | grad", dict(hi=0, res=1, grad=2, m=0, v=1)))

    def arrays(pl):
        slot = dict(hi=0, res=1, grad=2, m=3, v=4)
        if pl["grad"] == 2:
            slot["grad"] = 0
        return [at(pl[k], slot[k], n * (2 if k in ("hi", "res", "grad") else 4)) for k in ("hi", "res", "grad", "m", "v")]
    for what, pl in placements:
        hi, res, grad, m, v = arrays(pl)
        row("adam-copy", what, timed(lambda: probe.stream_probe(hi, res, grad, m, v, n, stream), 26 * n))
    hi, res, grad, m, v = arrays(placements[1][1])
    n_long = 1 << 31
    hi_l, res_l, grad_l, m_l, v_l = [at(r, sl, n_long * w) for r, sl, w in ((0, 0, 2), (1, 1, 2), (1, 2, 2), (0, 3, 4), (1, 4, 4))]
    row("adam-copy", "hi, m | res, v, grad; one launch over 2^31 parameters (55.8 GB)",
        timed(lambda: probe.stream_probe(hi_l, res_l, grad_l, m_l, v_l, n_long, stream), 26 * n_long, reps=min(3, default_reps)))
    # ---- variants of the launch shape, on the two-thirds placement -------------------------------------
    cus = props.multi_processor_count
    for i, what in enumerate(probe.variants()):
        row("variant", what, timed(lambda: probe.stream_variant(i, hi, res, grad, m, v, n, cus, stream), 26 * n))
    print(json.dumps(out), flush=True)


def measure_traffic_run(a):
    """HBM-side bytes per parameter of the step kernel, measured: two child runs of this script (the workload of the
    command line, 2 steps, with --calibrate-copy) under `rocprofv3 --pmc`, one with FETCH_SIZE and one with
    WRITE_SIZE (KiB per dispatch), each reading scaled by what the same counter shows for a plain kernel that reads
    1 GiB and writes 1 GiB.  This process never touches the GPU.  Prints one JSON line."""
    import csv
    import glob
    import shutil
    import subprocess
    if shutil.which("rocprofv3") is None:
        print("bench.py --measure-traffic: rocprofv3 is not on PATH", file=sys.stderr)
        sys.exit(1)
    out_root = os.path.join(ROOT, "gpurun_out", "traffic")
    passthrough = ["--workload", a.workload, "--optimizer", a.optimizer, "--res-bits", str(a.res_bits), "--round", a.round,
                   "--chunk", a.chunk] + (["--res-packed"] if a.res_packed else []) + (["--no-place"] if a.no_place else [])
    env = dict(os.environ, TMPDIR="/tmp")
    got = {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        d = os.path.join(out_root, counter)
        shutil.rmtree(d, ignore_errors=True)
        os.makedirs(d)
        cmd = ["rocprofv3", "--pmc", counter, "-d", d, "-o", "t", "--output-format", "csv", "--", "python3",
               os.path.join(ROOT, "bench.py"), *passthrough, "--steps", "2", "--warmup", "1", "--no-cpu-baseline",
               "--no-end-to-end", "--no-breakdown", "--calibrate-copy"]
        r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
        files = glob.glob(os.path.join(d, "**", "t_counter_collection.csv"), recursive=True)
        if r.returncode != 0 or not files:
            print("bench.py --measure-traffic: the %s run failed:\n%s" % (counter, (r.stderr or r.stdout)[-2000:]), file=sys.stderr)
            sys.exit(1)
        step, copy = {}, []
        for row in csv.DictReader(open(files[0])):
            if row["Counter_Name"] != counter:
                continue
            name, grid, val = row["Kernel_Name"], int(row["Grid_Size"]), float(row["Counter_Value"])
            if "step_kernel" in name:
                step.setdefault(grid, []).append(val)
            elif "elementwise" in name and "add" in name.lower() and grid >= (1 << 26):
                copy.append(val)
        if not step or not copy:
            print("bench.py --measure-traffic: no step_kernel or calibration dispatches in %s" % files[0], file=sys.stderr)
            sys.exit(1)
        big = max(step)
        got[counter] = {"lanes": big, "dispatches": len(step[big]), "KiB_per_dispatch": sum(step[big]) / len(step[big]),
                        "calibration_KiB_per_GiB": sum(copy) / len(copy), "scale": 1048576.0 / (sum(copy) / len(copy))}
        line = [l for l in r.stdout.split("\n") if l.startswith("{")]
        if line:
            got["config"] = json.loads(line[-1])["config"]
    # parameters of the largest launch: one workgroup of 256 lanes per chunk; the chunk length from the plan's default
    lanes = got["FETCH_SIZE"]["lanes"]
    if got["WRITE_SIZE"]["lanes"] != lanes:
        print("bench.py --measure-traffic: the two runs saw different launches", file=sys.stderr)
        sys.exit(1)
    from paper_2309_12381_amd import synth
    wl = synth.workload(a.workload)
    by_layer = {}
    for t in wl.tensors:
        by_layer[t.layer] = by_layer.get(t.layer, 0) + t.n
    params = max(by_layer.values()) if wl.per_layer else wl.num_params
    rd = got["FETCH_SIZE"]["KiB_per_dispatch"] * 1024.0 * got["FETCH_SIZE"]["scale"]
    wr = got["WRITE_SIZE"]["KiB_per_dispatch"] * 1024.0 * got["WRITE_SIZE"]["scale"]
    print(json.dumps({"metric": "HBM-side traffic of the step kernel's largest launch (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE)",
                      "unit": "bytes per parameter", "n_gpus": 1, "data": "synthetic",
                      "config": got.get("config", {"workload": a.workload}), "params_per_launch": params,
                      "read_bytes_per_param": rd / params, "written_bytes_per_param": wr / params,
                      "value": (rd + wr) / params, "traffic_bytes_per_launch": rd + wr,
                      "counters": {k: got[k] for k in ("FETCH_SIZE", "WRITE_SIZE")}}))


def c_caller_run(a):
    """The stand-alone C program as a child process (this process never touches the GPU); its JSON line is passed on."""
    import subprocess
    from paper_2309_12381_amd import build
    exe = build.C_CALLER
    if not os.path.exists(exe):
        print("bench.py --c-caller: %s is not built (python -c 'import __graft_entry__ as g; g.build()')" % exe, file=sys.stderr)
        sys.exit(1)
    shape = a.shape or {"c3": (4096, 11008, 32, 32000), "c4": (5120, 13824, 40, 32000)}.get(a.workload)
    if shape is None:
        print("bench.py --c-caller: --workload c3 or c4, or --shape", file=sys.stderr)
        sys.exit(2)
    out = subprocess.run([exe, *[str(x) for x in shape], str(a.steps or 20), "0" if a.no_place else "1"], capture_output=True, text=True)
    sys.stderr.write(out.stderr)
    sys.stdout.write(out.stdout)
    sys.exit(out.returncode)


def compare_libs_run(a, st, cfg, stream):
    """Two builds of libmpo.so stepping the same state in turn (4 rounds of `--steps`, default 10, steps each
    after 2 untimed ones; HIP events).  Where the arrays lie is then the same for both, which it is not between
    two processes.  The plan made by the in-tree build is used by both: the other build must come from the
    same host sources.  Prints one JSON line."""
    import torch
    from paper_2309_12381_amd import binding as mpo
    builds = {"in_tree": mpo.lib, "other": mpo.load_library(a.compare_lib)}
    steps = a.steps or 10
    rows = {k: [] for k in builds}
    step_no = 0
    try:
        for _ in range(4):
            for name, lib in builds.items():
                mpo.lib = lib
                for _ in range(2):
                    step_no += 1
                    st.step(step_no, cfg, stream)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(steps):
                    step_no += 1
                    st.step(step_no, cfg, stream)
                e1.record(stream)
                e1.synchronize()
                rows[name].append(e0.elapsed_time(e1) / steps)
    finally:
        mpo.lib = builds["in_tree"]
    print(json.dumps({"metric": "ms per step of two builds of libmpo.so in one process, in turn", "unit": "ms", "n_gpus": 1,
                      "data": "synthetic", "steps_per_round": steps, "config": {"workload": st.wl.key, "other": a.compare_lib,
                                                                              "placement": st.placement},
                      "ms_per_step": rows,
                      "other_over_in_tree": sum(rows["other"]) / sum(rows["in_tree"])}))


def split_merge_run(a):
    """mpo_split and mpo_merge (Section 3.1, Table 1: used when a model is brought in or exported) on 2^30
    parameters, 8 bytes per parameter, with the three arrays placed on purpose in thirds of the device memory
    (one allocation first thing in a fresh process, as --probe-streams).  Prints one JSON line."""
    import torch
    from paper_2309_12381_amd import binding as mpo
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    GiB = 1 << 30
    free, _ = torch.cuda.mem_get_info()
    if free < 276 * GiB:
        print("bench.py --split-merge: needs 276 GiB of free device memory in a fresh process", file=sys.stderr)
        sys.exit(1)
    whole = torch.empty(272 * GiB, dtype=torch.uint8, device=dev)
    n = 1 << 30

    def at(region, slot, nbytes):
        off = region * 96 * GiB + 4 * GiB + slot * 10 * GiB
        return whole[off:off + nbytes]
    stream = torch.cuda.current_stream()
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    for r in range(3):
        at(r, 0, 4 * GiB).view(torch.float32).normal_(0.0, 0.02, generator=gen)
    reps = a.steps or 10
    rows = []
    out = {"metric": "achieved HBM GB/s of mpo_split / mpo_merge on 2^30 parameters by placement", "unit": "GB/s", "n_gpus": 1,
           "data": "synthetic", "rows": rows}

    def timed(fn):
        fn(); fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        e1.synchronize()
        return 8.0 * n * reps / e0.elapsed_time(e1) / 1e6

    placements = [("fp32, hi, res in one third", (0, 0, 0)), ("fp32, hi | res", (0, 0, 1)), ("fp32 | hi, res", (0, 1, 1)),
                  ("fp32 | hi | res", (0, 1, 2))]
    for fmt_name, fmt in (("bf16", mpo.MPO_BF16), ("fp16", mpo.MPO_FP16)):
        for rname, rnd in (("trunc", mpo.MPO_ROUND_TRUNC), ("stochastic", mpo.MPO_ROUND_STOCHASTIC)):
            if fmt_name == "fp16" and rname == "stochastic" and not a.all_variants:
                continue
            for what, (rw, rh, rr) in placements:
                w = at(rw, 0, 4 * n).view(torch.float32)
                hi = at(rh, 1, 2 * n).view(torch.int16)
                res = at(rr, 2, 2 * n).view(torch.int16)
                sp = timed(lambda: mpo.mpo_split(w, hi, res, n, fmt=fmt, round=rnd, seed=3, stream=stream))
                back = at(rw, 3, 4 * n).view(torch.float32)
                mg = timed(lambda: mpo.mpo_merge(hi, res, back, n, fmt=fmt, round=rnd, stream=stream))
                rows.append({"format": fmt_name, "round": rname, "placement": what, "split_GBps": round(sp, 1),
                             "merge_GBps": round(mg, 1)})
                print("%-5s %-10s %-28s split %7.1f GB/s   merge %7.1f GB/s" % (fmt_name, rname, what, sp, mg),
                      file=sys.stderr, flush=True)
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c3", choices=["c0", "c1", "c2", "c3", "c4"])
    ap.add_argument("--optimizer", default="adam", choices=["adam", "sgd"],
                    help="adam (the headline metric) or sgd with momentum 0.9 (18 B per parameter)")
    ap.add_argument("--res-bits", type=int, default=0,
                    help="extra bits kept per weight: 0 = all (the headline), 8 = the paper's bf16+8 / fp16+8 "
                         "(byte residual, 24 B per parameter for Adam)")
    ap.add_argument("--res-packed", action="store_true",
                    help="store the extra bits in packed planes (--res-bits = bits stored per weight, 1 to 15, e.g. 12: 1.5 B "
                         "per weight; with --round stochastic one of them is the flag)")
    ap.add_argument("--round", default="trunc", choices=["trunc", "nearest", "stochastic"],
                    help="rounding of the 16-bit value: trunc is the method's base mode and the headline")
    ap.add_argument("--fresh-grads", action="store_true",
                    help="regenerate each layer's gradients inside the loop (adds generator kernels to the timing)")
    ap.add_argument("--chunk", default="auto", choices=["auto", "short", "long"],
                    help="chunk length per workgroup: auto = the library's default (1024 parameters; with packed planes 4096 in "
                         "layers of 2^26 parameters or more); short / long = 1024 / 4096 everywhere")
    ap.add_argument("--streams", type=int, default=1,
                    help="per-layer workloads: also time the steps with the layers' launches going round this many streams")
    ap.add_argument("--no-place", action="store_true",
                    help="allocate the state arrays one after the other instead of dividing them between two "
                         "HBM regions (paper_2309_12381_amd/placement.py)")
    ap.add_argument("--fused-backward", action="store_true",
                    help="instead of the optimizer-only benchmark: a real PyTorch backward with the step fused into "
                         "it (Section 3.2) against the classical schedule; see --width, --depth, --tokens")
    ap.add_argument("--probe-streams", action="store_true",
                    help="instead of the benchmark: plain and step-shaped streams by placement in the device memory and by "
                         "launch shape (csrc/stream_probe.hip); takes (almost) all device memory, run it in a fresh process")
    ap.add_argument("--split-merge", action="store_true",
                    help="instead of the benchmark: mpo_split / mpo_merge on 2^30 parameters by placement (fresh process)")
    ap.add_argument("--all-variants", action="store_true", help="--split-merge: also fp16 with stochastic rounding")
    ap.add_argument("--fb-variant", default=None,
                    choices=["fused", "fused_one_launch_per_parameter", "fused_one_launch_per_block", "fused_without_placement",
                             "fused_overlapped", "classical"],
                    help="--fused-backward: this one variant only, in this process (what the full run starts six times; "
                         "also the form to run under a profiler, which must not see child processes)")
    ap.add_argument("--width", type=int, default=4096)
    ap.add_argument("--depth", type=int, default=12)
    ap.add_argument("--tokens", type=int, default=1024)
    ap.add_argument("--seq", type=int, default=1024, help="--fused-backward: sequence length (tokens / seq sequences per iteration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cpu-full-configs", action="store_true",
                    help="CPU baseline on the sample only, not on c0, c1 and c2 in full as well")
    ap.add_argument("--no-end-to-end", action="store_true",
                    help="skip the extra steps that regenerate every gradient inside the loop")
    ap.add_argument("--graph", action="store_true",
                    help="single-launch workloads (c0, c1, c2): also capture the timed steps in ONE HIP graph and time "
                         "its replays (launch latency taken out)")
    ap.add_argument("--no-breakdown", action="store_true", help="skip the per-layer breakdown step")
    ap.add_argument("--no-probe", action="store_true", help="skip the arithmetic-free traffic probe")
    ap.add_argument("--cpu-sample", type=int, default=202_383_360,
                    help="parameters of the CPU baseline's sample (default: one transformer layer of the 7B-shaped set)")
    ap.add_argument("--compare-lib", default=None, metavar="PATH",
                    help="time the workload with the in-tree libmpo.so and with another build of it (same host sources, "
                         "e.g. paper_2309_12381_amd.build.build(force=True, out=PATH, csrc=<a modified copy of csrc/>)) in "
                         "turn, in this process and on the same arrays: differences between processes (1-2 %%) are "
                         "larger than those between builds of the kernel")
    ap.add_argument("--measure-traffic", action="store_true",
                    help="measure the HBM-side bytes per parameter of the step kernel: runs this script twice as a child "
                         "under rocprofv3 --pmc (FETCH_SIZE, then WRITE_SIZE; 2 steps with --calibrate-copy) and scales "
                         "the readings by those of a plain kernel of known size; the figure the default run carries "
                         "as roofline.traffic comes from this")
    ap.add_argument("--c-caller", action="store_true",
                    help="run paper_2309_12381_amd/mpo_c_caller (csrc/c_caller.cpp): the per-layer Adam steps of a "
                         "Llama-shaped list driven through the C interface alone (hipMalloc, mpo_place_second, "
                         "mpo_plan_create, mpo_step_layer), in a process of its own without Python or PyTorch; "
                         "--workload c3 (default) or c4 gives the shape (bf16 either way), --no-place skips the search")
    ap.add_argument("--shape", type=int, nargs=4, default=None, metavar=("HIDDEN", "INTER", "LAYERS", "VOCAB"),
                    help="--c-caller: another Llama shape")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain elementwise kernel that reads 1 GiB and writes 1 GiB (known traffic, "
                         "for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus %d is not supported"
              % a.gpus, file=sys.stderr)
        sys.exit(2)

    if a.c_caller:
        c_caller_run(a)
        return
    if a.measure_traffic:
        measure_traffic_run(a)
        return
    import torch
    from paper_2309_12381_amd import harness, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if a.probe_streams:
        probe_streams_run(a)
        return
    if a.split_merge:
        split_merge_run(a)
        return
    if a.fused_backward:
        fused_backward_run(a)
        return
    dev = "cuda:0"
    torch.cuda.set_device(0)
    wl = synth.workload(a.workload)
    # default: 100 steps for the per-layer sets (the configurations ask for 3-5; more steps only average the
    # same step, and a few seconds of sustained work read 0.5 % higher than half a second)
    steps = a.steps if a.steps is not None else max(wl.steps, 100 if wl.per_layer else wl.steps)
    props = torch.cuda.get_device_properties(0)
    t_setup = time.perf_counter()
    st = harness.ModelState(wl, dev, res_bits=a.res_bits, res_packed=a.res_packed,
                            round={"trunc": 0, "nearest": 1, "stochastic": 2}[a.round], place=not a.no_place,
                            small_layer_params={"auto": 0, "short": (1 << 64) - 1, "long": 1}[a.chunk])
    if wl.per_layer:
        # the reused buffer holds one (largest) layer's worth of gradient values, read by every layer
        st.grad.normal_(0.0, wl.grad_std * wl.loss_scale, generator=synth.generator(7, dev))
    else:
        st.fill_grads(range(len(st.views)), 0)
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup

    stream = torch.cuda.current_stream()
    cfg = st.adam_cfg() if a.optimizer == "adam" else st.sgd_cfg()
    if a.compare_lib:
        compare_libs_run(a, st, cfg, stream)
        return
    bpp = ADAM_BYTES_PER_PARAM if a.optimizer == "adam" else SGD_BYTES_PER_PARAM
    if a.res_packed:
        bpp += 2 * (a.res_bits / 8.0 - 2.0)  # packed planes: res_bits/8 bytes read and written instead of 2
    else:
        bpp -= 2 * (2 - st.res_bytes)        # a byte residual is read and written as 1 B instead of 2
    step_no = 0
    for _ in range(a.warmup):
        step_no += 1
        st.step(step_no, cfg, stream, fresh_grads=a.fresh_grads)
    torch.cuda.synchronize()
    # one event after every step, on the stream the kernels are launched on
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    launches = 0
    t0 = time.perf_counter()
    evs[0].record(stream)
    for k in range(steps):
        step_no += 1
        launches += st.step(step_no, cfg, stream, fresh_grads=a.fresh_grads)
        evs[k + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = evs[0].elapsed_time(evs[-1])
    step_ms = sorted(evs[k].elapsed_time(evs[k + 1]) for k in range(steps))

    P = wl.num_params
    value = P * steps / wall
    bytes_per_launch = bpp * P * steps / launches
    achieved = bpp * P * steps / (ev_ms * 1e-3) / 1e9
    res = {
        "metric": "params updated/sec, split-precision %s (achieved HBM GB/s and %% of peak in roofline)"
                  % ("Adam" if a.optimizer == "adam" else "SGD-momentum"),
        "value": value, "unit": "params/s", "n_gpus": 1, "steps": steps, "warmup": a.warmup,
        "ms_per_step": wall * 1e3 / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %s" % (wl.key, wl.description), "params": P, "tensors": len(wl.tensors),
                   "format": ("%s, %d bits stored per weight in packed planes%s"
                              % (wl.fmt, a.res_bits, " (the leading one is the rounding flag)" if a.round == "stochastic" else "")
                              if a.res_packed else
                              "%s+%d extra bits (%d-bit residual)"
                              % (wl.fmt, a.res_bits or (13 if wl.fmt == "fp16" else 15 if a.round == "stochastic" else 16),
                                 8 * st.res_bytes)),
                   "optimizer": wl.optimizer if a.optimizer == "adam" else "sgd-momentum", "round": a.round, "loss_scale": wl.loss_scale,
                   "launches_per_step": launches // steps, "per_layer": wl.per_layer, "chunk": a.chunk,
                   "fresh_grads_in_loop": bool(a.fresh_grads), "resident_GB": st.resident_bytes / 1e9,
                   "placement": st.placement,
                   "device": "%s (%d CUs) %s" % (props.name, props.multi_processor_count,
                                                 getattr(props, "uuid", ""))},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBPS,
                     "traffic": (MEASURED_TRAFFIC_BYTES_PER_PARAM[wl.key] * P * steps / launches
                                 if wl.key in MEASURED_TRAFFIC_BYTES_PER_PARAM and a.optimizer == "adam" and st.res_bytes == 2
                                 and not a.res_packed and a.chunk == "auto" else None),
                     "traffic_source": TRAFFIC_SOURCE,
                     "kernel": "step_kernel<%s,%s>" % (a.optimizer, wl.fmt), "bytes_per_param": bpp,
                     "bytes_per_launch": bytes_per_launch, "avg_launch_ms": ev_ms / launches,
                     "event_ms": ev_ms, "launches": launches,
                     "step_ms_median": step_ms[len(step_ms) // 2], "step_ms_min": step_ms[0]},
        "setup_s": setup_s,
    }
    if res["roofline"]["traffic"] is None:
        res["roofline"]["traffic_source"] = None
    if not a.fresh_grads and not a.no_end_to_end:
        # the same steps with backward's stand-in inside the loop: every layer's gradient is regenerated (seeded
        # normal draws cast to the gradient format, torch kernels) just before that layer's step
        k = 3 if wl.per_layer else min(steps, 10)
        step_no += 1
        st.step(step_no, cfg, stream, fresh_grads=True)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(k):
            step_no += 1
            st.step(step_no, cfg, stream, fresh_grads=True)
        torch.cuda.synchronize()
        e2e = (time.perf_counter() - t1) / k
        res["end_to_end_with_gradient_generation"] = {
            "ms_per_step": e2e * 1e3, "params_per_s": P / e2e, "steps": k,
            "what": "optimizer steps with each layer's gradient regenerated inside the loop by torch's generator and "
                    "cast kernels (the stand-in for backward); the headline times the library's launches alone"}
    if a.streams > 1 and wl.per_layer:
        # the same steps with the per-layer launches going round several streams: consecutive launches overlap where
        # one drains and the next fills the GPU
        side = [torch.cuda.Stream() for _ in range(a.streams)]
        for sd in side:
            sd.wait_stream(stream)
        for _ in range(2):
            step_no += 1
            st.step(step_no, cfg, streams=side)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(steps):
            step_no += 1
            st.step(step_no, cfg, streams=side)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t1) / steps
        for sd in side:
            stream.wait_stream(sd)
        res["launches_over_several_streams"] = {
            "streams": a.streams, "ms_per_step": dt * 1e3, "params_per_s": P / dt, "GBps": bpp * P / dt / 1e9,
            "frac_of_peak": bpp * P / dt / 1e9 / PEAK_HBM_GBPS,
            "what": "the timed steps again with the per-layer launches going round %d streams (wall clock); the headline "
                    "uses one stream" % a.streams}
    if a.graph and not wl.per_layer:
        res["hip_graph"] = graph_run(st, cfg, stream, step_no, steps, P, bpp)
        step_no += steps
    if wl.per_layer and not a.no_breakdown:
        res["breakdown"] = layer_breakdown(st, cfg, stream, step_no + 1, bpp)
    if st.res_bytes == 2 and not a.res_packed and not a.no_probe:
        pr = traffic_probe(st, stream, a.optimizer == "adam", bpp, min(steps, 5))
        pr["step_kernel_frac_of_this"] = achieved / pr["achieved"]
        res["roofline"]["probe"] = pr
    st.close()
    if a.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)       # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)                                   # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        res["calibration"] = "3 x torch.add(src, 1.0, out=dst) on 2^28 fp32: 1 GiB read + 1 GiB written each"
    if not a.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl, a.cpu_sample, 5, others=not a.no_cpu_full_configs)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
