#!/usr/bin/env python3
"""Benchmark of the gradient bucket hot path on one MI355X.

One step = one pass of the whole path over one synthetic gradient set:
  kt_bucket_pack         local gradients -> peer slot 0 of every bucket
  kt_weighted_reduce     K peer copies of every bucket -> reduced bucket
  kt_bucket_unpack_scale reduced buckets -> parameter gradients
each as one batched launch over all buckets, on torch's current stream, with
all inputs resident in HBM (peer slots 1..K-1 are filled before timing).

Prints ONE JSON line: whole-step throughput in GB/s of algorithmic bytes
((K + 5) * element size per element), the roofline figures of the dominant
kernel (the reduce: (K + 1) * element size per element) measured with
events around its launches inside the timed steps, and the CPU checker timed
on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the reduce kernel from the FETCH_SIZE / WRITE_SIZE counter runs
# summarised under profiles/ (reads scaled by the factor the 1 GiB calibration copy gives).
# They describe the kernel sources with the digest below; after any change to those
# sources the figure is reported as null until the counters are taken again.
KERNEL_SOURCES = ("kt_internal.h", "kt_device.h", "kt_sgd_device.h", "kt_pack_unpack.hip", "kt_reduce.hip", "kt_fused.hip",
                  "kt_sgd.hip", "kt_fused_sgd.hip")
TRAFFIC_SOURCES_SHA = "380d6c1e6ad918bb"
TRAFFIC_BYTES = {"decoder_1p3b": 23705640787, "vit_b16": 3119150390}


def measured_traffic(workload):
    import hashlib
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2505_10183_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    if h.hexdigest()[:16] != TRAFFIC_SOURCES_SHA:
        return None
    return TRAFFIC_BYTES.get(workload)


ALIGN_BYTES = 16      # --align: start of every tensor inside its bucket


def setup(name, dev, in_place=True, misalign=False):
    import torch
    import paper_2505_10183_amd as kt
    from paper_2505_10183_amd import workloads as wl

    w = wl.get(name)
    K = w.K
    plan = kt.Plan(w.numels, w.dtype, w.bucket_cap_bytes, ALIGN_BYTES)
    shares, weights = kt.kt_plan_shares(w.throughputs, w.global_batch)
    td = wl.torch_dtype(w.dtype)
    nb = plan.num_buckets
    elems = plan.bucket_elems()
    # peer slot 0 receives the packed local gradients; slots 1..K-1 stand for the buckets
    # that arrive from the other devices: seeded Gaussians written straight into the buffers
    sh = 1 if misalign else 0        # element offset of every bucket buffer inside its allocation
    peers = [[torch.empty(n + sh, dtype=td, device=dev)[sh:] for n in elems]]
    for k in range(1, K):
        peers.append([wl.flat_normal(n + sh, w.dtype, w.sigma, w.seed * 1000 + 100 * k + b, dev)[sh:]
                      for b, n in enumerate(elems)])
    local = wl.gradient_set(w, 0, dev)
    # like an AllReduce, the reduce writes its result over peer slot 0 (the C ABI allows the
    # output to be one of the inputs); --out-of-place gives it buffers of its own
    outs = peers[0] if in_place else [torch.empty(n + sh, dtype=td, device=dev)[sh:] for n in elems]
    result = [torch.empty_like(t) for t in local]
    st = {
        "w": w, "plan": plan, "K": K, "weights": weights, "shares": shares, "nb": nb,
        "local": local, "peers": peers, "outs": outs, "result": result,
        # pointer arrays marshalled once: the step itself only launches
        "a_local": plan.marshal(local), "a_slot0": plan.marshal(peers[0]),
        "a_peers": plan.marshal([peers[k][b] for b in range(nb) for k in range(K)]),
        "a_outs": plan.marshal(outs), "a_result": plan.marshal(result),
        "a_others": plan.marshal([peers[k][b] for b in range(nb) for k in range(1, K)]),
    }
    import ctypes
    st["a_w"] = (ctypes.c_float * K)(*weights)
    return st


def step(st, scale=1.0, ev=None):
    """One pass of the path.  `ev`: four events recorded on the stream the kernels are
    launched on (torch's current stream): step start, after pack, after reduce, step end."""
    p = st["plan"]
    if ev is not None:
        ev[0].record()
    p.kt_bucket_pack(-1, st["a_local"], st["a_slot0"])
    if ev is not None:
        ev[1].record()
    p.kt_weighted_reduce(-1, st["a_peers"], st["K"], st["a_w"], st["a_outs"])
    if ev is not None:
        ev[2].record()
    p.kt_bucket_unpack_scale(-1, st["a_outs"], scale, st["a_result"])
    if ev is not None:
        ev[3].record()


def time_workload(name, steps, warmup, dev, in_place=True, misalign=False, events_in_timed_loop=True):
    """Times `steps` chained steps (wall clock, synchronised on both sides) and, with events
    on the launch stream, the reduce inside the step and every step on its own.  The events
    are recorded inside the timed loop for the headline workload (`events_in_timed_loop`);
    for the small launch-bound sets, where four event records per step would themselves
    cost a third of the step, the wall-clock loop runs without them and a second loop
    carries the events."""
    import torch
    st = setup(name, dev, in_place, misalign)
    w = st["w"]
    for _ in range(warmup):
        step(st)
    torch.cuda.synchronize()
    evs = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(4)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(st, ev=evs[i] if events_in_timed_loop else None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / steps
    if not events_in_timed_loop:
        for i in range(steps):
            step(st, ev=evs[i])
        torch.cuda.synchronize()
    ms_reduce = sum(e[1].elapsed_time(e[2]) for e in evs) / steps
    per_step = sorted(e[0].elapsed_time(e[3]) for e in evs)
    per_reduce = sorted(e[1].elapsed_time(e[2]) for e in evs)
    # pack and unpack alone, each over its own event-bracketed loop (context only)
    p = st["plan"]

    def loop(fn):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(steps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / steps

    ms_pack = loop(lambda: p.kt_bucket_pack(-1, st["a_local"], st["a_slot0"]))
    ms_unpack = loop(lambda: p.kt_bucket_unpack_scale(-1, st["a_outs"], 1.0, st["a_result"]))
    ms_reduce_alone = loop(lambda: p.kt_weighted_reduce(-1, st["a_peers"], st["K"], st["a_w"], st["a_outs"]))
    # the fused single pass (same results, (K+1)*s bytes per element): reported beside the
    # chained step, never mixed into `value`
    ms_fused = loop(lambda: p.kt_fused_step(-1, st["a_local"], st["a_others"], st["K"], st["a_w"], 1.0,
                                            st["a_result"]))
    # the same pass writing its result over the local gradients (what a gradient hook does)
    ms_fused_inplace = loop(lambda: p.kt_fused_step(-1, st["a_local"], st["a_others"], st["K"], st["a_w"], 1.0,
                                                    st["a_local"]))
    # unpack fused with SGD momentum / weight decay: reads the bucket, p and v, writes p and v
    import torch as _t
    params = [_t.zeros(t.numel(), dtype=_t.float32, device=dev) for t in st["local"]]
    moms = [_t.zeros(t.numel(), dtype=_t.float32, device=dev) for t in st["local"]]
    a_p, a_v = p.marshal(params), p.marshal(moms)
    ms_sgd = loop(lambda: p.kt_bucket_unpack_sgd(-1, st["a_outs"], 1.0, a_p, a_v, 0.1, 0.9, 5e-4, False))
    # the same with a bf16 model copy written beside the binary32 master parameters (mixed precision)
    models = [_t.zeros(t.numel(), dtype=_t.bfloat16, device=dev) for t in st["local"]]
    a_m = p.marshal(models)
    ms_sgd_master = loop(lambda: p.kt_bucket_unpack_sgd_master(-1, st["a_outs"], 1.0, a_p, a_v, a_m, 0.1, 0.9, 5e-4,
                                                               False))
    # K gradient copies -> updated parameters in one pass: K*s + 16 bytes per element (+ 2 with the model copy)
    ms_fsgd = loop(lambda: p.kt_fused_step_sgd(-1, st["a_local"], st["a_others"], st["K"], st["a_w"], 1.0, a_p, a_v, None,
                                               0.1, 0.9, 5e-4, False))
    ms_fsgd_master = loop(lambda: p.kt_fused_step_sgd(-1, st["a_local"], st["a_others"], st["K"], st["a_w"], 1.0, a_p, a_v,
                                                      a_m, 0.1, 0.9, 5e-4, False))
    del params, moms, models
    # the chained step recorded once into a HIP graph and replayed (launch-bound small sets);
    # optional context: a failure here must not take the headline measurement down
    ms_graph = None
    try:
        graph = torch.cuda.CUDAGraph()
        step(st)        # the calls above used more pointer sets than the library keeps resident (8)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            step(st)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t0) * 1e3 / steps
        del graph
    except Exception as exc:                     # noqa: BLE001
        print("bench.py: graph replay skipped: %r" % (exc,), file=sys.stderr)
    e, s, K = w.total_elems, w.elem_size, st["K"]
    res = {
        "workload": name, "elements": e, "buckets": st["nb"], "K": K,
        "ms_per_step": ms_step,
        "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "reduce_ms_median": per_reduce[len(per_reduce) // 2], "reduce_ms_min": per_reduce[0],
        "step_GBps": (K + 5) * s * e / (ms_step * 1e-3) / 1e9,
        "buckets_per_s": st["nb"] / (ms_step * 1e-3),
        "reduce_ms_in_step": ms_reduce,
        "reduce_GBps": (K + 1) * s * e / (ms_reduce * 1e-3) / 1e9,
        "reduce_ms_alone": ms_reduce_alone,
        "pack_ms": ms_pack, "pack_GBps": 2 * s * e / (ms_pack * 1e-3) / 1e9,
        "unpack_ms": ms_unpack, "unpack_GBps": 2 * s * e / (ms_unpack * 1e-3) / 1e9,
        "fused_ms": ms_fused, "fused_GBps": (K + 1) * s * e / (ms_fused * 1e-3) / 1e9,
        "fused_buckets_per_s": st["nb"] / (ms_fused * 1e-3),
        "fused_inplace_ms": ms_fused_inplace, "fused_inplace_GBps": (K + 1) * s * e / (ms_fused_inplace * 1e-3) / 1e9,
        "unpack_sgd_ms": ms_sgd, "unpack_sgd_GBps": (s + 16) * e / (ms_sgd * 1e-3) / 1e9,
        "unpack_sgd_master_ms": ms_sgd_master, "unpack_sgd_master_GBps": (s + 18) * e / (ms_sgd_master * 1e-3) / 1e9,
        "fused_sgd_ms": ms_fsgd, "fused_sgd_GBps": (K * s + 16) * e / (ms_fsgd * 1e-3) / 1e9,
        "fused_sgd_buckets_per_s": st["nb"] / (ms_fsgd * 1e-3),
        "fused_sgd_master_ms": ms_fsgd_master, "fused_sgd_master_GBps": (K * s + 18) * e / (ms_fsgd_master * 1e-3) / 1e9,
    }
    if ms_graph:
        res.update({"graph_step_ms": ms_graph, "graph_step_GBps": (K + 5) * s * e / (ms_graph * 1e-3) / 1e9,
                    "graph_buckets_per_s": st["nb"] / (ms_graph * 1e-3)})
    return res, st


def wl_total(name):
    from paper_2505_10183_amd import workloads as wl
    return wl.get(name).total_elems


def host_threads():
    """(cores the host reports, threads the baseline uses).  The thread count is capped by
    the CPU share the machine grants a job (its OMP_NUM_THREADS setting), not by the core count."""
    cores = os.cpu_count() or 1
    try:
        cores_usable = len(os.sched_getaffinity(0))
    except AttributeError:
        cores_usable = cores
    cap = int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or 16
    return cores, max(1, min(cores_usable, cap))


def cpu_baseline(st, budget_elems):
    """The CPU checker as it stands (strict binary32 mode S: the arithmetic the GPU path
    performs) on the same workload, same inputs, one pack + reduce + unpack-scale pass per
    bucket: first on one host thread over the first buckets, then with one bucket per thread
    on all the threads this job may use, over up to two rounds of buckets."""
    from concurrent.futures import ThreadPoolExecutor
    import oracle
    from paper_2505_10183_amd import workloads as wl

    w, plan, K = st["w"], st["plan"], st["K"]
    nb = st["nb"]
    cores, threads = host_threads()
    wts = oracle.share_weights(oracle.plan_shares(w.throughputs, w.global_batch), w.global_batch)

    def fetch(b):
        n, first, cnt = plan.bucket_info(b)
        numels = w.numels[first:first + cnt]
        lay = oracle.assign_buckets(numels, w.elem_size, 0, ALIGN_BYTES)
        loc = [wl.to_host_array(st["local"][t]) for t in range(first, first + cnt)]
        others = [wl.to_host_array(st["peers"][k][b]) for k in range(1, K)]
        return lay, numels, loc, others

    def one_bucket(item):
        lay, numels, loc, others = item
        slot0 = oracle.pack(lay, loc, w.dtype)[0]
        red = oracle.weighted_reduce([slot0] + others, wts, w.dtype, "S")
        oracle.unpack_scale(lay, [red], numels, 1.0, w.dtype, "S")
        return sum(numels)

    def pick(limit_elems, limit_buckets):
        chosen, total = [], 0
        for b in range(nb):
            n = plan.bucket_info(b)[0]
            if chosen and (total + n > limit_elems or len(chosen) >= limit_buckets):
                break
            chosen.append(b)
            total += n
        return chosen

    single = pick(budget_elems, nb)
    items = [fetch(b) for b in single]
    t0 = time.perf_counter()
    payload1 = sum(one_bucket(it) for it in items)
    secs1 = time.perf_counter() - t0
    many = pick(8 * budget_elems, 2 * threads)
    items += [fetch(b) for b in many[len(single):]]
    items = items[:len(many)]
    with ThreadPoolExecutor(threads) as pool:
        t0 = time.perf_counter()
        payloadN = sum(pool.map(one_bucket, items))
        secsN = time.perf_counter() - t0
    bytes_per_elem = (K + 5) * w.elem_size
    return {"value": bytes_per_elem * payloadN / secsN / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "mode": "S (binary32 product, then fused multiply-adds in ascending k)",
            "threads_used": threads, "host_cores": cores,
            "single_thread_value": bytes_per_elem * payload1 / secs1 / 1e9,
            "sample": "buckets 0..%d of %s (%d of %d elements), one pack+reduce+unpack pass, one bucket per "
                      "thread on %d threads, %.1f s" % (many[-1], w.name, payloadN, w.total_elems, threads, secsN),
            "single_thread_sample": "buckets 0..%d (%d elements), the same pass on one thread, %.1f s"
                                    % (single[-1], payload1, secs1)}


def two_level(dev, name="vit_b16", reps=5):
    """The two-level combination (reduction inside each group of homogeneous devices, then
    across groups through host memory) on one workload: 8 peers in 2 groups of 4; level 1
    reduces this device's group on the GPU, level 2 combines its result with the other
    group's result, which it reads straight from pinned host memory (the stand-in for the
    relay between groups).  Context: what the host hop costs next to the flat K = 8 reduce."""
    import ctypes
    import torch
    import paper_2505_10183_amd as kt
    from paper_2505_10183_amd import workloads as wl
    w = wl.get(name)
    K, G = w.K, 2
    group_of = [0] * (K // 2) + [1] * (K - K // 2)
    plan = kt.Plan(w.numels, w.dtype, w.bucket_cap_bytes, ALIGN_BYTES)
    shares, flat_w = kt.kt_plan_shares(w.throughputs, w.global_batch)
    w1, w2, _ = kt.kt_plan_group_weights(shares, group_of, G)
    nb, elems, td = plan.num_buckets, plan.bucket_elems(), wl.torch_dtype(w.dtype)
    mine = [k for k in range(K) if group_of[k] == 0]
    peers = [[wl.flat_normal(n, w.dtype, w.sigma, 31 * k + b, dev) for b, n in enumerate(elems)] for k in range(K)]
    y0 = [torch.empty(n, dtype=td, device=dev) for n in elems]
    remote = [torch.empty(n, dtype=td, pin_memory=True).normal_(0, w.sigma) for n in elems]
    out = [torch.empty(n, dtype=td, device=dev) for n in elems]
    a_l1 = plan.marshal([peers[k][b] for b in range(nb) for k in mine])
    a_l2 = plan.marshal([t for b in range(nb) for t in (y0[b], remote[b])])
    a_flat = plan.marshal([peers[k][b] for b in range(nb) for k in range(K)])
    a_y0, a_out = plan.marshal(y0), plan.marshal(out)
    c_w1 = (ctypes.c_float * len(mine))(*[w1[k] for k in mine])
    c_w2 = (ctypes.c_float * G)(*w2)
    c_wf = (ctypes.c_float * K)(*flat_w)

    def loop(fn):
        fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    ms1 = loop(lambda: plan.kt_weighted_reduce(-1, a_l1, len(mine), c_w1, a_y0))
    ms2 = loop(lambda: plan.kt_weighted_reduce(-1, a_l2, G, c_w2, a_out))
    msf = loop(lambda: plan.kt_weighted_reduce(-1, a_flat, K, c_wf, a_out))
    byts = w.total_elems * w.elem_size
    return {"workload": name, "groups": "2 groups of %d devices" % (K // 2),
            "level1_ms": round(ms1, 4), "level1_GBps": round((len(mine) + 1) * byts / ms1 / 1e6, 1),
            "level2_from_pinned_host_ms": round(ms2, 4),
            "level2_host_read_GBps": round(byts / ms2 / 1e6, 1),
            "flat_reduce_ms": round(msf, 4)}


def call_cost(dev, n=5000):
    """Host cost of one device call on a launch-bound set (the MLP set, K = 2): wall time per
    call over n back-to-back kt_weighted_reduce calls, through the binding and straight
    through ctypes, next to PyTorch's own smallest launch (an in-place add on 1024 floats)."""
    import torch
    from paper_2505_10183_amd import binding
    st = setup("mlp", dev)
    p, K, L = st["plan"], st["K"], binding.lib()
    stream = binding._stream(None)
    x = torch.zeros(1024, device=dev)

    def per_call(fn):
        for _ in range(200):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return round((time.perf_counter() - t0) / n * 1e6, 2)

    return {"binding_us": per_call(lambda: p.kt_weighted_reduce(-1, st["a_peers"], K, st["a_w"], st["a_outs"])),
            "c_abi_us": per_call(lambda: L.kt_weighted_reduce(p._h, -1, st["a_peers"], K, st["a_w"], st["a_outs"], stream)),
            "torch_add_us": per_call(lambda: x.add_(1))}


def host_rows():
    """Wall time of the host-only entry points at a realistic size (milliseconds)."""
    import paper_2505_10183_amd as kt
    shares, _ = kt.kt_plan_shares([1, 1, .8, .8, .6, .6, .4, .4], 1024)
    t0 = time.perf_counter()
    idx = kt.kt_sampler_epoch(1281167, 1024, shares, 1, 0, 3)
    t1 = time.perf_counter()
    ema = [0.0] * 8
    for _ in range(1000):
        ema, shares, _ = kt.kt_replan_shares([1.0, 1.1, 1.3, 1.2, 1.7, 1.6, 2.4, 2.6], shares, ema, 0.2, 1024)
    t2 = time.perf_counter()
    return {"sampler_epoch_N1281167_B1024_K8_ms": round((t1 - t0) * 1e3, 2), "indices": len(idx),
            "replan_shares_K8_us": round((t2 - t1) * 1e3, 3)}


def load_probe():
    """bench_probe.hip built beside this file (libkt_bench_probe.so); None if it is not built."""
    import ctypes
    path = os.path.join(ROOT, "libkt_bench_probe.so")
    if not os.path.exists(path):
        return None
    lib = ctypes.CDLL(path)
    lib.bench_probe_read.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_int64, ctypes.c_void_p,
                                     ctypes.c_void_p]
    lib.bench_probe_read.restype = ctypes.c_int64
    return lib


def ceilings(dev, reps=10):
    """What the memory system sustains on flat 1 GiB buffers: a read-only stream of 8 buffers
    (bench_probe.hip: the reduce's loads with nothing stored), a plain copy (kt_weighted_reduce
    with K = 1, w = 1) and the 8:1 read:write mix of the reduce itself, in place and out of
    place.  Context for the roofline fraction: the 8 TB/s peak is not reachable even by pure reads."""
    import ctypes
    import torch
    import paper_2505_10183_amd as kt
    n = 1 << 28                                   # fp32 elements = 1 GiB per buffer
    bufs = [torch.empty(n, dtype=torch.float32, device=dev).normal_() for _ in range(8)]
    out = torch.empty(n, dtype=torch.float32, device=dev)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    plan = kt.Plan([n], "f32", 0, 16)
    a8, a1, ao, a0 = plan.marshal(bufs), plan.marshal(bufs[:1]), plan.marshal([out]), plan.marshal(bufs[:1])
    w8 = (ctypes.c_float * 8)(*([0.125] * 8))
    w1 = (ctypes.c_float * 1)(1.0)

    def loop(fn):
        for _ in range(3):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps * 1e-3

    gib = float(n * 4)
    res = {"buffers": "flat 1 GiB fp32 each"}
    probe = load_probe()
    if probe is not None:
        stream = torch.cuda.current_stream().cuda_stream

        def read_only():
            got = probe.bench_probe_read(a8, 8, int(gib), sink.data_ptr(), stream)
            assert got == int(gib), got
        res["read_only_8_streams_GBps"] = round(8 * gib / loop(read_only) / 1e9, 1)
    t_copy = loop(lambda: plan.kt_weighted_reduce(-1, a1, 1, w1, ao))
    t_mix = loop(lambda: plan.kt_weighted_reduce(-1, a8, 8, w8, ao))
    t_mix_in = loop(lambda: plan.kt_weighted_reduce(-1, a8, 8, w8, a0))
    res.update({"copy_GBps": round(2 * gib / t_copy / 1e9, 1),
                "reduce_8_reads_1_write_GBps": round(9 * gib / t_mix / 1e9, 1),
                "reduce_8_reads_1_write_in_place_GBps": round(9 * gib / t_mix_in / 1e9, 1)})
    # more peers than the kernels are specialised for (K > 8: peers taken in chunks)
    more = [torch.empty(n, dtype=torch.float32, device=dev).normal_() for _ in range(8)]
    a16 = plan.marshal(bufs + more)
    w16 = (ctypes.c_float * 16)(*([0.0625] * 16))
    t16 = loop(lambda: plan.kt_weighted_reduce(-1, a16, 16, w16, a0))
    res["reduce_16_reads_1_write_in_place_GBps"] = round(17 * gib / t16 / 1e9, 1)
    del more
    assert float(sink.abs().sum()) == 0.0
    return res


def k_sweep(dev, reps=10, passes=2):
    """Flat 1 GiB fp32 buffers, K = 1..8 peers: the read-only probe on K buffers, kt_weighted_reduce of
    K buffers into another, and in place over the first.  Prints one line per K and pass: GB/s of
    (K reads [+ 1 write]) x 1 GiB and the times, from which the cost of the written gigabyte on
    top of the reads follows."""
    import ctypes
    import torch
    import paper_2505_10183_amd as kt
    n = 1 << 28
    bufs = [torch.empty(n, dtype=torch.float32, device=dev).normal_() for _ in range(8)]
    out = torch.empty(n, dtype=torch.float32, device=dev)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    plan = kt.Plan([n], "f32", 0, 16)
    probe = load_probe()
    if probe is None:
        raise RuntimeError("libkt_bench_probe.so is not built")
    stream = torch.cuda.current_stream().cuda_stream
    gib = float(n * 4)

    def loop(fn):
        for _ in range(3):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps * 1e-3

    ao, a0 = plan.marshal([out]), plan.marshal(bufs[:1])
    print("# flat 1 GiB fp32 buffers; GB/s of (K reads [+ 1 write]) x 1 GiB; %d launches after 3 warm-up" % reps)
    print("# K  read_only  reduce_out_of_place  reduce_in_place  |  ms: read_only  out_of_place  in_place")
    for _ in range(passes):
        for K in (1, 2, 3, 4, 6, 8):
            ak = plan.marshal(bufs[:K])
            w = (ctypes.c_float * K)(*([1.0 / K] * K))
            tr = loop(lambda: probe.bench_probe_read(ak, K, int(gib), sink.data_ptr(), stream))
            to = loop(lambda: plan.kt_weighted_reduce(-1, ak, K, w, ao))
            ti = loop(lambda: plan.kt_weighted_reduce(-1, ak, K, w, a0))
            print("  %d  %9.1f  %19.1f  %15.1f  |  %13.4f  %12.4f  %8.4f"
                  % (K, K * gib / tr / 1e9, (K + 1) * gib / to / 1e9, (K + 1) * gib / ti / 1e9, tr * 1e3, to * 1e3, ti * 1e3))
            sys.stdout.flush()
    assert float(sink.abs().sum()) == 0.0
    plan.close()


def ab_compare(workload, kernel_names, variants, dev, rounds=5, reps=10):
    """Interleaved comparison of library builds (paper_2505_10183_amd/build.py --out ... -D...)
    in ONE process on ONE set of device buffers: every round times every kernel on every
    build in turn, so that machine drift (a few per cent between runs and boxes) hits all
    builds alike.  Prints one line per (kernel, build): median and best of the per-round
    means, in GB/s of algorithmic bytes.  Also times the same kernels with the gradient /
    parameter tensors laid out as views into flat buffers with the bucket layout
    (`*_views`: their addresses are then congruent with the bucket's 16 KiB tiles) and the
    chained step launched bucket by bucket instead of batched (`step_per_bucket`)."""
    import statistics
    import torch
    import paper_2505_10183_amd as kt
    from paper_2505_10183_amd import binding

    st = setup(workload, dev)
    w, K, nb = st["w"], st["K"], st["nb"]
    e, s = w.total_elems, w.elem_size
    libs, plans = {}, {}
    for name, path in variants:
        binding._lib = None
        binding.LIB_PATH = os.path.abspath(path)
        libs[name] = binding.lib()
        plans[name] = kt.Plan(w.numels, w.dtype, w.bucket_cap_bytes, ALIGN_BYTES)
        plans[name].kt_plan_set_weights(st["a_w"])
        plans[name].kt_plan_set_sgd(1.0, 0.1, 0.9, 5e-4)
    td = st["local"][0].dtype
    elems = st["plan"].bucket_elems()
    flat_l = [torch.empty(n, dtype=td, device=dev).normal_(0, w.sigma) for n in elems]
    flat_o = [torch.empty(n, dtype=td, device=dev) for n in elems]
    flat_p = [torch.zeros(n, dtype=torch.float32, device=dev) for n in elems]
    flat_v = [torch.zeros(n, dtype=torch.float32, device=dev) for n in elems]
    view_l, view_o, view_p, view_v = [], [], [], []
    for t, n in enumerate(w.numels):
        b, off = st["plan"].tensor_info(t)
        view_l.append(flat_l[b][off:off + n])
        view_o.append(flat_o[b][off:off + n])
        view_p.append(flat_p[b][off:off + n])
        view_v.append(flat_v[b][off:off + n])
    params = [torch.zeros(n, dtype=torch.float32, device=dev) for n in w.numels]
    moms = [torch.zeros(n, dtype=torch.float32, device=dev) for n in w.numels]
    models = [torch.zeros(n, dtype=torch.bfloat16, device=dev) for n in w.numels]
    m = st["plan"].marshal
    a_vl, a_vo, a_vp, a_vv, a_p, a_v = m(view_l), m(view_o), m(view_p), m(view_v), m(params), m(moms)
    a_m = m(models)
    a_l, a_s0, a_pe, a_ot, a_o, a_r, a_w = (st["a_local"], st["a_slot0"], st["a_peers"], st["a_others"], st["a_outs"],
                                            st["a_result"], st["a_w"])

    def table(p):
        def per_bucket():
            for b in range(nb):
                p.kt_bucket_pack(b, a_l, a_s0)
                p.kt_weighted_reduce(b, a_pe, K, a_w, a_o)
                p.kt_bucket_unpack_scale(b, a_o, 1.0, a_r)

        def batched():
            p.kt_bucket_pack(-1, a_l, a_s0)
            p.kt_weighted_reduce(-1, a_pe, K, a_w, a_o)
            p.kt_bucket_unpack_scale(-1, a_o, 1.0, a_r)
        return {
            "pack": (lambda: p.kt_bucket_pack(-1, a_l, a_s0), 2 * s),
            "pack_views": (lambda: p.kt_bucket_pack(-1, a_vl, a_s0), 2 * s),
            "reduce": (lambda: p.kt_weighted_reduce(-1, a_pe, K, a_w, a_o), (K + 1) * s),
            "reduce_resident_weights": (lambda: p.kt_weighted_reduce(-1, a_pe, K, None, a_o), (K + 1) * s),
            "unpack": (lambda: p.kt_bucket_unpack_scale(-1, a_o, 1.0, a_r), 2 * s),
            "unpack_views": (lambda: p.kt_bucket_unpack_scale(-1, a_o, 1.0, a_vo), 2 * s),
            "step": (batched, (K + 5) * s),
            "step_per_bucket": (per_bucket, (K + 5) * s),
            "fused": (lambda: p.kt_fused_step(-1, a_l, a_ot, K, a_w, 1.0, a_r), (K + 1) * s),
            "fused_scale037": (lambda: p.kt_fused_step(-1, a_l, a_ot, K, a_w, 0.37, a_r), (K + 1) * s),
            "fused_inplace": (lambda: p.kt_fused_step(-1, a_l, a_ot, K, a_w, 1.0, a_l), (K + 1) * s),
            "fused_views": (lambda: p.kt_fused_step(-1, a_vl, a_ot, K, a_w, 1.0, a_vo), (K + 1) * s),
            "fused_views_inplace": (lambda: p.kt_fused_step(-1, a_vl, a_ot, K, a_w, 1.0, a_vl), (K + 1) * s),
            "sgd": (lambda: p.kt_bucket_unpack_sgd(-1, a_o, 1.0, a_p, a_v, 0.1, 0.9, 5e-4, False), s + 16),
            "sgd_master": (lambda: p.kt_bucket_unpack_sgd_master(-1, a_o, 1.0, a_p, a_v, a_m, 0.1, 0.9, 5e-4, False), s + 18),
            "sgd_views": (lambda: p.kt_bucket_unpack_sgd(-1, a_o, 1.0, a_vp, a_vv, 0.1, 0.9, 5e-4, False), s + 16),
            "fused_sgd": (lambda: p.kt_fused_step_sgd(-1, a_l, a_ot, K, a_w, 1.0, a_p, a_v, None, 0.1, 0.9, 5e-4, False),
                          K * s + 16),
            "fused_sgd_master": (lambda: p.kt_fused_step_sgd(-1, a_l, a_ot, K, a_w, 1.0, a_p, a_v, a_m, 0.1, 0.9, 5e-4,
                                                             False), K * s + 18),
            "fused_sgd_views": (lambda: p.kt_fused_step_sgd(-1, a_vl, a_ot, K, a_w, 1.0, a_vp, a_vv, None, 0.1, 0.9, 5e-4,
                                                            False), K * s + 16),
            "sgd_resident_scalars": (lambda: p.kt_bucket_unpack_sgd_resident(-1, a_o, a_p, a_v, None, False), s + 16),
        }

    def timeit(fn):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        fn()
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    res = {(v, k): [] for v, _ in variants for k in kernel_names}
    for _ in range(rounds):
        for k in kernel_names:
            for v, _ in variants:
                binding._lib = libs[v]
                res[(v, k)].append(timeit(table(plans[v])[k][0]))
    print("# %s: %d elements %s, K=%d, %d buckets; %d rounds x %d launches per (kernel, build), interleaved"
          % (w.name, e, w.dtype, K, nb, rounds, reps))
    print("# %-20s %-12s %10s %9s %7s %10s %9s" % ("kernel", "build", "median_ms", "GB/s", "% peak", "best_ms", "GB/s"))
    for k in kernel_names:
        bpe = table(plans[variants[0][0]])[k][1]
        for v, _ in variants:
            t = res[(v, k)]
            med, mn = statistics.median(t), min(t)
            print("  %-20s %-12s %10.4f %9.1f %7.1f %10.4f %9.1f"
                  % (k, v, med, bpe * e / med / 1e6, bpe * e / med / 1e6 / (HBM_PEAK_GBS / 100), mn, bpe * e / mn / 1e6))
    sys.stdout.flush()
    for v, _ in variants:
        binding._lib = libs[v]
        plans[v].close()
    binding._lib = libs[variants[0][0]]
    st["plan"].close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="decoder_1p3b")
    ap.add_argument("--also", default="vit_b16,resnet18,mobilenetv2,mlp",
                    help="comma list of further workloads reported for context (the three small ones are "
                         "cache-resident and launch-bound: not comparable with the HBM peak)")
    ap.add_argument("--cpu-elems", type=int, default=0, help="element budget of the CPU baseline sample (0 = auto)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--out-of-place", action="store_true", help="reduce into separate output buffers")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the memory-system probe")
    ap.add_argument("--lib", default="", help="load this build of libkt.so instead of the in-tree one "
                                              "(variants made with paper_2505_10183_amd/build.py --out)")
    ap.add_argument("--align", type=int, default=16,
                    help="align_bytes of the bucket plan (16 as in the workload definitions; 16384 puts every "
                         "tensor on a tile boundary)")
    ap.add_argument("--misalign", action="store_true",
                    help="offset every bucket buffer by one element: the library then takes its "
                         "element-wise (4-byte / 2-byte) kernels instead of the 16-byte ones")
    ap.add_argument("--ab", default="", help="interleaved comparison of library builds: comma list of name=path "
                                             "(see ab_compare); prints a table instead of the JSON line")
    ap.add_argument("--kernels", default="reduce,fused,sgd", help="kernels compared by --ab")
    ap.add_argument("--rounds", type=int, default=5, help="rounds of --ab")
    ap.add_argument("--ceilings-only", action="store_true",
                    help="run only the memory-system probes on flat 1 GiB buffers and print their JSON "
                         "(the command the counter summaries under profiles/ are taken with)")
    ap.add_argument("--k-sweep", action="store_true",
                    help="read-only probe and reduce on flat 1 GiB buffers for K = 1..8; prints a table")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain 1 GiB device copy (torch copy_) three times, so that a counter "
                         "trace of this command holds a kernel of known traffic to scale FETCH_SIZE/WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (no collectives between GPUs); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    global ALIGN_BYTES
    ALIGN_BYTES = args.align
    if args.lib:
        from paper_2505_10183_amd import binding
        binding.LIB_PATH = os.path.abspath(args.lib)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU available", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.ab:
        variants = [tuple(x.split("=", 1)) for x in args.ab.split(",") if x]
        ab_compare(args.workload, [k for k in args.kernels.split(",") if k], variants, dev,
                   rounds=args.rounds, reps=10)
        return
    if args.calibrate:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()

    if args.ceilings_only:
        print(json.dumps({"memory_system": ceilings(dev)}))
        return
    if args.k_sweep:
        k_sweep(dev)
        return
    res, st = time_workload(args.workload, args.steps, args.warmup, dev, not args.out_of_place, args.misalign)
    w = st["w"]
    cpu = None
    if not args.no_cpu:
        budget = args.cpu_elems or (200_000_000 if w.dtype == "bf16" else 400_000_000)
        try:
            cpu = cpu_baseline(st, budget)
        except Exception as exc:                 # noqa: BLE001
            print("bench.py: CPU baseline failed: %r" % (exc,), file=sys.stderr)
    also = {}
    del st
    torch.cuda.empty_cache()
    for name in [x for x in args.also.split(",") if x and x != args.workload]:
        try:
            # the context workloads are short: at least 100 timed steps after 20 warm-up steps
            r, s2 = time_workload(name, max(args.steps, 100), max(args.warmup, 20), dev, not args.out_of_place,
                                  args.misalign, events_in_timed_loop=wl_total(name) >= 50_000_000)
            r["steps"], r["warmup"] = max(args.steps, 100), max(args.warmup, 20)
            also[name] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items()}
            del s2
        except Exception as exc:                 # noqa: BLE001
            also[name] = {"error": repr(exc)}
        torch.cuda.empty_cache()

    extra = {}
    if not args.no_ceilings:
        for key, fn in (("two_level", lambda: two_level(dev)), ("host_rows", host_rows),
                        ("call_cost", lambda: call_cost(dev))):
            try:
                extra[key] = fn()
            except Exception as exc:             # noqa: BLE001
                print("bench.py: %s skipped: %r" % (key, exc), file=sys.stderr)
        torch.cuda.empty_cache()
    ceil = None
    if not args.no_ceilings:
        try:
            ceil = ceilings(dev)
        except Exception as exc:                 # noqa: BLE001
            print("bench.py: memory-system probe skipped: %r" % (exc,), file=sys.stderr)
    line = {
        "metric": "weighted bucket-reduce+pack/unpack HBM GB/s",
        "value": round(res["step_GBps"], 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(res["ms_per_step"], 5),
        "ms_per_step_median": round(res["ms_per_step_median"], 5),
        "ms_per_step_min": round(res["ms_per_step_min"], 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.dtype == "f32" else "f32 accumulate, bf16 storage",
        "data": "synthetic",
        "config": {"workload": "%s: %d tensors, %d elements %s, K=%d, B=%d, %d buckets (cap %d MiB)"
                               % (w.name, len(w.shapes), w.total_elems, w.dtype, w.K, w.global_batch,
                                  res["buckets"], w.bucket_cap_bytes >> 20),
                   "launch": "one batched launch per kernel over all buckets; reduce %s"
                             % ("into its own output buffers" if args.out_of_place else "in place over peer slot 0")
                             + ("; buckets misaligned by one element (element-wise kernels)" if args.misalign else "")
                             + ("; tensors aligned to %d bytes inside the buckets" % args.align if args.align != 16 else ""),
                   "bytes_per_element": "(K+5)*s = %d" % ((w.K + 5) * w.elem_size)},
        "pct_of_hbm_peak": round(100.0 * res["step_GBps"] / HBM_PEAK_GBS, 2),
        "buckets_per_s": round(res["buckets_per_s"], 1),
        "kernels": {k: round(v, 4) for k, v in res.items() if k.endswith(("_ms", "_GBps", "_in_step", "_alone", "_per_s", "_median", "_min"))
                    and k not in ("buckets_per_s", "ms_per_step_median", "ms_per_step_min")},
        "roofline": {"kernel": "kt_weighted_reduce (kt_reduce_kernel, K=%d, %s)" % (w.K, w.dtype),
                     "bound": "hbm", "achieved": round(res["reduce_GBps"], 2), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(res["reduce_GBps"] / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic(w.name), "traffic_unit": "bytes per launch",
                     "traffic_source": "profiles/kt_kernels_%s.txt (FETCH_SIZE / WRITE_SIZE counter runs of this "
                                       "command, not of this run; null once the kernel sources have changed)" % w.name},
        "memory_system": ceil,
        "cpu_baseline": cpu,
        "two_level": extra.get("two_level"),
        "host_rows": extra.get("host_rows"),
        "call_cost": extra.get("call_cost"),
        "also": also,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
