"""GPU parity for kt_fused_step_sgd (K gradient copies -> updated parameters in
one pass): bit-identical to the CPU checker's chain pack -> reduce -> unpack
with SGD in its binary32 step mode S, and to the library's own chained calls.
Two steps each (the first writes the momentum without reading it), with and
without the bf16 model copy, canary-guarded parameter allocations."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2505_10183_amd as kt
from paper_2505_10183_amd import workloads as wl
from test_gpu_parity import DEV, host, raw, tdtype

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def announce(request):
    print("\n[gpu-case] %s" % request.node.nodeid, file=sys.stderr, flush=True)
    yield
    torch.cuda.synchronize()


def run_fused_sgd(w, align, scale, lr, mu, wd, K=None, steps=2, misalign=False, bucket_shift=0, per_bucket=False,
                  master=False, weights=None, chained=True):
    dtype = w.dtype
    K = K or w.K
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, align)
    L = oracle.assign_buckets(w.numels, w.elem_size, w.bucket_cap_bytes, align)
    nb, T = plan.num_buckets, len(w.numels)
    if weights is None:
        thr = [1.0 - 0.5 * k / max(1, K - 1) for k in range(K)]
        shares, weights = kt.kt_plan_shares(thr, 64 * K)
        wts = oracle.share_weights(oracle.plan_shares(thr, 64 * K), 64 * K)
        assert np.array(weights, np.float32).tobytes() == wts.tobytes()
    else:
        wts = np.array(weights, np.float32)
    gen = torch.Generator(DEV).manual_seed(w.seed)
    lo = [(1 if (misalign and t % 2) else 4) for t in range(T)]
    p_store = [torch.full((n + 12,), 9.0, device=DEV) for n in w.numels]
    v_store = [torch.full((n + 12,), 9.0, device=DEV) for n in w.numels]
    m_store = [torch.full((n + 12,), 9.0, dtype=torch.bfloat16, device=DEV) for n in w.numels]
    params = [s[l:l + n] for s, l, n in zip(p_store, lo, w.numels)]
    moms = [s[l:l + n] for s, l, n in zip(v_store, lo, w.numels)]
    models = [s[l:l + n] for s, l, n in zip(m_store, lo, w.numels)] if master else None
    for p in params:
        p.copy_(torch.randn(p.shape, generator=gen, device=DEV))
    for v in moms:
        v.fill_(float("nan"))          # must not be read on the first step
    hp, hv = [host(p) for p in params], [host(v) for v in moms]
    # the same state for the library's chained calls
    p2, v2 = [p.clone() for p in params], [v.clone() for v in moms]
    m2 = [torch.zeros(n, dtype=torch.bfloat16, device=DEV) for n in w.numels] if master else None
    elems = plan.bucket_elems()
    for step in range(steps):
        # local gradients (peer 0) as tensors, odd ones only element-aligned when misaligned; peers 1..K-1 as buckets
        g_store = [torch.zeros(n + 12, dtype=tdtype(dtype), device=DEV) for n in w.numels]
        local = [s[l:l + n] for s, l, n in zip(g_store, lo, w.numels)]
        for t, src in zip(local, wl.gradient_set(w, 50 * step, DEV)):
            t.copy_(src.reshape(-1))
        store = [[wl.flat_normal(n + 8, dtype, w.sigma, 7000 + 100 * k + 10 * step + b, DEV) for b, n in enumerate(elems)]
                 for k in range(1, K)]
        peers = [[s[bucket_shift:bucket_shift + n] for s, n in zip(store[k], elems)] for k in range(K - 1)]
        others = [peers[k][b] for b in range(nb) for k in range(K - 1)]
        first = step == 0
        for b in (range(nb) if per_bucket else [-1]):
            plan.kt_fused_step_sgd(b, local, others, K, weights, scale, params, moms, models, lr, mu, wd, first)
        torch.cuda.synchronize()
        # checker: pack the local tensors, reduce with the peers, unpack with SGD
        hl = [host(t) for t in local]
        slot0 = oracle.pack(L, hl, dtype)
        hb = [oracle.weighted_reduce([slot0[b]] + [host(peers[k][b]) for k in range(K - 1)], wts, dtype, "S")
              for b in range(nb)]
        if master:
            hp, hv, hm = oracle.unpack_sgd_master(L, hb, w.numels, scale, hp, hv, lr, mu, wd, first, dtype, "S")
        else:
            hp, hv = oracle.unpack_sgd(L, hb, w.numels, scale, hp, hv, lr, mu, wd, first, dtype, "S")
        for t, n in enumerate(w.numels):
            assert raw(host(params[t])).tobytes() == raw(hp[t]).tobytes(), ("param", step, t)
            assert raw(host(moms[t])).tobytes() == raw(hv[t]).tobytes(), ("momentum", step, t)
            assert raw(host(local[t])).tobytes() == raw(hl[t]).tobytes(), ("gradient untouched", step, t)
            stores = [p_store[t], v_store[t]] + ([m_store[t]] if master else [])
            if master:
                assert host(models[t]).tobytes() == hm[t].tobytes(), ("model copy", step, t)
            for s_ in stores:
                assert bool((s_[:lo[t]] == 9.0).all()) and bool((s_[lo[t] + n:] == 9.0).all()), ("canary", step, t)
        if chained:
            s0 = [torch.empty(n, dtype=tdtype(dtype), device=DEV) for n in elems]
            plan.kt_bucket_pack(-1, local, s0)
            flat = [([s0] + peers)[k][b] for b in range(nb) for k in range(K)]
            plan.kt_weighted_reduce(-1, flat, K, weights, s0)
            if master:
                plan.kt_bucket_unpack_sgd_master(-1, s0, scale, p2, v2, m2, lr, mu, wd, first)
            else:
                plan.kt_bucket_unpack_sgd(-1, s0, scale, p2, v2, lr, mu, wd, first)
            torch.cuda.synchronize()
            for t in range(T):
                assert raw(host(params[t])).tobytes() == raw(host(p2[t])).tobytes(), ("param vs chained", step, t)
                assert raw(host(moms[t])).tobytes() == raw(host(v2[t])).tobytes(), ("momentum vs chained", step, t)
                if master:
                    assert host(models[t]).tobytes() == host(m2[t]).tobytes(), ("model vs chained", step, t)
    plan.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("K", [1, 2, 3, 5, 8, 9, 13])
def test_fused_sgd_ragged_every_K(dtype, K):
    w = wl.ragged_workload(dtype=dtype, K=K, seed=300 + K)
    run_fused_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, master=(K % 2 == 1))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("master", [False, True])
def test_fused_sgd_layouts(dtype, master):
    w = wl.ragged_workload(dtype=dtype, K=4, seed=93)
    run_fused_sgd(w, 16, 0.37, 0.05, 0.9, 5e-4, per_bucket=True, master=master)
    run_fused_sgd(w, w.elem_size, 1.0, 0.1, 0.9, 5e-4, master=master)               # dense packing
    run_fused_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, misalign=True, master=master)         # element-aligned tensors
    run_fused_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, bucket_shift=1, master=master)        # element-aligned buckets
    run_fused_sgd(w, 16384, 0.5, 0.1, 0.9, 5e-4, master=master)                     # tensors on tile boundaries
    run_fused_sgd(w, 16, 1.0, 0.1, 0.0, 0.0, steps=1, master=master)                # plain SGD
    run_fused_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, K=11, misalign=True, master=master)   # K > 8, mixed alignments


def test_fused_sgd_tiny_and_many_tensors():
    numels = [1, 3, 5, 7, 2, 1, 1, 6, 4, 1] * 100 + [30000] + [4] * 1500
    for dtype in ("f32", "bf16"):
        w = wl.Workload("tm", dtype, tuple((n,) for n in numels), (1.0, 0.5, 0.5), 96, 0, 1e-2, 17)
        run_fused_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, master=(dtype == "bf16"))


def test_fused_sgd_special_values_and_one_hot_weights():
    """One-hot weights select a peer exactly (the update then equals SGD on that peer's gradient);
    zero-size tensors are skipped."""
    w = wl.Workload("oh", "f32", ((0,), (5000,), (0,), (3,), (70001,)), (1.0, 1.0, 1.0), 3, 32 * 1024, 1e-2, 23)
    run_fused_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, weights=[0.0, 1.0, 0.0])
    run_fused_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, weights=[1.0, 0.0, 0.0], master=True)


@pytest.mark.parametrize("name", ["mlp", "mobilenetv2", "resnet18", "vit_b16"])
def test_fused_sgd_workloads(name):
    w = wl.WORKLOADS[name]
    _, weights = kt.kt_plan_shares(w.throughputs, w.global_batch)
    run_fused_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, weights=weights, master=(name == "vit_b16"))


def test_fused_sgd_resident_weights_and_scalars_in_a_graph():
    """kt_fused_step_sgd_resident: weights from kt_plan_set_weights, scalars from kt_plan_set_sgd; one
    recording follows re-planned shares and a stepped learning rate."""
    K = 4
    w = wl.ragged_workload(dtype="bf16", K=K, seed=94, n_tensors=30)
    plan = kt.Plan(w.numels, "bf16", w.bucket_cap_bytes, 16)
    L = oracle.assign_buckets(w.numels, 2, w.bucket_cap_bytes, 16)
    nb, T = plan.num_buckets, len(w.numels)
    local = wl.gradient_set(w, 0, DEV)
    peers = [[wl.flat_normal(n, "bf16", w.sigma, 60 * k + b, DEV) for b, n in enumerate(plan.bucket_elems())]
             for k in range(1, K)]
    others = [peers[k][b] for b in range(nb) for k in range(K - 1)]
    gen = torch.Generator(DEV).manual_seed(11)
    params = [torch.randn(n, generator=gen, device=DEV) for n in w.numels]
    moms = [torch.full((n,), float("nan"), device=DEV) for n in w.numels]
    models = [torch.zeros(n, dtype=torch.bfloat16, device=DEV) for n in w.numels]
    hp, hv = [host(p) for p in params], [host(v) for v in moms]
    hl = [host(t) for t in local]
    slot0 = oracle.pack(L, hl, "bf16")
    hpeers = [[host(peers[k][b]) for k in range(K - 1)] for b in range(nb)]
    state = {"hp": hp, "hv": hv, "hm": None}

    def advance(wv, scale, lr, first):
        wv = np.array(wv, np.float32)
        hb = [oracle.weighted_reduce([slot0[b]] + hpeers[b], wv, "bf16", "S") for b in range(nb)]
        state["hp"], state["hv"], state["hm"] = oracle.unpack_sgd_master(L, hb, w.numels, scale, state["hp"], state["hv"],
                                                                         lr, 0.9, 5e-4, first, "bf16", "S")

    def check(tag):
        torch.cuda.synchronize()
        for t in range(T):
            assert raw(host(params[t])).tobytes() == raw(state["hp"][t]).tobytes(), (tag, "p", t)
            assert raw(host(moms[t])).tobytes() == raw(state["hv"][t]).tobytes(), (tag, "v", t)
            assert host(models[t]).tobytes() == state["hm"][t].tobytes(), (tag, "model", t)

    B = 128
    shares, w_now = kt.kt_plan_shares([1.0, 0.8, 0.5, 0.5], B)
    with pytest.raises(kt.KtError):
        plan.kt_fused_step_sgd_resident(-1, local, others, K, params, moms, models, True)     # no weights yet
    plan.kt_plan_set_weights(w_now)
    with pytest.raises(kt.KtError):
        plan.kt_fused_step_sgd_resident(-1, local, others, K, params, moms, models, True)     # no scalars yet
    plan.kt_plan_set_sgd(1.0, 0.1, 0.9, 5e-4)
    plan.kt_fused_step_sgd_resident(-1, local, others, K, params, moms, models, True)
    advance(w_now, 1.0, 0.1, True)
    check("first step")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        plan.kt_fused_step_sgd_resident(-1, local, others, K, params, moms, models, False)
    torch.cuda.synchronize()
    check("after recording")
    ema = [0.0] * K
    speed = np.array([1.0, 0.8, 0.5, 0.5])
    for r, lr in enumerate([0.1, 0.01, 0.01, 0.001]):
        speed[r % K] *= 0.6
        times = [float(b / s_) for b, s_ in zip(shares, speed)]
        ema, shares, w_now = kt.kt_replan_shares(times, shares, ema, 1.0, B)
        plan.kt_plan_set_weights(w_now)
        plan.kt_plan_set_sgd(0.5, lr, 0.9, 5e-4)
        torch.cuda.synchronize()
        g.replay()
        advance(w_now, 0.5, lr, False)
        check("replay %d" % r)
    plan.close()
