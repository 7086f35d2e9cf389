"""Seeded random plans on the GPU: random tensor sizes, alignment, bucket cap,
peer count and element type, every entry point against the CPU checker's
binary32 step mode (bit-identical) on every element."""
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


def random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    T = int(rng.integers(1, 60))
    kinds = rng.integers(0, 5, size=T)
    numels = []
    for k in kinds:
        numels.append(int({0: rng.integers(0, 9), 1: rng.integers(1, 300), 2: rng.integers(300, 6000),
                           3: rng.integers(4000, 4200), 4: rng.integers(6000, 40000)}[int(k)]))
    dtype = "f32" if rng.integers(0, 2) else "bf16"
    es = 4 if dtype == "f32" else 2
    align = int(rng.choice([es, 16, 16, 64, 1024, 16384]))
    cap = int(rng.choice([0, 32 * 1024, 200 * 1024]))
    K = int(rng.integers(1, 10))
    thr = tuple(float(x) for x in np.round(rng.uniform(0.2, 1.0, size=K), 2))
    B = int(rng.choice([64, 96, 1000, 1024]))
    scale = float(rng.choice([1.0, 0.5, 0.37]))
    return wl.Workload("rand%d" % seed, dtype, tuple((n,) for n in numels), thr, B, cap, 1e-3, 4000 + seed), align, scale


@pytest.mark.parametrize("seed", range(24))
def test_random_plan(seed):
    w, align, scale = random_case(seed)
    K, dtype = w.K, w.dtype
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, align)
    L = oracle.assign_buckets(w.numels, w.elem_size, w.bucket_cap_bytes, align)
    nb = plan.num_buckets
    assert plan.bucket_elems() == L["bucket_elems"]
    shares, weights = kt.kt_plan_shares(w.throughputs, w.global_batch)
    assert shares == oracle.plan_shares(w.throughputs, w.global_batch)
    wts = oracle.share_weights(shares, w.global_batch)
    grads = [wl.gradient_set(w, k, DEV) for k in range(K)]
    hg = [[host(t) for t in g] for g in grads]
    # chained path
    peers = [[torch.full((n,), 3.0, dtype=tdtype(dtype), device=DEV) for n in plan.bucket_elems()] for _ in range(K)]
    for k in range(K):
        plan.kt_bucket_pack(-1, grads[k], peers[k])
    torch.cuda.synchronize()
    for k in range(K):
        want = oracle.pack(L, hg[k], dtype)
        for b in range(nb):
            assert raw(host(peers[k][b])).tobytes() == raw(want[b]).tobytes(), ("pack", k, b)
    outs = [torch.empty_like(t) for t in peers[0]]
    plan.kt_weighted_reduce(-1, [peers[k][b] for b in range(nb) for k in range(K)], K, weights, outs)
    res = [torch.full((n,), 9.0, dtype=tdtype(dtype), device=DEV) for n in w.numels]
    plan.kt_bucket_unpack_scale(-1, outs, scale, res)
    # fused path
    res2 = [torch.full((n,), 9.0, dtype=tdtype(dtype), device=DEV) for n in w.numels]
    plan.kt_fused_step(-1, grads[0], [peers[k][b] for b in range(nb) for k in range(1, K)], K, weights, scale, res2)
    torch.cuda.synchronize()
    ref = oracle.direct(hg, wts, scale, dtype, "S")
    for t in range(len(w.numels)):
        assert raw(host(res[t])).tobytes() == raw(ref[t]).tobytes(), ("chained", t)
        assert raw(host(res2[t])).tobytes() == raw(ref[t]).tobytes(), ("fused", t)
    # SGD on unpack, two steps
    params = [torch.randn(n, device=DEV, generator=torch.Generator(DEV).manual_seed(7 + t)) for t, n in enumerate(w.numels)]
    moms = [torch.full((n,), float("nan"), device=DEV) for n in w.numels]
    hp, hv = [host(p) for p in params], [host(v) for v in moms]
    hb = [host(o) for o in outs]
    # the first step also in one pass from the local tensors and the peer buckets
    fp, fv = [p.clone() for p in params], [v.clone() for v in moms]
    plan.kt_fused_step_sgd(-1, grads[0], [peers[k][b] for b in range(nb) for k in range(1, K)], K, weights, scale,
                           fp, fv, None, 0.1, 0.9, 5e-4, True)
    for step in range(2):
        plan.kt_bucket_unpack_sgd(-1, outs, scale, params, moms, 0.1, 0.9, 5e-4, step == 0)
        torch.cuda.synchronize()
        hp, hv = oracle.unpack_sgd(L, hb, w.numels, scale, hp, hv, 0.1, 0.9, 5e-4, step == 0, dtype, "S")
        for t in range(len(w.numels)):
            assert raw(host(params[t])).tobytes() == raw(hp[t]).tobytes(), ("sgd p", step, t)
            assert raw(host(moms[t])).tobytes() == raw(hv[t]).tobytes(), ("sgd v", step, t)
            if step == 0:
                assert raw(host(fp[t])).tobytes() == raw(hp[t]).tobytes(), ("one-pass sgd p", t)
                assert raw(host(fv[t])).tobytes() == raw(hv[t]).tobytes(), ("one-pass sgd v", t)
