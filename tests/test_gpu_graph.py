"""The device calls recorded into a HIP graph (through torch.cuda.CUDAGraph) and
replayed: every replay, with changed inputs and eager work in between, must
equal the CPU checker; calls whose tables are not resident must refuse to be
captured."""
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


@pytest.mark.parametrize("name", ["mobilenetv2", "mlp"])
def test_graph_replays_match_checker(name):
    w = wl.WORKLOADS[name]
    K, dtype = w.K, w.dtype
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, 16)
    nb = plan.num_buckets
    shares, weights = kt.kt_plan_shares(w.throughputs, w.global_batch)
    wts = oracle.share_weights(oracle.plan_shares(w.throughputs, w.global_batch), w.global_batch)
    grads = [wl.gradient_set(w, k, DEV) for k in range(K)]
    peers = [[torch.empty(n, dtype=tdtype(dtype), device=DEV) for n in plan.bucket_elems()] for _ in range(K)]
    for k in range(1, K):
        plan.kt_bucket_pack(-1, grads[k], peers[k])
    flat = [peers[k][b] for b in range(nb) for k in range(K)]
    others = [peers[k][b] for b in range(nb) for k in range(1, K)]
    res = [torch.empty_like(t) for t in grads[0]]
    res2 = [torch.empty_like(t) for t in grads[0]]
    params = [torch.randn(t.numel(), device=DEV, generator=torch.Generator(DEV).manual_seed(3 + i))
              for i, t in enumerate(grads[0])]
    moms = [torch.zeros(t.numel(), device=DEV) for t in grads[0]]

    def step():
        plan.kt_bucket_pack(-1, grads[0], peers[0])
        plan.kt_weighted_reduce(-1, flat, K, weights, peers[0])          # in place over slot 0
        plan.kt_bucket_unpack_scale(-1, peers[0], 0.5, res)
        plan.kt_fused_step(-1, grads[0], others, K, weights, 0.5, res2)
        plan.kt_bucket_unpack_sgd(-1, peers[0], 0.5, params, moms, 0.1, 0.9, 5e-4, False)

    hp, hv = [host(p) for p in params], [host(v) for v in moms]
    L = oracle.assign_buckets(w.numels, w.elem_size, w.bucket_cap_bytes, 16)

    def check(tag):
        nonlocal hp, hv
        hg = [[host(t) for t in g] for g in grads]
        ref = oracle.direct(hg, wts, 0.5, dtype, "S")
        for t in range(len(w.numels)):
            assert raw(host(res[t])).tobytes() == raw(ref[t]).tobytes(), (tag, "chained", t)
            assert raw(host(res2[t])).tobytes() == raw(ref[t]).tobytes(), (tag, "fused", t)
        red = [oracle.weighted_reduce([pk[b] for pk in [oracle.pack(L, g, dtype) for g in hg]], wts, dtype, "S")
               for b in range(nb)]
        hp, hv = oracle.unpack_sgd(L, red, w.numels, 0.5, hp, hv, 0.1, 0.9, 5e-4, False, dtype, "S")
        for t in range(len(w.numels)):
            assert raw(host(params[t])).tobytes() == raw(hp[t]).tobytes(), (tag, "sgd p", t)
            assert raw(host(moms[t])).tobytes() == raw(hv[t]).tobytes(), (tag, "sgd v", t)

    step()                                  # eager: makes every table resident
    torch.cuda.synchronize()
    check("eager")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    torch.cuda.synchronize()
    for r in range(4):
        # new local gradients in the same tensors, eager library work and a sync between replays
        fresh = wl.gradient_set(w, 100 + r, DEV)
        for t, f in zip(grads[0], fresh):
            t.copy_(f)
        plan.kt_bucket_pack(-1, grads[1], peers[1])     # eager call between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        check("replay %d" % r)


def test_capture_refuses_unprepared_calls():
    plan = kt.Plan([5000, 300], "f32", 0, 16)
    a = [torch.randn(5000, device=DEV), torch.randn(300, device=DEV)]
    buf = [torch.empty(plan.bucket_elems()[0], device=DEV)]
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    err = None
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        g.capture_begin()
        try:
            plan.kt_bucket_pack(-1, a, buf)             # first use of the plan: would have to upload
        except kt.KtError as e:
            err = e
        g.capture_end()
    assert err is not None and err.status_name == "KT_EUNSUPPORTED"
    plan.kt_bucket_pack(-1, a, buf)                      # eager: fine
    torch.cuda.synchronize()
    b2 = [torch.empty(plan.bucket_elems()[0], device=DEV)]
    g2 = torch.cuda.CUDAGraph()
    err = None
    with torch.cuda.stream(s):
        g2.capture_begin()
        try:
            plan.kt_bucket_pack(-1, a, b2)              # other pointers: no resident table
        except kt.KtError as e:
            err = e
        g2.capture_end()
    assert err is not None and err.status_name == "KT_EUNSUPPORTED"
    torch.cuda.synchronize()
    plan.kt_bucket_pack(-1, a, b2)
    torch.cuda.synchronize()
    assert torch.equal(b2[0][:5000], a[0])


def test_tables_used_by_graphs_are_never_reused():
    """A plan keeps 8 pointer tables; each captured call pins one.  The ninth
    distinct pointer set can still run eagerly only if a table is free, and
    is refused with a clear error otherwise."""
    plan = kt.Plan([4096], "f32", 0, 16)
    src = [torch.randn(4096, device=DEV)]
    graphs, bufs = [], []
    for i in range(8):
        b = [torch.zeros(4096, device=DEV)]
        plan.kt_bucket_pack(-1, src, b)          # eager: table resident
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            plan.kt_bucket_pack(-1, src, b)
        graphs.append(g)
        bufs.append(b)
    extra = [torch.zeros(4096, device=DEV)]
    with pytest.raises(kt.KtError) as ei:
        plan.kt_bucket_pack(-1, src, extra)
    assert ei.value.status_name == "KT_EUNSUPPORTED"
    src[0].copy_(torch.arange(4096, device=DEV, dtype=torch.float32))
    for g in graphs:
        g.replay()
    torch.cuda.synchronize()
    for b in bufs:
        assert torch.equal(b[0], src[0])
