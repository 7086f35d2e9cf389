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


def test_tables_used_by_graphs_do_not_consume_the_eager_ring():
    """A pointer table read by a recorded call is set aside for the graph (kept
    until the plan is destroyed) and frees its place in the ring of 8 tables
    that eager calls use: after more captures than the ring has places, eager
    calls with new pointer sets keep working and every graph still replays."""
    plan = kt.Plan([4096], "f32", 0, 16)
    src = [torch.randn(4096, device=DEV)]
    graphs, bufs = [], []
    for i in range(12):
        b = [torch.zeros(4096, device=DEV)]
        plan.kt_bucket_pack(-1, src, b)          # eager: table resident
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            plan.kt_bucket_pack(-1, src, b)
        graphs.append(g)
        bufs.append(b)
    # more distinct eager pointer sets than the ring holds, interleaved with replays
    for i in range(20):
        extra = [torch.zeros(4096, device=DEV)]
        plan.kt_bucket_pack(-1, src, extra)
        graphs[i % 12].replay()
        torch.cuda.synchronize()
        assert torch.equal(extra[0], src[0])
    # an eager call with the pointers of a recorded one shares the graph's table
    plan.kt_bucket_pack(-1, src, bufs[3])
    src[0].copy_(torch.arange(4096, device=DEV, dtype=torch.float32))
    for g in graphs:
        g.replay()
    torch.cuda.synchronize()
    for b in bufs:
        assert torch.equal(b[0], src[0])


def test_recorded_weights_are_frozen_until_the_step_is_recorded_again():
    """Weights, scale and the SGD scalars travel as kernel arguments: a graph
    recorded before new shares were planned keeps applying the old weights when
    replayed; recording the step again applies the new ones.  A first SGD step
    cannot be recorded at all (it would reset the momentum on every replay)."""
    K = 3
    w = wl.ragged_workload(dtype="f32", K=K, seed=77, n_tensors=30)
    plan = kt.Plan(w.numels, "f32", w.bucket_cap_bytes, 16)
    nb = plan.num_buckets
    peers = [[wl.flat_normal(n, "f32", 1e-3, 40 * k + b, DEV) for b, n in enumerate(plan.bucket_elems())] for k in range(K)]
    flat = [peers[k][b] for b in range(nb) for k in range(K)]
    outs = [torch.empty_like(t) for t in peers[0]]
    B = 96
    shares_a, w_a = kt.kt_plan_shares([1.0, 0.5, 0.5], B)
    # online adaptation: device 0 turned out slower than planned
    _, shares_b, w_b = kt.kt_replan_shares([3.0, 1.0, 1.0], shares_a, [0.0] * K, 1.0, B)
    assert shares_b != shares_a
    hp = [[host(peers[k][b]) for k in range(K)] for b in range(nb)]

    def expect(wts):
        wv = np.array(wts, np.float32)
        return [oracle.weighted_reduce(hp[b], wv, "f32", "S") for b in range(nb)]

    def same(want):
        torch.cuda.synchronize()
        return all(raw(host(outs[b])).tobytes() == raw(want[b]).tobytes() for b in range(nb))

    plan.kt_weighted_reduce(-1, flat, K, w_a, outs)
    assert same(expect(w_a))
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        plan.kt_weighted_reduce(-1, flat, K, w_a, outs)
    for o in outs:
        o.zero_()
    g.replay()
    assert same(expect(w_a))
    # eager calls see the new weights at once ...
    plan.kt_weighted_reduce(-1, flat, K, w_b, outs)
    assert same(expect(w_b))
    # ... the old recording does not
    g.replay()
    assert same(expect(w_a)) and not same(expect(w_b))
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g2):
        plan.kt_weighted_reduce(-1, flat, K, w_b, outs)
    for o in outs:
        o.zero_()
    g2.replay()
    assert same(expect(w_b))

    # SGD: a first step is refused under capture, a later step is recorded
    params = [torch.randn(n, device=DEV) for n in w.numels]
    moms = [torch.zeros(n, device=DEV) for n in w.numels]
    plan.kt_bucket_unpack_sgd(-1, outs, 1.0, params, moms, 0.1, 0.9, 5e-4, True)
    torch.cuda.synchronize()
    g3 = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    err = None
    with torch.cuda.stream(s):
        g3.capture_begin()
        try:
            plan.kt_bucket_unpack_sgd(-1, outs, 1.0, params, moms, 0.1, 0.9, 5e-4, True)
        except kt.KtError as e:
            err = e
        plan.kt_bucket_unpack_sgd(-1, outs, 1.0, params, moms, 0.1, 0.9, 5e-4, False)
        g3.capture_end()
    assert err is not None and err.status_name == "KT_EUNSUPPORTED"
    torch.cuda.synchronize()
    hp_, hv_ = [host(p) for p in params], [host(v) for v in moms]
    L = oracle.assign_buckets(w.numels, 4, w.bucket_cap_bytes, 16)
    hb = [host(o) for o in outs]
    for r in range(2):
        g3.replay()
        torch.cuda.synchronize()
        hp_, hv_ = oracle.unpack_sgd(L, hb, w.numels, 1.0, hp_, hv_, 0.1, 0.9, 5e-4, False, "f32", "S")
        for t in range(len(w.numels)):
            assert raw(host(params[t])).tobytes() == raw(hp_[t]).tobytes(), (r, t)
            assert raw(host(moms[t])).tobytes() == raw(hv_[t]).tobytes(), (r, t)


def test_recorded_step_follows_resident_weights():
    """Calls recorded with weights=None read the plan's device-resident weights
    when they run: after new shares, kt_plan_set_weights on the replaying stream
    is enough, the graph is not recorded again.  Chained reduce and fused pass."""
    K = 4
    w = wl.ragged_workload(dtype="bf16", K=K, seed=78, n_tensors=30)
    plan = kt.Plan(w.numels, "bf16", w.bucket_cap_bytes, 16)
    nb = plan.num_buckets
    grads = [wl.gradient_set(w, k, DEV) for k in range(K)]
    peers = [[torch.empty(n, dtype=torch.bfloat16, device=DEV) for n in plan.bucket_elems()] for _ in range(K)]
    for k in range(K):
        plan.kt_bucket_pack(-1, grads[k], peers[k])
    flat = [peers[k][b] for b in range(nb) for k in range(K)]
    others = [peers[k][b] for b in range(nb) for k in range(1, K)]
    outs = [torch.empty_like(t) for t in peers[0]]
    res = [torch.empty_like(t) for t in grads[0]]
    B = 128
    shares, w_now = kt.kt_plan_shares([1.0, 0.8, 0.5, 0.5], B)
    hp = [[host(peers[k][b]) for k in range(K)] for b in range(nb)]
    hg = [[host(t) for t in g] for g in grads]

    def check(wts, tag):
        torch.cuda.synchronize()
        wv = np.array(wts, np.float32)
        for b in range(nb):
            want = oracle.weighted_reduce(hp[b], wv, "bf16", "S")
            assert host(outs[b]).tobytes() == want.tobytes(), (tag, "reduce", b)
        ref = oracle.direct(hg, wv, 0.5, "bf16", "S")
        for t in range(len(w.numels)):
            assert host(res[t]).tobytes() == ref[t].tobytes(), (tag, "fused", t)

    def step():
        plan.kt_weighted_reduce(-1, flat, K, None, outs)
        plan.kt_fused_step(-1, grads[0], others, K, None, 0.5, res)

    with pytest.raises(kt.KtError):
        step()                                    # no resident weights yet
    plan.kt_plan_set_weights(w_now)
    step()                                        # eager: tables resident, resident weights read
    check(w_now, "eager")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    ema = [0.0] * K
    speed = np.array([1.0, 0.8, 0.5, 0.5])
    for r in range(4):
        # a device slows down; re-plan; push the new weights; replay the same graph
        speed[r % K] *= 0.6
        times = [float(b / s_) for b, s_ in zip(shares, speed)]
        ema, shares, w_now = kt.kt_replan_shares(times, shares, ema, 1.0, B)
        plan.kt_plan_set_weights(w_now)
        for t in outs + res:
            t.zero_()
        g.replay()
        check(w_now, "replay %d" % r)
    # weights given by value still work beside the resident ones, and K must match them
    plan.kt_weighted_reduce(-1, flat, K, [0.25] * K, outs)
    plan.kt_fused_step(-1, grads[0], others, K, [0.25] * K, 0.5, res)
    check([0.25] * K, "by value")
    with pytest.raises(kt.KtError):
        plan.kt_weighted_reduce(-1, flat[:nb * 3], 3, None, outs)
    # the upload itself cannot be recorded
    s = torch.cuda.Stream()
    g2 = torch.cuda.CUDAGraph()
    err = None
    with torch.cuda.stream(s):
        g2.capture_begin()
        try:
            plan.kt_plan_set_weights(w_now)
        except kt.KtError as e:
            err = e
        g2.capture_end()
    assert err is not None and err.status_name == "KT_EUNSUPPORTED"



@pytest.mark.parametrize("dtype,master", [("f32", False), ("bf16", True)])
def test_recorded_sgd_step_follows_resident_scalars(dtype, master):
    """kt_bucket_unpack_sgd_resident reads scale, lr, momentum and weight decay
    from the plan's device memory when it runs: one recording follows a stepped
    learning rate (and a changed scale) pushed with kt_plan_set_sgd.  Eager
    calls equal the by-value entry points bit for bit."""
    K = 3
    w = wl.ragged_workload(dtype=dtype, K=K, seed=79, n_tensors=30)
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, 16)
    L = oracle.assign_buckets(w.numels, w.elem_size, w.bucket_cap_bytes, 16)
    bufs = [wl.flat_normal(n, dtype, 1e-2, 900 + b, DEV) for b, n in enumerate(plan.bucket_elems())]
    hb = [host(b) for b in bufs]
    T = len(w.numels)
    gen = torch.Generator(DEV).manual_seed(5)
    params = [torch.randn(n, generator=gen, device=DEV) for n in w.numels]
    moms = [torch.full((n,), float("nan"), device=DEV) for n in w.numels]
    models = [torch.zeros(n, dtype=torch.bfloat16, device=DEV) for n in w.numels] if master else None
    hp, hv = [host(p) for p in params], [host(v) for v in moms]
    hm = None

    def advance(scale, lr, first):
        nonlocal hp, hv, hm
        if master:
            hp, hv, hm = oracle.unpack_sgd_master(L, hb, w.numels, scale, hp, hv, lr, 0.9, 5e-4, first, dtype, "S")
        else:
            hp, hv = oracle.unpack_sgd(L, hb, w.numels, scale, hp, hv, lr, 0.9, 5e-4, first, dtype, "S")

    def check(tag):
        torch.cuda.synchronize()
        for t in range(T):
            assert raw(host(params[t])).tobytes() == raw(hp[t]).tobytes(), (tag, "p", t)
            assert raw(host(moms[t])).tobytes() == raw(hv[t]).tobytes(), (tag, "v", t)
            if master:
                assert host(models[t]).tobytes() == hm[t].tobytes(), (tag, "model", t)

    with pytest.raises(kt.KtError):
        plan.kt_bucket_unpack_sgd_resident(-1, bufs, params, moms, models, True)     # nothing set yet
    plan.kt_plan_set_sgd(1.0, 0.1, 0.9, 5e-4)
    plan.kt_bucket_unpack_sgd_resident(-1, bufs, params, moms, models, True)         # first step, eager
    advance(1.0, 0.1, True)
    check("first step")
    # same state through the by-value entry: bit-identical
    p2, v2 = [t.clone() for t in params], [t.clone() for t in moms]
    m2 = [torch.zeros_like(t) for t in models] if master else None
    plan.kt_bucket_unpack_sgd_resident(-1, bufs, params, moms, models, False)
    if master:
        plan.kt_bucket_unpack_sgd_master(-1, bufs, 1.0, p2, v2, m2, 0.1, 0.9, 5e-4, False)
    else:
        plan.kt_bucket_unpack_sgd(-1, bufs, 1.0, p2, v2, 0.1, 0.9, 5e-4, False)
    advance(1.0, 0.1, False)
    check("second step")
    for t in range(T):
        assert torch.equal(params[t], p2[t]) and torch.equal(moms[t], v2[t])
        if master:
            assert torch.equal(models[t], m2[t])
    # a first step cannot be recorded; later steps can
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    err = None
    with torch.cuda.stream(s):
        g.capture_begin()
        try:
            plan.kt_bucket_unpack_sgd_resident(-1, bufs, params, moms, models, True)
        except kt.KtError as e:
            err = e
        try:
            plan.kt_plan_set_sgd(1.0, 0.1, 0.9, 5e-4, stream=s)
        except kt.KtError as e:
            err2 = e
        plan.kt_bucket_unpack_sgd_resident(-1, bufs, params, moms, models, False, stream=s)
        g.capture_end()
    assert err is not None and err.status_name == "KT_EUNSUPPORTED"
    assert err2.status_name == "KT_EUNSUPPORTED"
    torch.cuda.synchronize()
    check("after capture")                       # recording ran nothing
    # a stepped learning rate, and a changed scale, with eager work and a sync between replays
    for r, (scale, lr) in enumerate([(1.0, 0.1), (1.0, 0.01), (0.5, 0.01), (0.37, 0.001), (0.37, 0.001)]):
        plan.kt_plan_set_sgd(scale, lr, 0.9, 5e-4)
        torch.cuda.synchronize()
        g.replay()
        advance(scale, lr, False)
        check("replay %d" % r)
