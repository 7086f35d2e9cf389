"""GPU parity: the HIP path, called through the C ABI, against the CPU checker
on the same seeded inputs.  Integer / index / copy work must be bit-exact;
the fp32 reduce must satisfy |gpu - checker_D| <= 1e-6 * max|g| + 1e-9 (max
over all K peer inputs of the bucket); bf16 results must lie within one bf16
ulp of checker mode D after binary32 accumulation, i.e. within one bf16
spacing of the result plus the per-element binary32 accumulation bound
K * 2^-24 * sum_k |w_k x_k|; against checker mode S (the same binary32 steps)
the results must be bit-identical."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2505_10183_amd as kt
from paper_2505_10183_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(autouse=True)
def announce(request):
    print("\n[gpu-case] %s" % request.node.nodeid, file=sys.stderr, flush=True)
    yield
    torch.cuda.synchronize()


# ------------------------------------------------------------- helpers ----

def tdtype(dtype):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def host(t):
    return wl.to_host_array(t)


def raw(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


def accum_bound(hp, wts, dtype):
    """What the binary32 accumulation can differ from the exact sum by, per
    element: K roundings of at most half an ulp of a partial sum each, i.e.
    K * 2^-24 * sum_k |w_k x_k|."""
    acc = np.zeros(hp[0].shape, np.float64)
    for x, w in zip(hp, wts):
        xf = x if dtype == "f32" else oracle.bf16_to_f32_array(x)
        acc += np.abs(np.float64(w) * xf.astype(np.float64))
    return len(hp) * 2.0 ** -24 * acc


def bf16_ulp(r):
    """Spacing of bf16 numbers at the magnitude of r (float64 array)."""
    with np.errstate(divide="ignore"):
        ex = np.floor(np.log2(np.maximum(np.abs(r), 2.0 ** -126)))
    return np.exp2(ex - 7)


def assert_close(got, want_D, dtype, gmax, what="", bound=None):
    """fp32: |got - D| <= 1e-6 * max|g| + 1e-9.  bf16: one bf16 ulp of the result
    after binary32 accumulation, i.e. |got - D| <= ulp_bf16(D) + bound, where
    `bound` is the per-element accumulation bound (accum_bound; None for steps
    that accumulate nothing, such as the scale of unpack)."""
    if dtype == "f32":
        tol = 1e-6 * gmax + 1e-9
        err = np.abs(got.astype(np.float64) - want_D.astype(np.float64))
        bad = ~(err <= tol)
        assert not bad.any(), "%s: max err %g > tol %g at %d" % (what, np.nanmax(err), tol, int(np.argmax(bad)))
    else:
        g = oracle.bf16_to_f32_array(got).astype(np.float64)
        r = oracle.bf16_to_f32_array(want_D).astype(np.float64)
        tol = bf16_ulp(r) * (1.0 + 1e-9)
        if bound is not None:
            tol = tol + bound
        err = np.abs(g - r)
        both_nan = np.isnan(g) & np.isnan(r)
        bad = ~((err <= tol) | both_nan | (g == r))
        assert not bad.any(), "%s: err %g > tol %g at %d" % (what, err[bad][0], tol[bad][0], int(np.argmax(bad)))


def alloc_buckets(plan, dtype, fill=None):
    bufs = []
    for n in plan.bucket_elems():
        t = torch.empty(n, dtype=tdtype(dtype), device=DEV)
        if fill is not None:
            t.view(torch.int16 if dtype == "bf16" else torch.int32).fill_(fill)
        bufs.append(t)
    return bufs


def layout_for(w, align):
    return oracle.assign_buckets(w.numels, w.elem_size, w.bucket_cap_bytes, align)


def tagged_tensors(w, seed=0):
    """Raw bit-pattern tags, including NaN payloads and denormals (pack must
    copy bits, not values)."""
    rng = np.random.default_rng(seed)
    out = []
    for n in w.numels:
        if w.dtype == "f32":
            bits = rng.integers(0, 2 ** 32, size=n, dtype=np.uint64).astype(np.uint32)
            t = torch.from_numpy(bits.view(np.int32)).to(DEV).view(torch.float32)
        else:
            bits = rng.integers(0, 2 ** 16, size=n, dtype=np.uint64).astype(np.uint16)
            t = torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)
        out.append(t)
    return out


# ---------------------------------------------------------------- pack ----

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("align", [16, 0, 256])
@pytest.mark.parametrize("batched", [True, False])
def test_pack_bit_exact(dtype, align, batched):
    w = wl.ragged_workload(dtype=dtype, seed=21)
    align = align or w.elem_size
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, align)
    L = layout_for(w, align)
    tensors = tagged_tensors(w, seed=3)
    bufs = alloc_buckets(plan, dtype, fill=0x5A5A if dtype == "bf16" else 0x5A5A5A5A)
    if batched:
        plan.kt_bucket_pack(kt.binding.KT_ALL_BUCKETS, tensors, bufs)
    else:
        for b in range(plan.num_buckets):
            plan.kt_bucket_pack(b, tensors, bufs)
    torch.cuda.synchronize()
    want = oracle.pack(L, [host(t) for t in tensors], dtype)
    for b in range(plan.num_buckets):
        assert raw(host(bufs[b])).tobytes() == raw(want[b]).tobytes(), "bucket %d" % b


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pack_unpack_misaligned_pointers(dtype):
    """Tensor and bucket addresses that are only element-aligned."""
    w = wl.ragged_workload(dtype=dtype, seed=22, n_tensors=30)
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, 16)
    L = layout_for(w, 16)
    base = tagged_tensors(w, seed=4)
    # odd tensors live one element into a larger allocation
    tensors = []
    for i, t in enumerate(base):
        if i % 2:
            big = torch.zeros(t.numel() + 3, dtype=t.dtype, device=DEV)
            big[1:1 + t.numel()] = t
            tensors.append(big[1:1 + t.numel()])
        else:
            tensors.append(t)
    want = oracle.pack(L, [host(t) for t in tensors], dtype)
    for shift in (0, 1):          # aligned buckets, then buckets off by one element
        store = [torch.zeros(n + 8, dtype=tdtype(dtype), device=DEV) for n in plan.bucket_elems()]
        bufs = [s[shift:shift + n] for s, n in zip(store, plan.bucket_elems())]
        plan.kt_bucket_pack(-1, tensors, bufs)
        torch.cuda.synchronize()
        for b in range(plan.num_buckets):
            assert raw(host(bufs[b])).tobytes() == raw(want[b]).tobytes(), (shift, b)
            assert int(store[b][shift + bufs[b].numel():].view(torch.int16).abs().sum()) == 0
        # unpack with scale 1 into canary-guarded tensors (finite values only)
        fin = wl.gradient_set(w, 0, DEV)
        plan.kt_bucket_pack(-1, fin, bufs)
        outs_store = [torch.full((t.numel() + 6,), 7.0, dtype=t.dtype, device=DEV) for t in fin]
        outs = [s[(3 if i % 2 else 0):(3 if i % 2 else 0) + t.numel()] for i, (s, t) in enumerate(zip(outs_store, fin))]
        plan.kt_bucket_unpack_scale(-1, bufs, 1.0, outs)
        torch.cuda.synchronize()
        for i, (o, t, s) in enumerate(zip(outs, fin, outs_store)):
            assert torch.equal(o, t), i
            lo = 3 if i % 2 else 0
            assert bool((s[:lo] == 7.0).all()) and bool((s[lo + t.numel():] == 7.0).all()), i


def test_pack_tiny_tensors_only():
    """Every tensor is 1..7 elements: all tiles are mixed, most vectors partial."""
    numels = [1, 3, 5, 7, 2, 1, 1, 6, 4, 1] * 120
    for dtype, align in (("f32", 16), ("bf16", 16), ("f32", 4), ("bf16", 2)):
        es = 4 if dtype == "f32" else 2
        plan = kt.Plan(numels, dtype, 0, align)
        L = oracle.assign_buckets(numels, es, 0, align)
        w = wl.Workload("tiny", dtype, tuple((n,) for n in numels), (1.0,), 1, 0, 1.0, 5)
        tensors = tagged_tensors(w, seed=6)
        bufs = alloc_buckets(plan, dtype, fill=0x1111)
        plan.kt_bucket_pack(-1, tensors, bufs)
        torch.cuda.synchronize()
        want = oracle.pack(L, [host(t) for t in tensors], dtype)
        assert raw(host(bufs[0])).tobytes() == raw(want[0]).tobytes(), (dtype, align)


def test_pack_more_tensors_than_lds_table():
    """A 16 KiB tile overlapped by more than 512 tensors takes the global-table search."""
    numels = [4] * 3000 + [50000] + [3] * 100
    plan = kt.Plan(numels, "f32", 0, 16)
    L = oracle.assign_buckets(numels, 4, 0, 16)
    w = wl.Workload("many", "f32", tuple((n,) for n in numels), (1.0,), 1, 0, 1.0, 5)
    tensors = tagged_tensors(w, seed=8)
    bufs = alloc_buckets(plan, "f32", fill=0x2222)
    plan.kt_bucket_pack(-1, tensors, bufs)
    torch.cuda.synchronize()
    want = oracle.pack(L, [host(t) for t in tensors], "f32")
    assert raw(host(bufs[0])).tobytes() == raw(want[0]).tobytes()
    fin = wl.gradient_set(w, 0, DEV)
    plan.kt_bucket_pack(-1, fin, bufs)
    outs = [torch.zeros_like(t) for t in fin]
    plan.kt_bucket_unpack_scale(-1, bufs, 0.5, outs)
    torch.cuda.synchronize()
    for o, t in zip(outs, fin):
        assert torch.equal(o, t * 0.5)


# -------------------------------------------------------------- unpack ----

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("align", [16, 0])
@pytest.mark.parametrize("scale", [1.0, 0.5, 0.37])
def test_unpack_scale(dtype, align, scale):
    w = wl.ragged_workload(dtype=dtype, seed=23)
    align = align or w.elem_size
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, align)
    L = layout_for(w, align)
    nb = plan.num_buckets
    # bucket contents: seeded Gaussians, including the padding positions
    bufs = [wl.flat_normal(n, dtype, 1e-3, 100 + b, DEV) for b, n in enumerate(plan.bucket_elems())]
    stores = [torch.full((n + 16,), 3.0, dtype=tdtype(dtype), device=DEV) for n in w.numels]
    outs = [s[8:8 + n] for s, n in zip(stores, w.numels)]
    for b in range(nb):
        plan.kt_bucket_unpack_scale(b, bufs, scale, outs)
    torch.cuda.synchronize()
    hb = [host(b) for b in bufs]
    wantD = oracle.unpack_scale(L, hb, w.numels, scale, dtype, "D")
    wantS = oracle.unpack_scale(L, hb, w.numels, scale, dtype, "S")
    for t in range(len(w.numels)):
        got = host(outs[t])
        assert raw(got).tobytes() == raw(wantS[t]).tobytes(), t
        if dtype == "f32":
            assert raw(got).tobytes() == raw(wantD[t]).tobytes(), t
        else:
            assert_close(got, wantD[t], dtype, 0.0, "tensor %d" % t)
        s = stores[t]
        assert bool((s[:8] == 3.0).all()) and bool((s[8 + w.numels[t]:] == 3.0).all()), t


# -------------------------------------------------------------- reduce ----

def run_reduce(plan, peers, weights, outs=None, bucket=-1):
    nb, K = plan.num_buckets, len(peers)
    flat = [peers[k][b] for b in range(nb) for k in range(K)]
    if outs is None:
        outs = [torch.empty_like(peers[0][b]) for b in range(nb)]
    plan.kt_weighted_reduce(bucket, flat, K, list(weights), outs)
    torch.cuda.synchronize()
    return outs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 6, 7, 8, 9, 13, 16, 23])
def test_reduce_vs_checker(dtype, K):
    w = wl.ragged_workload(dtype=dtype, K=K, seed=30 + K)
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, 16)
    shares, weights = kt.kt_plan_shares(w.throughputs, w.global_batch)
    assert shares == oracle.plan_shares(w.throughputs, w.global_batch)
    wts = oracle.share_weights(shares, w.global_batch)
    assert np.array(weights, dtype=np.float32).tobytes() == wts.tobytes()
    peers = [[wl.flat_normal(n, dtype, w.sigma, 1000 * k + b, DEV) for b, n in enumerate(plan.bucket_elems())]
             for k in range(K)]
    outs = run_reduce(plan, peers, weights)
    for b in range(plan.num_buckets):
        hp = [host(peers[k][b]) for k in range(K)]
        got = host(outs[b])
        wantD = oracle.weighted_reduce(hp, wts, dtype, "D")
        wantS = oracle.weighted_reduce(hp, wts, dtype, "S")
        if dtype == "f32":
            gmax = max(float(np.abs(x).max()) for x in hp)
        else:
            gmax = max(float(np.abs(oracle.bf16_to_f32_array(x)).max()) for x in hp)
        assert_close(got, wantD, dtype, gmax, "bucket %d" % b, bound=accum_bound(hp, wts, dtype))
        assert raw(got).tobytes() == raw(wantS).tobytes(), "strict mode, bucket %d" % b


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_reduce_identical_peers_and_integers(dtype):
    name = "vit_b16" if dtype == "f32" else "decoder_1p3b"
    cfg = wl.WORKLOADS[name]
    K = cfg.K
    numels = [70001, 5, 12345]
    plan = kt.Plan(numels, dtype, 0, 16)
    shares, weights = kt.kt_plan_shares(cfg.throughputs, cfg.global_batch)
    n = plan.bucket_elems()[0]
    x = wl.flat_normal(n, dtype, cfg.sigma, 77, DEV)
    outs = run_reduce(plan, [[x]] * K, weights)
    if dtype == "bf16":
        # 8-bit significands times <= 12-bit shares: no product or sum rounds
        assert torch.equal(outs[0], x)
    else:
        gmax = float(x.abs().max())
        assert_close(host(outs[0]), host(x), dtype, gmax, "identical peers")
    # integer-valued gradients, all-ones weights: exact integer sums
    # (bf16 holds integers exactly only up to 256: keep |sum| <= 8 * 16)
    lim = 64 if dtype == "f32" else 16
    ints = [torch.randint(-lim, lim + 1, (n,), device=DEV, generator=torch.Generator(DEV).manual_seed(k)).to(tdtype(dtype))
            for k in range(K)]
    outs = run_reduce(plan, [[t] for t in ints], [1.0] * K)
    ref = sum(t.to(torch.int64) for t in ints)
    assert torch.equal(outs[0].to(torch.int64), ref)
    if dtype == "f32":
        # w = b_k / B with B a power of two: exactly (sum_k b_k x_k) / B
        outs = run_reduce(plan, [[t] for t in ints], weights)
        num = sum(int(s) * t.to(torch.int64) for s, t in zip(shares, ints))
        assert torch.equal((outs[0].double() * cfg.global_batch).to(torch.int64), num)
    # one-hot weights select a peer bit for bit
    oh = [0.0] * K
    oh[K - 2] = 1.0
    outs = run_reduce(plan, [[t] for t in ints], oh)
    assert torch.equal(outs[0], ints[K - 2])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_reduce_in_place_and_misaligned_and_dense(dtype):
    K = 4
    es = 4 if dtype == "f32" else 2
    numels = [33001, 7, 1, 40005]
    wts = oracle.share_weights([91, 73, 46, 46], 256)
    for align in (16, es):
        plan = kt.Plan(numels, dtype, 0, align)
        n = plan.bucket_elems()[0]
        if align == es:
            assert n % (16 // es) != 0          # ragged tail shorter than a vector
        for shift in (0, 1):                    # 16-byte aligned, then element-aligned only
            store = [wl.flat_normal(n + 8, dtype, 1e-3, 50 + k, DEV) for k in range(K)]
            peers = [[s[shift:shift + n]] for s in store]
            hp = [host(p[0]) for p in peers]
            wantS = oracle.weighted_reduce(hp, wts, dtype, "S")
            tails = [s[shift + n:].clone() for s in store]
            # in place: the output is peer 2
            run_reduce(plan, peers, list(wts), outs=[peers[2][0]])
            assert raw(host(peers[2][0])).tobytes() == raw(wantS).tobytes(), (align, shift)
            for s, tl in zip(store, tails):
                assert torch.equal(s[shift + n:], tl)
            for k in (0, 1, 3):
                assert raw(host(peers[k][0])).tobytes() == raw(hp[k]).tobytes()


def test_reduce_single_bucket_selection():
    w = wl.ragged_workload(dtype="f32", K=3, seed=41)
    plan = kt.Plan(w.numels, "f32", w.bucket_cap_bytes, 16)
    nb = plan.num_buckets
    wts = [0.5, 0.25, 0.25]
    peers = [[wl.flat_normal(n, "f32", 1e-3, 10 * k + b, DEV) for b, n in enumerate(plan.bucket_elems())] for k in range(3)]
    outs = [torch.full((n,), 9.0, device=DEV) for n in plan.bucket_elems()]
    run_reduce(plan, peers, wts, outs=outs, bucket=nb - 2)
    for b in range(nb):
        if b == nb - 2:
            want = oracle.weighted_reduce([host(peers[k][b]) for k in range(3)], np.array(wts, np.float32), "f32", "S")
            assert raw(host(outs[b])).tobytes() == raw(want).tobytes()
        else:
            assert bool((outs[b] == 9.0).all())


def test_special_values():
    """NaN / Inf / zero weights follow IEEE: 0 * Inf = NaN propagates."""
    plan = kt.Plan([16], "f32", 0, 16)
    a = torch.tensor([1.0, float("inf"), float("-inf"), float("nan"), 0.0, -0.0, 1e-45, 3e38] * 2, device=DEV)
    b = torch.tensor([2.0, 1.0, float("inf"), 1.0, -0.0, -0.0, 1e-45, 3e38] * 2, device=DEV)
    for wts in ([0.5, 0.5], [0.0, 1.0], [1.0, 1.0]):
        outs = run_reduce(plan, [[a], [b]], wts)
        want = oracle.weighted_reduce([host(a), host(b)], np.array(wts, np.float32), "f32", "S")
        got = host(outs[0])
        same = (raw(got) == raw(want)) | (np.isnan(got) & np.isnan(want))
        assert same.all(), wts
    planb = kt.Plan([16], "bf16", 0, 16)
    ab, bb = a.to(torch.bfloat16), b.to(torch.bfloat16)
    outs = run_reduce(planb, [[ab], [bb]], [0.5, 0.5])
    want = oracle.weighted_reduce([host(ab), host(bb)], np.array([0.5, 0.5], np.float32), "bf16", "S")
    got = host(outs[0])
    gotf, wantf = oracle.bf16_to_f32_array(got), oracle.bf16_to_f32_array(want)
    assert ((got == want) | (np.isnan(gotf) & np.isnan(wantf))).all()


# ---------------------------------------------------------- end to end ----

def full_step_check(name, align=16, scale=1.0):
    """pack (K times) -> reduce -> unpack on a whole workload, every element
    against the checker, bucketed and un-bucketed."""
    w = wl.WORKLOADS[name]
    K, dtype = w.K, w.dtype
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, align)
    L = layout_for(w, align)
    shares, weights = kt.kt_plan_shares(w.throughputs, w.global_batch)
    assert shares == oracle.plan_shares(w.throughputs, w.global_batch)
    wts = oracle.share_weights(shares, w.global_batch)
    grads = [wl.gradient_set(w, k, DEV) for k in range(K)]
    peers = [alloc_buckets(plan, dtype, fill=0x7F7F if dtype == "bf16" else 0x7F7F7F7F) for _ in range(K)]
    for k in range(K):
        plan.kt_bucket_pack(-1, grads[k], peers[k])
    outs = run_reduce(plan, peers, weights)
    result = [torch.empty_like(t) for t in grads[0]]
    plan.kt_bucket_unpack_scale(-1, outs, scale, result)
    torch.cuda.synchronize()
    hg = [[host(t) for t in g] for g in grads]
    for k in range(K):
        want = oracle.pack(L, hg[k], dtype)
        for b in range(plan.num_buckets):
            assert raw(host(peers[k][b])).tobytes() == raw(want[b]).tobytes(), (k, b)
    refD = oracle.direct(hg, wts, scale, dtype, "D")
    refS = oracle.direct(hg, wts, scale, dtype, "S")
    if dtype == "f32":
        gmax = max(float(np.abs(x).max()) for g in hg for x in g if x.size)
    else:
        gmax = max(float(np.abs(oracle.bf16_to_f32_array(x)).max()) for g in hg for x in g if x.size)
    for t in range(len(w.numels)):
        got = host(result[t])
        assert_close(got, refD[t], dtype, gmax * abs(scale), "%s tensor %d" % (name, t))
        assert raw(got).tobytes() == raw(refS[t]).tobytes(), "%s tensor %d strict" % (name, t)


@pytest.mark.parametrize("name", ["mlp", "resnet18", "mobilenetv2"])
def test_full_step_small_workloads(name):
    full_step_check(name)
    full_step_check(name, align=wl.WORKLOADS[name].elem_size, scale=0.37)
    full_step_check(name, align=16384, scale=0.5)       # every tensor starts on a tile boundary


def test_full_step_vit_b16():
    full_step_check("vit_b16")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_two_level_reduce_with_pinned_host_inputs(dtype):
    """Two groups of four devices: level 1 on the device, level 2 reads the
    other group's result from pinned host memory (the stand-in for the host
    relay between groups)."""
    cfg = wl.WORKLOADS["vit_b16"]
    K, G = 8, 2
    group_of = [0, 0, 0, 0, 1, 1, 1, 1]
    w = wl.ragged_workload(dtype=dtype, K=K, seed=88)
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, 16)
    nb = plan.num_buckets
    shares, flat_w = kt.kt_plan_shares(cfg.throughputs, cfg.global_batch)
    w1, w2, gb = kt.kt_plan_group_weights(shares, group_of, G)
    o1, o2, ob = oracle.group_weights(shares, group_of, G)
    assert np.array(w1, np.float32).tobytes() == o1.tobytes() and np.array(w2, np.float32).tobytes() == o2.tobytes()
    peers = [[wl.flat_normal(n, dtype, 1e-3, 300 * k + b, DEV) for b, n in enumerate(plan.bucket_elems())] for k in range(K)]
    # level 1, group 0 (this device's group) and group 1 (computed here too, then "sent" to pinned host memory)
    ys = []
    for g in range(G):
        idx = [k for k in range(K) if group_of[k] == g]
        outs = [torch.empty_like(peers[0][b]) for b in range(nb)]
        plan.kt_weighted_reduce(-1, [peers[k][b] for b in range(nb) for k in idx], len(idx), [w1[k] for k in idx], outs)
        ys.append(outs)
    torch.cuda.synchronize()
    remote = [torch.empty(y.shape, dtype=y.dtype, pin_memory=True).copy_(y) for y in ys[1]]
    torch.cuda.synchronize()
    final = [torch.empty_like(peers[0][b]) for b in range(nb)]
    plan.kt_weighted_reduce(-1, [t for b in range(nb) for t in (ys[0][b], remote[b])], G, w2, final)
    torch.cuda.synchronize()
    flat = oracle.share_weights(shares, cfg.global_batch)
    for b in range(nb):
        hp = [host(peers[k][b]) for k in range(K)]
        want = oracle.two_level_reduce(hp, shares, group_of, G, dtype, "S")
        got = host(final[b])
        assert raw(got).tobytes() == raw(want).tobytes(), b
        if dtype == "f32":   # and it agrees with the flat combination within the fp32 bound
            gmax = max(float(np.abs(x).max()) for x in hp)
            assert_close(got, oracle.weighted_reduce(hp, flat, dtype, "D"), dtype, gmax, "flat, bucket %d" % b)


def test_pointer_churn_and_streams():
    """More distinct pointer sets than the library keeps resident (tables are
    evicted and re-uploaded while earlier launches may still run), on two
    streams, with results checked for every call."""
    w = wl.ragged_workload(dtype="f32", K=2, seed=55, n_tensors=30)
    plan = kt.Plan(w.numels, "f32", w.bucket_cap_bytes, 16)
    nb = plan.num_buckets
    wts = np.array([0.75, 0.25], np.float32)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    rounds = []
    for r in range(40):
        st = streams[r % 2]
        with torch.cuda.stream(st):
            peers = [[wl.flat_normal(n, "f32", 1e-3, 5000 + 100 * r + 10 * k + b, DEV)
                      for b, n in enumerate(plan.bucket_elems())] for k in range(2)]
            outs = [torch.empty_like(peers[0][b]) for b in range(nb)]
            plan.kt_weighted_reduce(-1, [peers[k][b] for b in range(nb) for k in range(2)], 2, list(wts), outs, stream=st)
        rounds.append((peers, outs))
    torch.cuda.synchronize()
    for r, (peers, outs) in enumerate(rounds):
        for b in (0, nb - 1):
            want = oracle.weighted_reduce([host(peers[k][b]) for k in range(2)], wts, "f32", "S")
            assert raw(host(outs[b])).tobytes() == raw(want).tobytes(), (r, b)
    # the same table used from two streams, then evicted
    peers, outs = rounds[-1]
    flat = [peers[k][b] for b in range(nb) for k in range(2)]
    for st in streams:
        plan.kt_weighted_reduce(-1, flat, 2, list(wts), outs, stream=st)
    for r in range(10):
        p2 = [[torch.full_like(t, float(r)) for t in pk] for pk in peers]
        o2 = [torch.empty_like(t) for t in outs]
        plan.kt_weighted_reduce(-1, [p2[k][b] for b in range(nb) for k in range(2)], 2, list(wts), o2)
        torch.cuda.synchronize()
        assert all(bool((t == float(r)).all()) for t in o2)


@pytest.mark.parametrize("dtype,K", [("f32", 5), ("bf16", 4)])
def test_reduce_large_launch_with_store_windows(dtype, K):
    """A launch large enough (65 536 tiles, K >= 4) for the reduce to hold its stores back until the
    chip-wide store window: every element of every bucket against the checker's strict mode, in place
    and into separate outputs."""
    w = wl.get("sized_%s_65536" % dtype)
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, 16)
    nb, elems = plan.num_buckets, plan.bucket_elems()
    assert plan.num_tiles >= 65536
    thr = w.throughputs[:K]
    shares, weights = kt.kt_plan_shares(thr, 1024)
    wts = oracle.share_weights(oracle.plan_shares(thr, 1024), 1024)
    peers = [[wl.flat_normal(n, dtype, 1e-3, 3000 + 50 * k + b, DEV) for b, n in enumerate(elems)] for k in range(K)]
    hp0 = [host(peers[0][b]) for b in range(nb)]
    outs = [torch.empty_like(t) for t in peers[0]]
    flat = [peers[k][b] for b in range(nb) for k in range(K)]
    plan.kt_weighted_reduce(-1, flat, K, weights, outs)
    plan.kt_weighted_reduce(-1, flat, K, weights, peers[0])          # in place over peer 0
    torch.cuda.synchronize()
    for b in range(nb):
        want = oracle.weighted_reduce([hp0[b]] + [host(peers[k][b]) for k in range(1, K)], wts, dtype, "S")
        assert raw(host(outs[b])).tobytes() == raw(want).tobytes(), ("own output", b)
        assert raw(host(peers[0][b])).tobytes() == raw(want).tobytes(), ("in place", b)


def test_two_host_threads_share_a_plan():
    """Two host threads, each with a stream of its own, call into one plan at
    the same time with pointer sets of their own (the library serialises calls
    on a plan; tables are evicted under both threads); every result is checked."""
    import threading
    w = wl.ragged_workload(dtype="bf16", K=3, seed=56, n_tensors=30)
    plan = kt.Plan(w.numels, "bf16", w.bucket_cap_bytes, 16)
    nb = plan.num_buckets
    wts = np.array([0.5, 0.25, 0.25], np.float32)
    grads = [wl.gradient_set(w, k, DEV) for k in range(3)]
    plan.kt_bucket_pack(-1, grads[0], [torch.empty(n, dtype=torch.bfloat16, device=DEV) for n in plan.bucket_elems()])
    torch.cuda.synchronize()
    results, errors = {}, []

    def worker(tid):
        try:
            torch.cuda.set_device(0)
            st = torch.cuda.Stream()
            mine = []
            for r in range(25):
                with torch.cuda.stream(st):
                    peers = [[wl.flat_normal(n, "bf16", 1e-3, 9000 + 1000 * tid + 30 * r + 10 * k + b, DEV)
                              for b, n in enumerate(plan.bucket_elems())] for k in range(3)]
                    outs = [torch.empty_like(t) for t in peers[0]]
                    res = [torch.empty_like(t) for t in grads[0]]
                    plan.kt_weighted_reduce(-1, [peers[k][b] for b in range(nb) for k in range(3)], 3, list(wts), outs,
                                            stream=st)
                    plan.kt_bucket_unpack_scale(-1, outs, 0.5, res, stream=st)
                mine.append((peers, outs, res))
            st.synchronize()
            results[tid] = mine
        except Exception as exc:          # noqa: BLE001
            errors.append((tid, repr(exc)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    L = oracle.assign_buckets(w.numels, 2, w.bucket_cap_bytes, 16)
    for tid in range(2):
        for r, (peers, outs, res) in enumerate(results[tid]):
            if r % 6:
                continue
            hb = [oracle.weighted_reduce([host(peers[k][b]) for k in range(3)], wts, "bf16", "S") for b in range(nb)]
            for b in range(nb):
                assert host(outs[b]).tobytes() == hb[b].tobytes(), (tid, r, b)
            want = oracle.unpack_scale(L, hb, w.numels, 0.5, "bf16", "S")
            for t in range(len(w.numels)):
                assert host(res[t]).tobytes() == want[t].tobytes(), (tid, r, t)


def test_edge_shapes():
    """Zero-size tensors, a one-element plan, a bucket of exactly one tile, the
    maximum peer count, and an empty plan."""
    # zero-size tensors between real ones (their pointers may be NULL)
    numels = [0, 5, 0, 0, 4096, 0, 3, 0]
    plan = kt.Plan(numels, "f32", 0, 16)
    L = oracle.assign_buckets(numels, 4, 0, 16)
    assert [plan.tensor_info(t) for t in range(8)] == list(zip(L["tensor_bucket"], L["tensor_offset"]))
    tensors = [torch.randn(n, device=DEV) if n else None for n in numels]
    bufs = alloc_buckets(plan, "f32", fill=0x33333333)
    plan.kt_bucket_pack(-1, tensors, bufs)
    torch.cuda.synchronize()
    want = oracle.pack(L, [host(t) if t is not None else np.zeros(0, np.float32) for t in tensors], "f32")
    assert raw(host(bufs[0])).tobytes() == raw(want[0]).tobytes()
    outs = [torch.zeros(n, device=DEV) if n else None for n in numels]
    plan.kt_bucket_unpack_scale(-1, bufs, 2.0, outs)
    plan.kt_fused_step(-1, tensors, [], 1, [1.0], 2.0, [torch.zeros(n, device=DEV) if n else None for n in numels])
    torch.cuda.synchronize()
    for t, o in zip(tensors, outs):
        if t is not None:
            assert torch.equal(o, t * 2.0)
    # one element
    p1 = kt.Plan([1], "bf16", 0, 16)
    assert p1.bucket_elems() == [8]
    x = torch.tensor([1.5], dtype=torch.bfloat16, device=DEV)
    b1 = alloc_buckets(p1, "bf16", fill=0x4444)
    p1.kt_bucket_pack(0, [x], b1)
    o1 = [torch.empty(8, dtype=torch.bfloat16, device=DEV)]
    p1.kt_weighted_reduce(0, [b1[0], b1[0]], 2, [0.5, 0.25], o1)
    r1 = [torch.zeros(1, dtype=torch.bfloat16, device=DEV)]
    p1.kt_bucket_unpack_scale(0, o1, 2.0, r1)
    torch.cuda.synchronize()
    assert float(b1[0][0]) == 1.5 and bool((b1[0][1:] == 0).all()) and float(r1[0][0]) == 2.25
    # exactly one full tile, then one element more
    for n in (4096, 4097):
        pt = kt.Plan([n], "f32", 0, 16)
        assert pt.num_tiles == (1 if n == 4096 else 2)
        xs = [torch.randn(pt.bucket_elems()[0], device=DEV) for _ in range(3)]
        o = [torch.empty_like(xs[0])]
        pt.kt_weighted_reduce(-1, xs, 3, [0.5, 0.25, 0.25], o)
        torch.cuda.synchronize()
        wantS = oracle.weighted_reduce([host(t) for t in xs], np.array([0.5, 0.25, 0.25], np.float32), "f32", "S")
        assert raw(host(o[0])).tobytes() == raw(wantS).tobytes()
    # the maximum number of peers
    K = kt.binding.KT_MAX_PEERS
    pk = kt.Plan([5000, 3], "bf16", 0, 16)
    n = pk.bucket_elems()[0]
    xs = [wl.flat_normal(n, "bf16", 1e-3, 40 + k, DEV) for k in range(K)]
    wts = np.full(K, 1.0 / K, np.float32)
    o = [torch.empty_like(xs[0])]
    pk.kt_weighted_reduce(-1, xs, K, list(wts), o)
    loc = [xs[0][:5000].clone(), xs[0][5000:5003].clone()]
    res = [torch.empty_like(t) for t in loc]
    pk.kt_fused_step(-1, loc, xs[1:], K, list(wts), 1.0, res)
    torch.cuda.synchronize()
    wantS = oracle.weighted_reduce([host(t) for t in xs], wts, "bf16", "S")
    assert host(o[0]).tobytes() == wantS.tobytes()
    assert host(res[0]).tobytes() == wantS[:5000].tobytes() and host(res[1]).tobytes() == wantS[5000:5003].tobytes()
    # nothing to do
    pe = kt.Plan([], "f32", 0, 16)
    pe.kt_bucket_pack(-1, [], [])
    pz = kt.Plan([0, 0], "f32", 0, 16)
    assert pz.num_buckets == 1 and pz.bucket_elems() == [0] and pz.num_tiles == 0
    pz.kt_bucket_pack(-1, [None, None], [None])
    pz.kt_weighted_reduce(-1, [None], 1, [1.0], [None])
