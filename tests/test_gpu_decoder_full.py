"""The 1.3B-parameter bf16 gradient set at full size, every element of every
bucket against the CPU checker, in the launch configuration the benchmark
times: one batched launch per kernel over all 50 buckets, the reduce in place
over peer slot 0.

The GPU path runs once (module fixture): pack, reduce, unpack-scale; the fused
single pass; two steps of unpack fused with SGD (the second through the
mixed-precision entry, which also writes the bf16 model copy); the same two
steps through kt_fused_step_sgd (peer copies to parameters in one pass).  The checker then goes through
the workload bucket by bucket.  Its inputs are the seeded tensors and peer
buckets only: peer slot 0 is the checker's own pack of the local tensors, the
reduced bucket is the checker's own reduce, and so on down the chain; nothing
the library wrote is fed back into it.  The checker is applied to contiguous
element ranges on several host threads (every step is element-wise, so ranges
are independent); its arithmetic is the single-threaded code as it stands.

Bars: pack bit-exact; reduce, unpack, fused pass and both SGD steps (either
way) bit-identical to checker mode S; reduce and unpack also within one bf16 ulp
after binary32 accumulation of checker mode D (ulp_bf16(D) + K * 2^-24 *
sum_k |w_k x_k| per element; scale 1.0 leaves the value unchanged)."""
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
import paper_2505_10183_amd as kt
from paper_2505_10183_amd import workloads as wl
from test_gpu_parity import DEV, bf16_ulp, host

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

NAME = "decoder_1p3b"
FUSED_SCALE = 0.37
LR, MU, WD = 0.1, 0.9, 5e-4
SGD_SCALES = (1.0, 0.5)            # step 1 (first step), step 2
GROUP = 5                          # buckets per test case
NTHREADS = max(1, min(16, os.cpu_count() or 1))
_pool = ThreadPoolExecutor(NTHREADS)


def say(msg):
    print(msg, file=sys.stderr, flush=True)


def ranges(n):
    """Contiguous element ranges, one per host thread."""
    step = max(1, -(-n // NTHREADS))
    return [(lo, min(n, lo + step)) for lo in range(0, n, step)] or [(0, 0)]


def sliced(fn, n):
    """np.concatenate of fn(lo, hi) over the ranges, run on the thread pool."""
    parts = list(_pool.map(lambda r: fn(*r), ranges(n)))
    return parts[0] if len(parts) == 1 else np.concatenate(parts)


def reduce_sliced(hp, wts, mode):
    return sliced(lambda lo, hi: oracle.weighted_reduce([x[lo:hi] for x in hp], wts, "bf16", mode), hp[0].size)


def scale_sliced(x, scale, mode):
    return sliced(lambda lo, hi: oracle.scale_array(x[lo:hi], scale, "bf16", mode), x.size)


def same_bits(a, b):
    return a.shape == b.shape and np.array_equal(a.view(np.uint16 if a.dtype == np.uint16 else np.uint32),
                                                 b.view(np.uint16 if b.dtype == np.uint16 else np.uint32))


def first_diff(a, b):
    ua = a.view(np.uint16 if a.dtype == np.uint16 else np.uint32)
    ub = b.view(np.uint16 if b.dtype == np.uint16 else np.uint32)
    i = int(np.argmax(ua != ub))
    return "first difference at %d: got 0x%x want 0x%x" % (i, int(ua[i]), int(ub[i]))


def within_one_ulp_of_D(got, wantD, hp, wts, what):
    """|got - D| <= ulp_bf16(D) + K * 2^-24 * sum_k |w_k x_k|, evaluated where the two differ at all."""
    idx = np.flatnonzero(got != wantD)
    if idx.size == 0:
        return 0
    g = oracle.bf16_to_f32_array(got[idx]).astype(np.float64)
    r = oracle.bf16_to_f32_array(wantD[idx]).astype(np.float64)
    acc = np.zeros(idx.size, np.float64)
    for x, w in zip(hp, wts):
        acc += np.abs(np.float64(w) * oracle.bf16_to_f32_array(x[idx]).astype(np.float64))
    tol = bf16_ulp(r) * (1.0 + 1e-9) + len(hp) * 2.0 ** -24 * acc
    err = np.abs(g - r)
    bad = ~((err <= tol) | (np.isnan(g) & np.isnan(r)))
    assert not bad.any(), "%s: err %g > tol %g at element %d" % (what, err[bad][0], tol[bad][0], int(idx[bad][0]))
    return int(idx.size)


@pytest.fixture(scope="module")
def dec():
    w = wl.WORKLOADS[NAME]
    K, dtype = w.K, w.dtype
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, 16)
    L = oracle.assign_buckets(w.numels, w.elem_size, w.bucket_cap_bytes, 16)
    nb = plan.num_buckets
    elems = plan.bucket_elems()
    assert nb == 50 and elems == L["bucket_elems"]
    assert [plan.tensor_info(t) for t in range(len(w.numels))] == list(zip(L["tensor_bucket"], L["tensor_offset"]))
    shares, weights = kt.kt_plan_shares(w.throughputs, w.global_batch)
    assert shares == oracle.plan_shares(w.throughputs, w.global_batch) == [409, 409, 287, 287, 205, 205, 123, 123]
    wts = oracle.share_weights(shares, w.global_batch)
    assert np.array(weights, np.float32).tobytes() == wts.tobytes()
    say("[decoder] generating inputs on the device")
    # peers 1..K-1 arrive as flat buckets; peer 0 is packed from the local tensors
    peers = [None] + [[wl.flat_normal(elems[b], dtype, w.sigma, 7000 + 100 * k + b, DEV) for b in range(nb)]
                      for k in range(1, K)]
    local = wl.gradient_set(w, 0, DEV)
    slot0 = [torch.empty(n, dtype=torch.bfloat16, device=DEV) for n in elems]
    for t in slot0:
        t.view(torch.int16).fill_(0x7F7F)
    peers[0] = slot0
    say("[decoder] pack, reduce (in place over slot 0), unpack: one batched launch each")
    plan.kt_bucket_pack(-1, local, slot0)
    packed = [t.clone() for t in slot0]
    plan.kt_weighted_reduce(-1, [peers[k][b] for b in range(nb) for k in range(K)], K, weights, slot0)
    result = [torch.empty_like(t) for t in local]
    plan.kt_bucket_unpack_scale(-1, slot0, 1.0, result)
    say("[decoder] fused single pass")
    fused = [torch.empty_like(t) for t in local]
    plan.kt_fused_step(-1, local, [peers[k][b] for b in range(nb) for k in range(1, K)], K, weights, FUSED_SCALE, fused)
    say("[decoder] two steps of unpack fused with SGD")
    gen = torch.Generator(DEV).manual_seed(w.seed)
    p0 = [torch.randn(n, generator=gen, device=DEV) for n in w.numels]
    params = [t.clone() for t in p0]
    moms = [torch.full((n,), float("nan"), device=DEV) for n in w.numels]     # not to be read on the first step
    plan.kt_bucket_unpack_sgd(-1, slot0, SGD_SCALES[0], params, moms, LR, MU, WD, True)
    p1, v1 = [t.clone() for t in params], [t.clone() for t in moms]
    # the second step through the mixed-precision entry: same update, plus the bf16 model copy
    model = [torch.empty(n, dtype=torch.bfloat16, device=DEV) for n in w.numels]
    plan.kt_bucket_unpack_sgd_master(-1, slot0, SGD_SCALES[1], params, moms, model, LR, MU, WD, False)
    say("[decoder] the same two steps in one pass each, from the local tensors and the peer buckets")
    others = [peers[k][b] for b in range(nb) for k in range(1, K)]
    fp = [t.clone() for t in p0]
    fv = [torch.full((n,), float("nan"), device=DEV) for n in w.numels]
    plan.kt_fused_step_sgd(-1, local, others, K, weights, SGD_SCALES[0], fp, fv, None, LR, MU, WD, True)
    fp1, fv1 = [t.clone() for t in fp], [t.clone() for t in fv]
    fmodel = [torch.empty(n, dtype=torch.bfloat16, device=DEV) for n in w.numels]
    plan.kt_fused_step_sgd(-1, local, others, K, weights, SGD_SCALES[1], fp, fv, fmodel, LR, MU, WD, False)
    torch.cuda.synchronize()
    say("[decoder] device work done; %d host threads for the checker" % NTHREADS)
    yield dict(w=w, L=L, wts=wts, peers=peers, local=local, packed=packed, reduced=slot0, result=result, fused=fused,
               p0=p0, p1=p1, v1=v1, p2=params, v2=moms, model=model, plan=plan,
               fp1=fp1, fv1=fv1, fp2=fp, fv2=fv, fmodel=fmodel)
    torch.cuda.empty_cache()


@pytest.mark.parametrize("group", range(50 // GROUP))
def test_decoder_every_element_of_every_bucket(dec, group):
    w, L, wts = dec["w"], dec["L"], dec["wts"]
    K = w.K
    for b in range(group * GROUP, (group + 1) * GROUP):
        t_start = time.perf_counter()
        first, cnt, n = L["bucket_first"][b], L["bucket_count"][b], L["bucket_elems"][b]
        ts = range(first, first + cnt)
        numels = [w.numels[t] for t in ts]
        # the checker's layout restricted to this bucket
        sub = {"tensor_bucket": [0] * cnt, "tensor_offset": [L["tensor_offset"][t] for t in ts], "bucket_elems": [n]}
        assert all(L["tensor_bucket"][t] == b for t in ts)

        # pack: peer slot 0 as the checker builds it from the local tensors
        want0 = oracle.pack(sub, [host(dec["local"][t]) for t in ts], "bf16")[0]
        got0 = host(dec["packed"][b])
        assert same_bits(got0, want0), "pack, bucket %d: %s" % (b, first_diff(got0, want0))

        # reduce: K peer copies -> one bucket
        hp = [want0] + [host(dec["peers"][k][b]) for k in range(1, K)]
        wantS = reduce_sliced(hp, wts, "S")
        wantD = reduce_sliced(hp, wts, "D")
        got = host(dec["reduced"][b])
        assert same_bits(got, wantS), "reduce vs strict checker, bucket %d: %s" % (b, first_diff(got, wantS))
        ndiff = within_one_ulp_of_D(got, wantD, hp, wts, "reduce vs definition, bucket %d" % b)

        # unpack-scale (scale 1.0), the fused single pass, and SGD on unpack, tensor by tensor
        unpS = oracle.unpack_scale(sub, [wantS], numels, 1.0, "bf16", "S")
        unpD = oracle.unpack_scale(sub, [wantD], numels, 1.0, "bf16", "D")
        hp0 = [host(dec["p0"][t]) for t in ts]
        hv0 = [np.full(m, np.nan, np.float32) for m in numels]
        p1w, v1w = oracle.unpack_sgd(sub, [wantS], numels, SGD_SCALES[0], hp0, hv0, LR, MU, WD, True, "bf16", "S")
        p2w, v2w, m2w = oracle.unpack_sgd_master(sub, [wantS], numels, SGD_SCALES[1], p1w, v1w, LR, MU, WD, False,
                                                 "bf16", "S")
        for i, t in enumerate(ts):
            o, m = sub["tensor_offset"][i], numels[i]
            got_t = host(dec["result"][t])
            assert same_bits(got_t, unpS[i]), "unpack vs strict checker, tensor %d: %s" % (t, first_diff(got_t, unpS[i]))
            within_one_ulp_of_D(got_t, unpD[i], [x[o:o + m] for x in hp], wts, "unpack vs definition, tensor %d" % t)
            want_f = scale_sliced(wantS[o:o + m], FUSED_SCALE, "S")
            got_f = host(dec["fused"][t])
            assert same_bits(got_f, want_f), "fused pass, tensor %d: %s" % (t, first_diff(got_f, want_f))
            for what, dev_t, want_t in (("parameters after step 1", dec["p1"][t], p1w[i]),
                                        ("momentum after step 1", dec["v1"][t], v1w[i]),
                                        ("parameters after step 2", dec["p2"][t], p2w[i]),
                                        ("momentum after step 2", dec["v2"][t], v2w[i]),
                                        ("bf16 model copy after step 2", dec["model"][t], m2w[i]),
                                        ("one pass: parameters after step 1", dec["fp1"][t], p1w[i]),
                                        ("one pass: momentum after step 1", dec["fv1"][t], v1w[i]),
                                        ("one pass: parameters after step 2", dec["fp2"][t], p2w[i]),
                                        ("one pass: momentum after step 2", dec["fv2"][t], v2w[i]),
                                        ("one pass: bf16 model copy after step 2", dec["fmodel"][t], m2w[i])):
                got_s = host(dev_t)
                assert same_bits(got_s, want_t), "SGD %s, tensor %d: %s" % (what, t, first_diff(got_s, want_t))
        say("[decoder] bucket %d: %d tensors, %d elements, %d of them differ from the double-accumulated definition "
            "(all within one bf16 ulp), %.1f s" % (b, cnt, n, ndiff, time.perf_counter() - t_start))
