"""Several data-parallel steps in a row through every stage of the path, with
the shares re-planned from measured step times after each step (Sec. III-C,
phase 1 and 2): plan shares -> pack the K peers' gradients -> K-way weighted
reduce -> SGD on unpack -> re-plan.  The CPU checker runs the same loop; shares
and weights must agree exactly and parameters and momentum bit for bit after
every step (checker mode S), whichever way the step is launched: chained calls,
the fused pass followed by a separate SGD unpack, per bucket or batched, or the
one-pass call from the K gradient copies to the parameters."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2505_10183_amd as kt
from paper_2505_10183_amd import workloads as wl
from test_gpu_parity import DEV, host, raw, tdtype

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_steps_with_online_replanning(dtype):
    print("\n[gpu-case] training loop %s" % dtype, file=sys.stderr, flush=True)
    K, B, steps = 4, 256, 6
    w = wl.ragged_workload(dtype=dtype, K=K, seed=123, n_tensors=36)
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, 16)
    L = oracle.assign_buckets(w.numels, w.elem_size, w.bucket_cap_bytes, 16)
    nb, elems = plan.num_buckets, plan.bucket_elems()
    lr, mu, wd, alpha = 0.05, 0.9, 5e-4, 0.5
    # initial scores from a benchmarking run, then measured step times that drift
    shares, weights = kt.kt_plan_shares([1.0, 0.9, 0.5, 0.4], B)
    o_shares = oracle.plan_shares([1.0, 0.9, 0.5, 0.4], B)
    assert shares == o_shares
    ema, o_ema = [0.0] * K, [0.0] * K
    speed = np.array([1.0, 0.9, 0.5, 0.4])
    gen = torch.Generator(DEV).manual_seed(5)
    params = [torch.randn(n, generator=gen, device=DEV) for n in w.numels]
    moms = [torch.zeros(n, device=DEV) for n in w.numels]
    hp, hv = [host(p) for p in params], [host(v) for v in moms]
    # a second replica of the model state, advanced by the one-pass call (peer copies -> parameters)
    params1, moms1 = [p.clone() for p in params], [v.clone() for v in moms]
    slots = [[torch.empty(n, dtype=tdtype(dtype), device=DEV) for n in elems] for _ in range(K)]
    red = [torch.empty(n, dtype=tdtype(dtype), device=DEV) for n in elems]
    grad_out = [torch.empty(n, dtype=tdtype(dtype), device=DEV) for n in w.numels]
    flat = [slots[k][b] for b in range(nb) for k in range(K)]
    others = [slots[k][b] for b in range(nb) for k in range(1, K)]
    for step in range(steps):
        grads = [wl.gradient_set(wl.Workload(w.name, dtype, w.shapes, w.throughputs, B, w.bucket_cap_bytes, 1e-2,
                                             1000 * step + 7), k, DEV) for k in range(K)]
        hg = [[host(t) for t in g] for g in grads]
        wts = oracle.share_weights(o_shares, B)
        assert np.array(weights, np.float32).tobytes() == wts.tobytes()
        for k in range(K):
            plan.kt_bucket_pack(-1, grads[k], slots[k])
        if step % 2 == 0:            # chained, per bucket
            for b in range(nb):
                plan.kt_weighted_reduce(b, flat, K, weights, red)
        else:                        # batched
            plan.kt_weighted_reduce(-1, flat, K, weights, red)
        plan.kt_bucket_unpack_sgd(-1, red, 1.0, params, moms, lr, mu, wd, step == 0)
        # the fused pass gives the averaged gradient itself (what a framework would hand to its own optimizer)
        plan.kt_fused_step(-1, grads[0], others, K, weights, 1.0, grad_out)
        # ... and the one-pass form applies the update straight from the K copies
        plan.kt_fused_step_sgd(-1, grads[0], others, K, weights, 1.0, params1, moms1, None, lr, mu, wd, step == 0)
        torch.cuda.synchronize()
        packed = [oracle.pack(L, hg[k], dtype) for k in range(K)]
        reduced = [oracle.weighted_reduce([packed[k][b] for k in range(K)], wts, dtype, "S") for b in range(nb)]
        hp, hv = oracle.unpack_sgd(L, reduced, w.numels, 1.0, hp, hv, lr, mu, wd, step == 0, dtype, "S")
        want_g = oracle.unpack_scale(L, reduced, w.numels, 1.0, dtype, "S")
        for t in range(len(w.numels)):
            assert raw(host(params[t])).tobytes() == raw(hp[t]).tobytes(), ("parameters", step, t)
            assert raw(host(moms[t])).tobytes() == raw(hv[t]).tobytes(), ("momentum", step, t)
            assert raw(host(grad_out[t])).tobytes() == raw(want_g[t]).tobytes(), ("fused gradient", step, t)
            assert raw(host(params1[t])).tobytes() == raw(hp[t]).tobytes(), ("one-pass parameters", step, t)
            assert raw(host(moms1[t])).tobytes() == raw(hv[t]).tobytes(), ("one-pass momentum", step, t)
        # measured step times: samples / speed, with device 1 slowing down over time
        speed[1] *= 0.8
        times = [float(b / s) if b else 1.0 for b, s in zip(shares, speed)]
        ema, shares, weights = kt.kt_replan_shares(times, shares, ema, alpha, B)
        o_ema, o_shares = oracle.replan_shares(times, o_shares, o_ema, alpha, B)
        assert ema == o_ema and shares == o_shares and sum(shares) == B
    assert shares[1] < 70 and shares != oracle.plan_shares([1.0, 0.9, 0.5, 0.4], B)     # the plan did adapt
