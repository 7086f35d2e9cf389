"""GPU parity for kt_bucket_unpack_sgd (unpack fused with SGD momentum /
weight decay, Sec. IV-B's optimizer) against the CPU checker: bit-identical to
its binary32 step mode S, within a few binary32 roundings of its double mode D."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2505_10183_amd as kt
from paper_2505_10183_amd import workloads as wl
from test_gpu_parity import DEV, host, raw

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def announce(request):
    print("\n[gpu-case] %s" % request.node.nodeid, file=sys.stderr, flush=True)
    yield
    torch.cuda.synchronize()


def run_sgd(w, align, scale, lr, mu, wd, steps=2, misalign=False, bucket_shift=0, per_bucket=False, master=False):
    dtype = w.dtype
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, align)
    L = oracle.assign_buckets(w.numels, w.elem_size, w.bucket_cap_bytes, align)
    nb = plan.num_buckets
    gen = torch.Generator(DEV).manual_seed(w.seed)
    # parameters and momentum live inside canary-guarded allocations
    lo = [(1 if (misalign and t % 2) else 4) for t in range(len(w.numels))]
    p_store = [torch.full((n + 12,), 9.0, device=DEV) for n in w.numels]
    v_store = [torch.full((n + 12,), 9.0, device=DEV) for n in w.numels]
    params = [s[l:l + n] for s, l, n in zip(p_store, lo, w.numels)]
    moms = [s[l:l + n] for s, l, n in zip(v_store, lo, w.numels)]
    # mixed precision: the bf16 model copy, canary-guarded too (odd tensors only 2-byte aligned when misaligned)
    m_store = [torch.full((n + 12,), 9.0, dtype=torch.bfloat16, device=DEV) for n in w.numels]
    models = [s[l:l + n] for s, l, n in zip(m_store, lo, w.numels)]
    for p in params:
        p.copy_(torch.randn(p.shape, generator=gen, device=DEV))
    for v in moms:
        v.fill_(float("nan"))          # must not be read on the first step
    hp = [host(p) for p in params]
    hv = [host(v) for v in moms]
    hpD, hvD = [x.copy() for x in hp], [x.copy() for x in hv]
    for step in range(steps):
        store = [wl.flat_normal(n + 8, dtype, 1e-2, 900 + 10 * step + b, DEV) for b, n in enumerate(plan.bucket_elems())]
        bufs = [s[bucket_shift:bucket_shift + n] for s, n in zip(store, plan.bucket_elems())]
        for b in (range(nb) if per_bucket else [-1]):
            if master:
                plan.kt_bucket_unpack_sgd_master(b, bufs, scale, params, moms, models, lr, mu, wd, step == 0)
            else:
                plan.kt_bucket_unpack_sgd(b, bufs, scale, params, moms, lr, mu, wd, step == 0)
        torch.cuda.synchronize()
        hb = [host(b) for b in bufs]
        if master:
            hp, hv, hm = oracle.unpack_sgd_master(L, hb, w.numels, scale, hp, hv, lr, mu, wd, step == 0, dtype, "S")
            for t, n in enumerate(w.numels):
                assert host(models[t]).tobytes() == hm[t].tobytes(), ("model copy", step, t)
                s_, l = m_store[t], lo[t]
                assert bool((s_[:l] == 9.0).all()) and bool((s_[l + n:] == 9.0).all()), ("model canary", t)
        else:
            hp, hv = oracle.unpack_sgd(L, hb, w.numels, scale, hp, hv, lr, mu, wd, step == 0, dtype, "S")
        hpD, hvD = oracle.unpack_sgd(L, hb, w.numels, scale, hpD, hvD, lr, mu, wd, step == 0, dtype, "D")
        for t, n in enumerate(w.numels):
            gp, gv = host(params[t]), host(moms[t])
            assert raw(gp).tobytes() == raw(hp[t]).tobytes(), ("param", step, t)
            assert raw(gv).tobytes() == raw(hv[t]).tobytes(), ("momentum", step, t)
            if n:
                # against double arithmetic: three roundings in v', one more in p' (errors carried over steps)
                tv = (3 + 4 * step) * 2.0 ** -24 * (np.abs(hvD[t]).max() + 1e-2) + 1e-12
                assert np.abs(gv.astype(np.float64) - hvD[t]).max() <= tv, ("momentum D", step, t)
                tp = (1 + 2 * step) * 2.0 ** -24 * np.abs(hpD[t]).max() + lr * tv * (step + 1) + 1e-12
                assert np.abs(gp.astype(np.float64) - hpD[t]).max() <= tp, ("param D", step, t)
            for s_, l in ((p_store[t], lo[t]), (v_store[t], lo[t])):
                assert bool((s_[:l] == 9.0).all()) and bool((s_[l + n:] == 9.0).all()), ("canary", t)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sgd_ragged(dtype):
    w = wl.ragged_workload(dtype=dtype, seed=91)
    run_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4)
    run_sgd(w, 16, 0.37, 0.05, 0.9, 5e-4, per_bucket=True)
    run_sgd(w, w.elem_size, 1.0, 0.1, 0.9, 5e-4)                 # dense packing
    run_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, misalign=True)           # 4-byte aligned parameters
    run_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, bucket_shift=1)          # element-aligned buckets
    run_sgd(w, 16, 1.0, 0.1, 0.0, 0.0, steps=1)                  # plain SGD
    run_sgd(w, 16384, 0.5, 0.1, 0.9, 5e-4)                       # every tensor starts on a tile boundary


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sgd_master_ragged(dtype):
    """Mixed precision: binary32 master parameters updated, bf16 model copy written."""
    w = wl.ragged_workload(dtype=dtype, seed=92)
    run_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, master=True)
    run_sgd(w, 16, 0.37, 0.05, 0.9, 5e-4, per_bucket=True, master=True)
    run_sgd(w, w.elem_size, 1.0, 0.1, 0.9, 5e-4, master=True)               # dense packing
    run_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, misalign=True, master=True)         # 4-byte / 2-byte aligned tensors
    run_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, bucket_shift=1, master=True)        # element-aligned buckets
    run_sgd(w, 16384, 0.5, 0.1, 0.9, 5e-4, master=True)


def test_sgd_tiny_and_many_tensors():
    numels = [1, 3, 5, 7, 2, 1, 1, 6, 4, 1] * 100 + [30000] + [4] * 1500
    for dtype in ("f32", "bf16"):
        w = wl.Workload("tm", dtype, tuple((n,) for n in numels), (1.0,), 1, 0, 1e-2, 17)
        run_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4)
        run_sgd(w, 16, 1.0, 0.1, 0.9, 5e-4, master=True)


@pytest.mark.parametrize("name", ["mobilenetv2", "resnet18", "vit_b16"])
def test_sgd_workloads(name):
    run_sgd(wl.WORKLOADS[name], 16, 1.0, 0.1, 0.9, 5e-4, steps=2)
    run_sgd(wl.WORKLOADS[name], 16, 1.0, 0.1, 0.9, 5e-4, steps=2, master=True)
