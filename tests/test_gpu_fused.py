"""GPU parity for the fused single pass (kt_fused_step): against the CPU
checker's un-bucketed definition g_t = scale * sum_k w_k g_t^(k), and against
the chained pack -> reduce -> unpack path on the GPU (must be bit-identical)."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2505_10183_amd as kt
from paper_2505_10183_amd import workloads as wl
from test_gpu_parity import DEV, accum_bound, assert_close, host, raw, tdtype

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def announce(request):
    print("\n[gpu-case] %s" % request.node.nodeid, file=sys.stderr, flush=True)
    yield
    torch.cuda.synchronize()


def gmax_of(hg, dtype):
    if dtype == "f32":
        return max(float(np.abs(x).max()) for g in hg for x in g if x.size)
    return max(float(np.abs(oracle.bf16_to_f32_array(x)).max()) for g in hg for x in g if x.size)


def run_case(w, align, scale, in_place=False, misalign=False, batched=True):
    K, dtype = w.K, w.dtype
    plan = kt.Plan(w.numels, dtype, w.bucket_cap_bytes, align)
    nb = plan.num_buckets
    shares, weights = kt.kt_plan_shares(w.throughputs, w.global_batch)
    wts = oracle.share_weights(oracle.plan_shares(w.throughputs, w.global_batch), w.global_batch)
    grads = [wl.gradient_set(w, k, DEV) for k in range(K)]
    if misalign:    # odd tensors of the local set start one element into an allocation
        loc = []
        for i, t in enumerate(grads[0]):
            if i % 2:
                big = torch.zeros(t.numel() + 3, dtype=t.dtype, device=DEV)
                big[1:1 + t.numel()] = t.reshape(-1)
                loc.append(big[1:1 + t.numel()])
            else:
                loc.append(t)
        grads[0] = loc
    hg = [[host(t) for t in g] for g in grads]
    # peers 1..K-1 arrive packed (by the pack kernel, checked elsewhere)
    peers = [[torch.empty(n, dtype=tdtype(dtype), device=DEV) for n in plan.bucket_elems()] for _ in range(K)]
    for k in range(K):
        plan.kt_bucket_pack(-1, grads[k], peers[k])
    flat_others = [peers[k][b] for b in range(nb) for k in range(1, K)]
    if in_place:
        stores = None
        outs = grads[0]
    else:
        stores = [torch.full((t.numel() + 16,), 5.0, dtype=t.dtype, device=DEV) for t in grads[0]]
        outs = [s[8:8 + t.numel()] for s, t in zip(stores, grads[0])]
    # chained reference on the GPU
    red = [torch.empty_like(p) for p in peers[0]]
    plan.kt_weighted_reduce(-1, [peers[k][b] for b in range(nb) for k in range(K)], K, weights, red)
    chained = [torch.empty(t.numel(), dtype=t.dtype, device=DEV) for t in grads[0]]
    plan.kt_bucket_unpack_scale(-1, red, scale, chained)
    if batched:
        plan.kt_fused_step(-1, grads[0], flat_others, K, weights, scale, outs)
    else:
        for b in range(nb):
            plan.kt_fused_step(b, grads[0], flat_others, K, weights, scale, outs)
    torch.cuda.synchronize()
    refS = oracle.direct(hg, wts, scale, dtype, "S")
    refD = oracle.direct(hg, wts, scale, dtype, "D")
    gm = gmax_of(hg, dtype) * max(abs(scale), 1.0)
    for t in range(len(w.numels)):
        got = host(outs[t])
        assert raw(got).tobytes() == raw(refS[t]).tobytes(), "tensor %d vs strict checker" % t
        assert raw(got).tobytes() == raw(host(chained[t])).tobytes(), "tensor %d vs chained path" % t
        if dtype == "f32" or scale == 1.0:
            bound = accum_bound([g[t] for g in hg], wts, dtype) if dtype == "bf16" else None
            assert_close(got, refD[t], dtype, gm, "tensor %d" % t, bound=bound)
        if stores is not None:
            s = stores[t]
            assert bool((s[:8] == 5.0).all()) and bool((s[8 + w.numels[t]:] == 5.0).all()), t


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("K", [1, 2, 3, 4, 7, 8, 9, 13, 16, 23])
def test_fused_vs_checker_and_chained(dtype, K):
    w = wl.ragged_workload(dtype=dtype, K=K, seed=60 + K)
    run_case(w, 16, 1.0)
    run_case(w, 16, 0.37, batched=False)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fused_dense_in_place_misaligned(dtype):
    w = wl.ragged_workload(dtype=dtype, K=4, seed=71)
    run_case(w, w.elem_size, 0.5)                  # dense packing: vectors straddle tensors
    run_case(w, 16, 1.0, in_place=True)            # output is the local gradient itself
    run_case(w, 16, 0.37, misalign=True)           # element-aligned local tensors
    run_case(w, 256, 1.0)                          # large alignment gaps
    run_case(w, 16384, 0.37)                       # every tensor starts on a tile boundary


def test_fused_tiny_and_many_tensors():
    numels = [1, 3, 5, 7, 2, 1, 1, 6, 4, 1] * 150 + [40000] + [4] * 2000
    w = wl.Workload("tinymany", "f32", tuple((n,) for n in numels), (1.0, 0.6, 0.5), 96, 0, 1e-3, 9)
    run_case(w, 16, 0.37)
    wb = wl.Workload("tinymany16", "bf16", tuple((n,) for n in numels), (1.0, 0.6, 0.5), 96, 0, 1e-3, 9)
    run_case(wb, 16, 1.0)


@pytest.mark.parametrize("name", ["mlp", "mobilenetv2", "resnet18", "vit_b16"])
def test_fused_workloads(name):
    run_case(wl.WORKLOADS[name], 16, 1.0)


def test_store_windows_can_be_switched_off():
    """KT_STORE_WINDOW_NS=0 in the environment (read once per process) switches the store windows of
    large launches off; results are the same either way.  Runs the ViT-B/16 case, whose fused pass is
    large enough to use a window, in a child process with the variable set."""
    import os
    import subprocess
    env = dict(os.environ, KT_STORE_WINDOW_NS="0")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "gpu", "-p", "no:cacheprovider",
                        os.path.join(root, "tests", "test_gpu_fused.py"), "-k", "test_fused_workloads and vit_b16"],
                       cwd=root, env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert "1 passed" in r.stdout, r.stdout[-500:]
