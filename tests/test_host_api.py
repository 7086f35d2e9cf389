"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every declared symbol, plans shares and bucket layouts bit-identically to the
CPU checker, builds a consistent tile table, and rejects bad arguments."""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import oracle
import paper_2505_10183_amd as kt
from paper_2505_10183_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = []
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(kt_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"kt_plan_shares", "kt_bucket_pack", "kt_weighted_reduce", "kt_bucket_unpack_scale"} <= set(names)
    L = kt.binding.lib()
    for n in names:
        assert hasattr(L, n), n
    assert b"gfx950" in L.kt_version()


def test_no_checker_in_product_path():
    """The GPU package never imports or mentions the CPU checker."""
    pkg = os.path.join(ROOT, "paper_2505_10183_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, os.path.join(dirpath, f)
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2505_10183_amd" not in text and "libkt.so" not in text and "binding" not in text


thr_lists = st.lists(st.floats(min_value=1e-3, max_value=1e3, allow_nan=False), min_size=1, max_size=16)


@settings(max_examples=500, deadline=None)
@given(thr=thr_lists, B=st.integers(0, 1 << 40))
def test_shares_bit_exact_vs_checker(thr, B):
    want = oracle.plan_shares(thr, B)
    got, w = kt.kt_plan_shares(thr, B, want_weights=B > 0)
    assert got == want
    if B > 0:
        ww = oracle.share_weights(want, B)
        assert np.array(w, dtype=np.float32).tobytes() == ww.tobytes()


def test_shares_workloads_and_golden():
    for name in wl.WORKLOAD_ORDER:
        w = wl.WORKLOADS[name]
        got, wt = kt.kt_plan_shares(w.throughputs, w.global_batch)
        assert got == oracle.plan_shares(w.throughputs, w.global_batch)
        assert sum(got) == w.global_batch and abs(sum(wt) - 1.0) == 0.0
    assert kt.kt_plan_shares([1.0, 0.7], 256)[0] == [151, 105]


def test_shares_errors_leave_outputs_untouched():
    L = kt.binding.lib()
    thr = (ctypes.c_double * 2)(1.0, float("nan"))
    b = (ctypes.c_int64 * 2)(-7, -7)
    w = (ctypes.c_float * 2)(-7.0, -7.0)
    assert L.kt_plan_shares(thr, 2, 10, b, w) == 1
    assert list(b) == [-7, -7] and list(w) == [-7.0, -7.0]
    assert b"finite" in L.kt_last_error()
    good = (ctypes.c_double * 2)(1.0, 2.0)
    for args in ((None, 2, 10, b, w), (good, 0, 10, b, w), (good, 65, 10, b, w), (good, 2, -1, b, w),
                 (good, 2, (1 << 40) + 1, b, w), (good, 2, 0, b, w), (good, 2, 10, None, w)):
        assert L.kt_plan_shares(*args) == 1
        assert list(b) == [-7, -7]
    neg = (ctypes.c_double * 2)(1.0, -2.0)
    zero = (ctypes.c_double * 2)(0.0, 2.0)
    inf = (ctypes.c_double * 2)(float("inf"), 2.0)
    for t in (neg, zero, inf):
        assert L.kt_plan_shares(t, 2, 10, b, None) == 1
    assert L.kt_plan_shares(good, 2, 0, b, None) == 0 and list(b) == [0, 0]


def layout_of(plan):
    return {"tensor_bucket": [plan.tensor_info(t)[0] for t in range(plan.num_tensors)],
            "tensor_offset": [plan.tensor_info(t)[1] for t in range(plan.num_tensors)],
            "bucket_first": [plan.bucket_info(b)[1] for b in range(plan.num_buckets)],
            "bucket_count": [plan.bucket_info(b)[2] for b in range(plan.num_buckets)],
            "bucket_elems": [plan.bucket_info(b)[0] for b in range(plan.num_buckets)]}


def check_tiles(plan, numels, es):
    """Replay what a kernel workgroup assumes about its tile."""
    E = 16384 // es
    VE = 16 // es
    L = layout_of(plan)
    nb = plan.num_buckets
    tiles = [plan.tile_info(i) for i in range(plan.num_tiles)]
    # tiles enumerate every bucket in order with no gaps
    i = 0
    for b in range(nb):
        n = L["bucket_elems"][b]
        cnt = (n + E - 1) // E
        for k in range(cnt):
            tb, tk, t0, nt = tiles[i]
            i += 1
            assert (tb, tk) == (b, k)
            s, e = k * E, min((k + 1) * E, n)
            first, last = L["bucket_first"][b], L["bucket_first"][b] + L["bucket_count"][b] - 1
            assert first <= t0 <= last and t0 + max(nt, 1) - 1 <= last
            owners = [t for t in range(first, last + 1)
                      if numels[t] > 0 and L["tensor_offset"][t] < e and L["tensor_offset"][t] + numels[t] > s]
            if nt == 0:
                assert owners == [t0]
                assert L["tensor_offset"][t0] <= s and L["tensor_offset"][t0] + numels[t0] >= e
                assert (e - s) % VE == 0
            else:
                assert all(t0 <= t < t0 + nt for t in owners)
    assert i == len(tiles)


@settings(max_examples=150, deadline=None)
@given(numels=st.lists(st.one_of(st.integers(0, 40), st.integers(0, 30000)), min_size=0, max_size=30),
       dtype=st.sampled_from(["f32", "bf16"]), cap=st.sampled_from([0, 64, 4096, 65536, 200000]),
       lg=st.integers(0, 12))
def test_layout_and_tiles_vs_checker(numels, dtype, cap, lg):
    es = 4 if dtype == "f32" else 2
    align = es << lg
    plan = kt.Plan(numels, dtype, cap, align)
    assert layout_of(plan) == oracle.assign_buckets(numels, es, cap, align)
    check_tiles(plan, numels, es)
    plan.close()


def test_layout_workloads_vs_checker():
    for name in wl.WORKLOAD_ORDER:
        w = wl.WORKLOADS[name]
        for align in (16, w.elem_size, 256, 16384):
            plan = kt.Plan(w.numels, w.dtype, w.bucket_cap_bytes, align)
            assert layout_of(plan) == oracle.assign_buckets(w.numels, w.elem_size, w.bucket_cap_bytes, align)
            plan.close()
    for name in ("mlp", "resnet18", "mobilenetv2"):
        w = wl.WORKLOADS[name]
        plan = kt.Plan(w.numels, w.dtype, w.bucket_cap_bytes, 16)
        check_tiles(plan, w.numels, w.elem_size)
    r = wl.ragged_workload()
    plan = kt.Plan(r.numels, r.dtype, r.bucket_cap_bytes, 16)
    assert plan.num_buckets > 3
    check_tiles(plan, r.numels, 4)


def test_plan_argument_errors():
    for args in (([1, 2], "f32", -1, 16), ([1, -2], "f32", 0, 16), ([1], "f32", 0, 3), ([1], "f32", 0, 2),
                 ([1], "f32", 0, 32768), ([1], "bf16", 0, 1), ([1], "f32", 0, 24)):
        with pytest.raises(kt.KtError) as ei:
            kt.Plan(*args)
        assert ei.value.status_name == "KT_EINVAL"
    p = kt.Plan([], "f32", 0, 16)
    assert p.num_buckets == 0 and p.num_tensors == 0 and p.num_tiles == 0
    with pytest.raises(kt.KtError):
        p.bucket_info(0)
    with pytest.raises(kt.KtError):
        p.tensor_info(0)
    # nothing to do: returns before any GPU is touched
    p.kt_bucket_pack(-1, [], [], stream=0)
    p.kt_weighted_reduce(-1, [], 1, [1.0], [], stream=0)
    p.kt_bucket_unpack_scale(-1, [], 1.0, [], stream=0)
    L = kt.binding.lib()
    assert L.kt_plan_destroy(None) == 0
    assert L.kt_plan_num_buckets(None) == -1


def test_device_call_argument_errors_without_gpu():
    """Argument validation happens on the host before any GPU call."""
    p = kt.Plan([10, 20], "f32", 0, 16)
    cases = [
        (lambda: p.kt_bucket_pack(2, [16, 1600], [3200], stream=0), "KT_EINVAL"),
        (lambda: p.kt_bucket_pack(-1, [0, 1600], [3200], stream=0), "KT_EINVAL"),
        (lambda: p.kt_bucket_pack(-1, [16, 1600], [0], stream=0), "KT_EINVAL"),
        (lambda: p.kt_bucket_pack(-1, [18, 1600], [3200], stream=0), "KT_EALIGN"),
        (lambda: p.kt_bucket_pack(-1, [16, 1600], [3202], stream=0), "KT_EALIGN"),
        (lambda: p.kt_bucket_pack(-1, [3200, 1600], [3200], stream=0), "KT_EINVAL"),       # overlap
        (lambda: p.kt_bucket_unpack_scale(-1, [3200], 1.0, [16, 3216], stream=0), "KT_EINVAL"),
        (lambda: p.kt_weighted_reduce(-1, [4096], 0, [], [8192], stream=0), "KT_EINVAL"),
        (lambda: p.kt_weighted_reduce(-1, [4096] * 65, 65, [1.0] * 65, [8192], stream=0), "KT_EINVAL"),
        (lambda: p.kt_weighted_reduce(-1, [4096, 0], 2, [1.0, 1.0], [8192], stream=0), "KT_EINVAL"),
        (lambda: p.kt_weighted_reduce(-1, [4096, 4098], 2, [1.0, 1.0], [8192], stream=0), "KT_EALIGN"),
        (lambda: p.kt_weighted_reduce(-1, [4096, 4160], 2, [1.0, 1.0], [4100], stream=0), "KT_EINVAL"),  # partial overlap
        (lambda: p.kt_weighted_reduce(3, [4096, 4160], 2, [1.0, 1.0], [8192], stream=0), "KT_EINVAL"),
    ]
    for fn, want in cases:
        with pytest.raises(kt.KtError) as ei:
            fn()
        assert ei.value.status_name == want, str(ei.value)


def test_fused_argument_errors_without_gpu():
    p = kt.Plan([10, 20], "f32", 0, 16)
    ok_l, ok_o = [16, 1600], [32000, 48000]
    cases = [
        (lambda: p.kt_fused_step(-1, ok_l, [4096], 0, [], 1.0, ok_o, stream=0), "KT_EINVAL"),
        (lambda: p.kt_fused_step(5, ok_l, [4096], 2, [1.0, 1.0], 1.0, ok_o, stream=0), "KT_EINVAL"),
        (lambda: p.kt_fused_step(-1, [0, 1600], [4096], 2, [1.0, 1.0], 1.0, ok_o, stream=0), "KT_EINVAL"),
        (lambda: p.kt_fused_step(-1, ok_l, [0], 2, [1.0, 1.0], 1.0, ok_o, stream=0), "KT_EINVAL"),
        (lambda: p.kt_fused_step(-1, ok_l, [4098], 2, [1.0, 1.0], 1.0, ok_o, stream=0), "KT_EALIGN"),
        (lambda: p.kt_fused_step(-1, [18, 1600], [4096], 2, [1.0, 1.0], 1.0, ok_o, stream=0), "KT_EALIGN"),
        (lambda: p.kt_fused_step(-1, ok_l, [4096], 2, [1.0, 1.0], 1.0, [20, 48000], stream=0), "KT_EINVAL"),   # partial overlap with input
        (lambda: p.kt_fused_step(-1, ok_l, [4096], 2, [1.0, 1.0], 1.0, [4100, 48000], stream=0), "KT_EINVAL"),  # overlaps a peer
    ]
    for fn, want in cases:
        with pytest.raises(kt.KtError) as ei:
            fn()
        assert ei.value.status_name == want, str(ei.value)


@settings(max_examples=120, deadline=None)
@given(N=st.integers(0, 3000), thr=st.lists(st.integers(1, 100).map(lambda v: v / 100.0), min_size=1, max_size=6),
       B=st.integers(1, 300), seed=st.integers(0, 2 ** 64 - 1), epoch=st.integers(0, 1000),
       shuffle=st.booleans(), drop_last=st.booleans())
def test_sampler_bit_exact_vs_checker(N, thr, B, seed, epoch, shuffle, drop_last):
    shares, _ = kt.kt_plan_shares(thr, B, want_weights=False)
    for rank in range(len(thr)):
        want = oracle.sampler_epoch(N, B, shares, seed, epoch, rank, shuffle, drop_last)
        got = kt.kt_sampler_epoch(N, B, shares, seed, epoch, rank, shuffle, drop_last)
        assert got == want


def test_sampler_paper_setting_and_errors():
    # the paper's run: CIFAR-10 (50 000 training images), global batch 256, scores (1.0, 0.7)
    shares, _ = kt.kt_plan_shares([1.0, 0.7], 256)
    a = kt.kt_sampler_epoch(50000, 256, shares, 5, 0, 0)
    b = kt.kt_sampler_epoch(50000, 256, shares, 5, 0, 1)
    assert len(a) == 196 * 151 and len(b) == 196 * 105
    assert a == oracle.sampler_epoch(50000, 256, shares, 5, 0, 0)
    assert b == oracle.sampler_epoch(50000, 256, shares, 5, 0, 1)
    assert set(a) | set(b) == set(range(50000))
    for args in ((10, 0, [1], 0, 0, 0), (10, 4, [3, 2], 0, 0, 0), (10, 4, [3, 1], 0, 0, 2), (-1, 4, [3, 1], 0, 0, 0),
                 (10, 4, [5, -1], 0, 0, 0)):
        with pytest.raises(kt.KtError):
            kt.kt_sampler_epoch(*args)
    L = kt.binding.lib()
    sh = (ctypes.c_int64 * 2)(3, 1)
    out = (ctypes.c_int64 * 4)(-9, -9, -9, -9)
    assert L.kt_sampler_epoch(10, 4, sh, 2, 0, 0, 1, 0, 0, out, 4, None) == 1      # needs 9 entries
    assert list(out) == [-9] * 4


def test_plan_too_large_is_rejected():
    with pytest.raises(kt.KtError) as ei:
        kt.Plan([1 << 36], "f32", 0, 16)          # 2^24 tiles of 4096 elements
    assert ei.value.status_name == "KT_EUNSUPPORTED"
    p = kt.Plan([(1 << 36) - 4096], "f32", 0, 16)
    assert p.num_tiles == (1 << 24) - 1


@settings(max_examples=200, deadline=None)
@given(data=st.data(), K=st.integers(1, 12))
def test_group_weights_bit_exact_vs_checker(data, K):
    G = data.draw(st.integers(1, K))
    shares = data.draw(st.lists(st.integers(1, 5000), min_size=K, max_size=K))
    # every group non-empty: first G devices seed the groups
    group_of = list(range(G)) + [data.draw(st.integers(0, G - 1)) for _ in range(K - G)]
    w1, w2, gb = kt.kt_plan_group_weights(shares, group_of, G)
    o1, o2, ob = oracle.group_weights(shares, group_of, G)
    assert np.array(w1, np.float32).tobytes() == o1.tobytes()
    assert np.array(w2, np.float32).tobytes() == o2.tobytes()
    assert gb == ob


def test_group_weights_errors():
    for args in (([1, 2], [0, 2], 2), ([1, 2], [0, 0], 2), ([1, 2], [0, 1], 3), ([1, -2], [0, 1], 2), ([0, 0], [0, 0], 1)):
        with pytest.raises(kt.KtError):
            kt.kt_plan_group_weights(*args)


def test_unpack_sgd_argument_errors_without_gpu():
    p = kt.Plan([10, 20], "f32", 0, 16)
    ok_p, ok_v, ok_b = [16000, 32000], [48000, 64000], [4096]
    cases = [
        (lambda: p.kt_bucket_unpack_sgd(3, ok_b, 1.0, ok_p, ok_v, 0.1, 0.9, 0.0, True, stream=0), "KT_EINVAL"),
        (lambda: p.kt_bucket_unpack_sgd(-1, [0], 1.0, ok_p, ok_v, 0.1, 0.9, 0.0, True, stream=0), "KT_EINVAL"),
        (lambda: p.kt_bucket_unpack_sgd(-1, ok_b, 1.0, [0, 32000], ok_v, 0.1, 0.9, 0.0, True, stream=0), "KT_EINVAL"),
        (lambda: p.kt_bucket_unpack_sgd(-1, ok_b, 1.0, [16002, 32000], ok_v, 0.1, 0.9, 0.0, True, stream=0), "KT_EALIGN"),
        (lambda: p.kt_bucket_unpack_sgd(-1, [4098], 1.0, ok_p, ok_v, 0.1, 0.9, 0.0, True, stream=0), "KT_EALIGN"),
        (lambda: p.kt_bucket_unpack_sgd(-1, ok_b, 1.0, ok_p, [16008, 64000], 0.1, 0.9, 0.0, True, stream=0), "KT_EINVAL"),
        (lambda: p.kt_bucket_unpack_sgd(-1, ok_b, 1.0, [4100, 32000], ok_v, 0.1, 0.9, 0.0, True, stream=0), "KT_EINVAL"),
    ]
    for fn, want in cases:
        with pytest.raises(kt.KtError) as ei:
            fn()
        assert ei.value.status_name == want, str(ei.value)


@settings(max_examples=300, deadline=None)
@given(data=st.data(), K=st.integers(1, 8), B=st.integers(1, 5000),
       alpha=st.floats(min_value=0.01, max_value=1.0))
def test_replan_bit_exact_vs_checker(data, K, B, alpha):
    times = data.draw(st.lists(st.floats(min_value=1e-3, max_value=1e3), min_size=K, max_size=K))
    used = data.draw(st.lists(st.integers(0, 500), min_size=K, max_size=K))
    ema = data.draw(st.lists(st.one_of(st.just(0.0), st.floats(min_value=1e-4, max_value=10.0)), min_size=K, max_size=K))
    try:
        want_e, want_s = oracle.replan_shares(times, used, ema, alpha, B)
    except ValueError:
        with pytest.raises(kt.KtError):
            kt.kt_replan_shares(times, used, ema, alpha, B)
        return
    got_e, got_s, got_w = kt.kt_replan_shares(times, used, ema, alpha, B)
    assert got_e == want_e and got_s == want_s
    assert np.array(got_w, np.float32).tobytes() == oracle.share_weights(want_s, B).tobytes()


def test_replan_errors_leave_state_untouched():
    L = kt.binding.lib()
    t = (ctypes.c_double * 2)(1.0, float("nan"))
    u = (ctypes.c_int64 * 2)(4, 4)
    e = (ctypes.c_double * 2)(0.5, 0.5)
    b = (ctypes.c_int64 * 2)(-7, -7)
    assert L.kt_replan_shares(t, u, e, 0.5, 2, 8, b, None) == 1
    assert list(e) == [0.5, 0.5] and list(b) == [-7, -7]
    t2 = (ctypes.c_double * 2)(1.0, 1.0)
    assert L.kt_replan_shares(t2, u, e, 0.0, 2, 8, b, None) == 1
    assert L.kt_replan_shares(t2, u, e, 0.5, 2, 8, b, None) == 0 and sum(b) == 8


def test_resident_weights_argument_errors_without_gpu():
    p = kt.Plan([10, 20], "f32", 0, 16)
    L = kt.binding.lib()
    w2 = (ctypes.c_float * 2)(0.5, 0.5)
    assert L.kt_plan_set_weights(None, w2, 2, None) == 1
    assert L.kt_plan_set_weights(p._h, None, 2, None) == 1
    assert L.kt_plan_set_weights(p._h, w2, 0, None) == 1
    assert L.kt_plan_set_weights(p._h, w2, 65, None) == 1
    # device calls without weights need resident ones
    with pytest.raises(kt.KtError) as ei:
        p.kt_weighted_reduce(-1, [4096, 8192], 2, None, [16384], stream=0)
    assert ei.value.status_name == "KT_EINVAL" and "kt_plan_set_weights" in str(ei.value)
    with pytest.raises(kt.KtError) as ei:
        p.kt_fused_step(-1, [16, 1600], [4096], 2, None, 1.0, [32000, 48000], stream=0)
    assert ei.value.status_name == "KT_EINVAL"


def test_resident_sgd_scalars_argument_errors_without_gpu():
    p = kt.Plan([10, 20], "f32", 0, 16)
    L = kt.binding.lib()
    assert L.kt_plan_set_sgd(None, 1.0, 0.1, 0.9, 0.0, None) == 1
    ok_p, ok_v, ok_m, ok_b = [16000, 32000], [48000, 64000], [80000, 96000], [4096]
    # no scalars set yet: refused before anything touches the GPU, with or without the model copy
    for models in (None, ok_m):
        with pytest.raises(kt.KtError) as ei:
            p.kt_bucket_unpack_sgd_resident(-1, ok_b, ok_p, ok_v, models, False, stream=0)
        assert ei.value.status_name == "KT_EINVAL" and "kt_plan_set_sgd" in str(ei.value)
    # the pointer checks of the by-value calls apply
    with pytest.raises(kt.KtError) as ei:
        p.kt_bucket_unpack_sgd_resident(3, ok_b, ok_p, ok_v, None, False, stream=0)
    assert ei.value.status_name == "KT_EINVAL"
    with pytest.raises(kt.KtError) as ei:
        p.kt_bucket_unpack_sgd_resident(-1, ok_b, [0, 32000], ok_v, None, False, stream=0)
    assert ei.value.status_name == "KT_EINVAL"
    with pytest.raises(ValueError):
        p.kt_bucket_unpack_sgd_resident(-1, ok_b, ok_p, ok_v, ok_m[:1], False, stream=0)


def test_fused_step_sgd_argument_errors_without_gpu():
    p = kt.Plan([10, 20], "bf16", 0, 16)
    g, pa, va, ma, peer = [1600, 3200], [16000, 32000], [48000, 64000], [80000, 96000], [409600]
    w2 = [0.5, 0.5]

    def call(**kw):
        a = dict(bucket=-1, g=g, peers=peer, K=2, w=w2, pa=pa, va=va, ma=None)
        a.update(kw)
        return p.kt_fused_step_sgd(a["bucket"], a["g"], a["peers"], a["K"], a["w"], 1.0, a["pa"], a["va"], a["ma"],
                                   0.1, 0.9, 0.0, True, stream=0)

    cases = [
        (dict(bucket=3), "KT_EINVAL"),
        (dict(K=0), "KT_EINVAL"),
        (dict(K=65), "KT_EINVAL"),
        (dict(g=[0, 3200]), "KT_EINVAL"),                 # NULL gradient
        (dict(g=[1601, 3200]), "KT_EALIGN"),              # gradient not element-aligned
        (dict(pa=[16002, 32000]), "KT_EALIGN"),           # parameters not 4-byte aligned
        (dict(ma=[80001, 96000]), "KT_EALIGN"),           # model copy not 2-byte aligned
        (dict(peers=[0]), "KT_EINVAL"),                   # NULL peer
        (dict(peers=[409601]), "KT_EALIGN"),
        (dict(va=[16008, 64000]), "KT_EINVAL"),           # momentum over the parameters
        (dict(pa=[1604, 32000]), "KT_EINVAL"),            # parameters over the gradient
        (dict(ma=[16010, 96000]), "KT_EINVAL"),           # model copy over the parameters
        (dict(pa=[409604, 32000]), "KT_EINVAL"),          # parameters over a peer bucket
        (dict(w=None), "KT_EINVAL"),                      # no resident weights
    ]
    for kw, want in cases:
        with pytest.raises(kt.KtError) as ei:
            call(**kw)
        assert ei.value.status_name == want, (kw, str(ei.value))
    with pytest.raises(ValueError):
        call(ma=ma[:1])
    with pytest.raises(ValueError):
        call(peers=[409600, 819200])
    with pytest.raises(kt.KtError) as ei:                 # resident form: nothing set
        p.kt_fused_step_sgd_resident(-1, g, peer, 2, pa, va, None, False, stream=0)
    assert ei.value.status_name == "KT_EINVAL"


def test_unpack_sgd_master_argument_errors_without_gpu():
    p = kt.Plan([10, 20], "bf16", 0, 16)
    ok_p, ok_v, ok_m, ok_b = [16000, 32000], [48000, 64000], [80000, 96000], [4096]
    cases = [
        (lambda: p.kt_bucket_unpack_sgd_master(-1, ok_b, 1.0, ok_p, ok_v, [0, 96000], 0.1, 0.9, 0.0, True, stream=0), "KT_EINVAL"),
        (lambda: p.kt_bucket_unpack_sgd_master(-1, ok_b, 1.0, ok_p, ok_v, [80001, 96000], 0.1, 0.9, 0.0, True, stream=0), "KT_EALIGN"),
        (lambda: p.kt_bucket_unpack_sgd_master(-1, ok_b, 1.0, ok_p, ok_v, [16010, 96000], 0.1, 0.9, 0.0, True, stream=0), "KT_EINVAL"),   # over the master copy
        (lambda: p.kt_bucket_unpack_sgd_master(-1, ok_b, 1.0, ok_p, ok_v, [4100, 96000], 0.1, 0.9, 0.0, True, stream=0), "KT_EINVAL"),    # over the bucket
        (lambda: p.kt_bucket_unpack_sgd_master(-1, ok_b, 1.0, [16002, 32000], ok_v, ok_m, 0.1, 0.9, 0.0, True, stream=0), "KT_EALIGN"),
    ]
    for fn, want in cases:
        with pytest.raises(kt.KtError) as ei:
            fn()
        assert ei.value.status_name == want, str(ei.value)
    with pytest.raises(ValueError):
        p.kt_bucket_unpack_sgd_master(-1, ok_b, 1.0, ok_p, ok_v, ok_m[:1], 0.1, 0.9, 0.0, True, stream=0)


def test_binding_rejects_arrays_of_the_wrong_length():
    """The library copies whole pointer arrays whatever bucket is selected; the
    binding, which knows T, the bucket count and K, refuses arrays of any other
    length before an address crosses the C ABI."""
    p = kt.Plan([70000, 10, 70000], "f32", 100000, 16)
    assert p.num_buckets == 3
    t3, b3 = [4096, 8192, 12288], [1 << 20, 2 << 20, 3 << 20]
    bad = [
        lambda: p.kt_bucket_pack(1, [8192], [2 << 20], stream=0),                 # "this bucket's" tensors only
        lambda: p.kt_bucket_pack(1, t3, [2 << 20], stream=0),
        lambda: p.kt_bucket_pack(-1, t3 + [1], b3, stream=0),
        lambda: p.kt_bucket_unpack_scale(0, b3[:1], 1.0, t3, stream=0),
        lambda: p.kt_weighted_reduce(0, [1 << 20, 5 << 20], 2, [0.5, 0.5], b3, stream=0),   # needs 3 * 2 peers
        lambda: p.kt_weighted_reduce(-1, b3 + b3, 2, [0.5], b3, stream=0),
        lambda: p.kt_weighted_reduce(-1, b3 + b3, 2, [0.5, 0.5], b3[:2], stream=0),
        lambda: p.kt_fused_step(-1, t3, b3[:2], 2, [0.5, 0.5], 1.0, t3, stream=0),
        lambda: p.kt_fused_step(-1, t3[:2], b3, 2, [0.5, 0.5], 1.0, t3, stream=0),
        lambda: p.kt_fused_step_noalloc(-1, t3, b3, 2, [0.5, 0.5], 1.0, t3[:1], stream=0),
        lambda: p.kt_bucket_unpack_sgd(-1, b3, 1.0, t3, t3[:2], 0.1, 0.9, 0.0, True, stream=0),
        lambda: p.kt_bucket_unpack_sgd(-1, b3[:1], 1.0, t3, t3, 0.1, 0.9, 0.0, True, stream=0),
        lambda: p.kt_bucket_pack(-1, p.marshal(t3[:2]), p.marshal(b3), stream=0),     # pre-marshalled arrays too
    ]
    for fn in bad:
        with pytest.raises(ValueError):
            fn()


def test_noalloc_limits_and_argument_errors_without_gpu():
    """The entry point that allocates nothing rejects plans beyond its fixed
    table space, and bad arguments, on the host before any GPU call."""
    big = kt.Plan([1 << 31], "f32", 0, 16)                  # 2^19 tiles: 8 MiB of tile table
    with pytest.raises(kt.KtError) as ei:
        big.kt_fused_step_noalloc(-1, [4096], [], 1, [1.0], 1.0, [1 << 40], stream=0)
    assert ei.value.status_name == "KT_EUNSUPPORTED" and "at most" in str(ei.value)
    many = kt.Plan([4] * 40000, "f32", 0, 16)               # 80 000 pointers
    with pytest.raises(kt.KtError) as ei:
        many.kt_fused_step_noalloc(-1, [4096 + 16 * i for i in range(40000)], [], 1, [1.0], 1.0,
                                   [(1 << 30) + 16 * i for i in range(40000)], stream=0)
    assert ei.value.status_name == "KT_EUNSUPPORTED"
    p = kt.Plan([10, 20], "f32", 0, 16)
    for fn, want in ((lambda: p.kt_fused_step_noalloc(-1, [16, 1600], [4096], 0, [], 1.0, [32000, 48000], stream=0), "KT_EINVAL"),
                     (lambda: p.kt_fused_step_noalloc(-1, [16, 1600], [4098], 2, [1.0, 1.0], 1.0, [32000, 48000], stream=0), "KT_EALIGN"),
                     (lambda: p.kt_fused_step_noalloc(-1, [16, 1600], [4096], 2, [1.0, 1.0], 1.0, [4100, 48000], stream=0), "KT_EINVAL")):
        with pytest.raises(kt.KtError) as ei:
            fn()
        assert ei.value.status_name == want, str(ei.value)
    # nothing to do: returns before any GPU is touched
    kt.Plan([], "f32", 0, 16).kt_fused_step_noalloc(-1, [], [], 1, [1.0], 1.0, [], stream=0)
