"""Pins for the checker's integer planning: batch shares (Sec. III-C), combine
weights, and the bucket layout.  No GPU, no GPU library."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import oracle
from paper_2505_10183_amd.workloads import WORKLOADS, WORKLOAD_ORDER

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "shares_examples.txt")


def golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            B, thr, exp, _ = [p.strip() for p in line.split(";")]
            rows.append((int(B), thr.split(), [int(x) for x in exp.split()]))
    return rows


def exact_quotas(thr_strs, B):
    """Quotas in exact rational arithmetic from the decimal literals."""
    fr = [Fraction(s) for s in thr_strs]
    S = sum(fr)
    return [x / S * B for x in fr]


def exact_shares(thr_strs, B):
    q = exact_quotas(thr_strs, B)
    fl = [x.numerator // x.denominator for x in q]
    R = B - sum(fl)
    order = sorted(range(len(q)), key=lambda i: (-(q[i] - fl[i]), i))
    for i in order[:R]:
        fl[i] += 1
    return fl


@pytest.mark.parametrize("B,thr,expected", golden_rows())
def test_shares_golden(B, thr, expected):
    assert oracle.plan_shares([float(x) for x in thr], B) == expected
    assert exact_shares(thr, B) == expected


def test_shares_workloads_sum_and_weights():
    for name in WORKLOAD_ORDER:
        w = WORKLOADS[name]
        b = oracle.plan_shares(w.throughputs, w.global_batch)
        assert sum(b) == w.global_batch
        wt = oracle.share_weights(b, w.global_batch)
        # every B here is a power of two: weights are exact and sum to 1 exactly
        assert float(np.sum(wt.astype(np.float64))) == 1.0
        s = np.float32(0)
        for x in wt:
            s = np.float32(s + x)
        assert s == np.float32(1.0)
        for bk, wk in zip(b, wt):
            assert float(wk) * w.global_batch == bk


thr_lists = st.lists(st.integers(1, 400).map(lambda v: v / 100.0), min_size=1, max_size=9)


@settings(max_examples=300, deadline=None)
@given(thr=thr_lists, B=st.integers(0, 5000))
def test_shares_invariants(thr, B):
    b = oracle.plan_shares(thr, B)
    K = len(thr)
    assert sum(b) == B and all(x >= 0 for x in b)
    strs = ["%.2f" % t for t in thr]
    q = exact_quotas(strs, B)
    for bi, qi in zip(b, q):
        assert abs(bi - qi) < 1                       # a rounding of the quota
    # doubles agree with exact rationals (when two different quotas tie exactly
    # at the cut, rounding noise may pick either: then only validity is checked)
    fl = [x.numerator // x.denominator for x in q]
    fr = sorted((x - f for x, f in zip(q, fl)), reverse=True)
    R = B - sum(fl)
    if 0 < R < K and fr[R - 1] == fr[R]:
        assert all(bi - f in (0, 1) for bi, f in zip(b, fl))
        assert all(bi - f == 1 for bi, f, x in zip(b, fl, q) if x - f > fr[R])
    else:
        assert b == exact_shares(strs, B)
    for i in range(K):                                # faster device never gets less
        for j in range(K):
            if thr[i] > thr[j]:
                assert b[i] >= b[j]
            if thr[i] == thr[j] and i < j:
                assert b[i] - b[j] in (0, 1)
    assert oracle.plan_shares([4.0 * t for t in thr], B) == b   # only ratios matter
    # when plain round-half-up of every quota already sums to B, that is the answer
    near = [int(x + Fraction(1, 2)) for x in q]
    if sum(near) == B and all((x - int(x)) != Fraction(1, 2) for x in q):
        assert near == b


def test_shares_equal_devices():
    for K in (1, 2, 3, 4, 8):
        for m in (0, 1, 5, 64):
            assert oracle.plan_shares([0.37] * K, K * m) == [m] * K


def test_shares_permutation_equivariant():
    thr = [1.0, 0.83, 0.61, 0.47, 0.29]
    B = 1000
    base = oracle.plan_shares(thr, B)
    for perm in itertools.permutations(range(5)):
        got = oracle.plan_shares([thr[p] for p in perm], B)
        assert got == [base[p] for p in perm]


def test_shares_bruteforce_minimises_deviation():
    """Among all integer vectors summing to B, the rule's answer has the
    smallest maximum and the smallest total deviation from the quotas."""
    cases = [(["1.0", "0.7"], 9), (["1.0", "0.6", "0.3"], 11),
             (["1.0", "0.8", "0.5", "0.5"], 13), (["0.9", "0.2", "0.2"], 7),
             (["1", "1", "1"], 8)]
    for strs, B in cases:
        K = len(strs)
        q = exact_quotas(strs, B)
        b = oracle.plan_shares([float(s) for s in strs], B)
        best_max = best_sum = None
        for v in itertools.product(range(B + 1), repeat=K - 1):
            last = B - sum(v)
            if last < 0:
                continue
            cand = list(v) + [last]
            dev = [abs(c - x) for c, x in zip(cand, q)]
            best_max = max(dev) if best_max is None else min(best_max, max(dev))
            best_sum = sum(dev) if best_sum is None else min(best_sum, sum(dev))
        dev = [abs(c - x) for c, x in zip(b, q)]
        assert max(dev) == best_max and sum(dev) == best_sum


def test_shares_equalise_step_time():
    """Sec. III-C: with b_i proportional to score_i the per-device step times
    b_i / thr_i become similar; the spread shrinks as B grows."""
    thr = [1.0, 1.0, 0.7, 0.7, 0.5, 0.5, 0.3, 0.3]
    prev = None
    for B in (64, 1024, 16384, 262144):
        b = oracle.plan_shares(thr, B)
        t = [bi / ti for bi, ti in zip(b, thr)]
        spread = max(t) / min(t)
        if prev is not None:
            assert spread <= prev
        prev = spread
    assert prev < 1.001


def test_shares_rejects_bad_input():
    for bad in ([], [0.0, 1.0], [-1.0], [float("nan")], [float("inf")]):
        with pytest.raises(ValueError):
            oracle.plan_shares(bad, 10)
    with pytest.raises(ValueError):
        oracle.plan_shares([1.0], -1)


def test_weights_general_B():
    b = oracle.plan_shares([1.0, 0.7, 0.4], 1000)
    w = oracle.share_weights(b, 1000)
    assert abs(float(np.sum(w.astype(np.float64))) - 1.0) <= 3 * 2.0 ** -24
    for bk, wk in zip(b, w):
        assert wk == np.float32(np.float32(bk) / np.float32(1000))


# ---------------------------------------------------------------- buckets --

def check_layout(numels, es, cap, align, L):
    A = align // es
    T = len(numels)
    assert len(L["tensor_bucket"]) == T and len(L["tensor_offset"]) == T
    nb = len(L["bucket_elems"])
    assert sum(L["bucket_count"]) == T
    t = 0
    for b in range(nb):
        assert L["bucket_first"][b] == t
        end = 0
        for j in range(L["bucket_count"][b]):
            assert L["tensor_bucket"][t] == b
            off = L["tensor_offset"][t]
            assert off % A == 0
            assert off >= end and off - end < A      # tight: only alignment gaps
            end = off + numels[t]
            t += 1
        padded = (end + A - 1) // A * A
        assert L["bucket_elems"][b] == padded
        if cap > 0 and L["bucket_count"][b] > 1:
            assert padded * es <= cap
        if cap > 0 and b + 1 < nb:
            # greedy: the next bucket's first tensor did not fit here
            nxt = numels[L["bucket_first"][b + 1]]
            assert ((padded + nxt + A - 1) // A * A) * es > cap
    if cap == 0 and T > 0:
        assert nb == 1


@settings(max_examples=200, deadline=None)
@given(numels=st.lists(st.integers(0, 3000), min_size=0, max_size=40),
       es=st.sampled_from([2, 4]), cap=st.sampled_from([0, 64, 1000, 4096, 20000]),
       lg=st.integers(0, 12))
def test_bucket_layout_invariants(numels, es, cap, lg):
    align = es << lg
    L = oracle.assign_buckets(numels, es, cap, align)
    check_layout(numels, es, cap, align, L)


def test_bucket_layout_workloads():
    expect = {"mlp": 1, "resnet18": 2, "mobilenetv2": 1, "vit_b16": 16,
              "decoder_1p3b": 50}
    for name in WORKLOAD_ORDER:
        w = WORKLOADS[name]
        L = oracle.assign_buckets(w.numels, w.elem_size, w.bucket_cap_bytes, 16)
        check_layout(w.numels, w.elem_size, w.bucket_cap_bytes, 16, L)
        assert len(L["bucket_elems"]) == expect[name]
    # the 206 MB embedding is larger than the 64 MiB cap and sits alone
    w = WORKLOADS["decoder_1p3b"]
    L = oracle.assign_buckets(w.numels, 2, w.bucket_cap_bytes, 16)
    assert L["bucket_count"][0] == 1 and L["bucket_elems"][0] == 50304 * 2048


def test_bucket_layout_hand_example():
    # fp32, 16-byte alignment (4 elements), cap 64 bytes = 16 elements
    L = oracle.assign_buckets([5, 3, 9, 1, 20, 2], 4, 64, 16)
    assert L["tensor_bucket"] == [0, 0, 1, 1, 2, 3]
    assert L["tensor_offset"] == [0, 8, 0, 12, 0, 0]
    assert L["bucket_elems"] == [12, 16, 20, 4]
    # dense packing (alignment = element size)
    L = oracle.assign_buckets([5, 3, 9, 1, 20, 2], 4, 64, 4)
    assert L["tensor_bucket"] == [0, 0, 1, 1, 2, 3]
    assert L["tensor_offset"] == [0, 5, 0, 9, 0, 0]
    assert L["bucket_elems"] == [8, 10, 20, 2]
    # alignment to 16384 bytes (the largest allowed): 4096 fp32 / 8192 bf16 elements
    L = oracle.assign_buckets([5, 4096, 3, 4097], 4, 0, 16384)
    assert L["tensor_offset"] == [0, 4096, 8192, 12288] and L["bucket_elems"] == [20480]
    L = oracle.assign_buckets([5, 9000, 3], 2, 40000, 16384)
    assert L["tensor_bucket"] == [0, 1, 2] and L["tensor_offset"] == [0, 0, 0]
    assert L["bucket_elems"] == [8192, 16384, 8192]
    with pytest.raises(ValueError):
        oracle.assign_buckets([5], 4, 0, 32768)
