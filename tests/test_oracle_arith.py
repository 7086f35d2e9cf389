"""Pins for the checker's element arithmetic: bf16 helpers, the K-way weighted
combine, the scale step, pack/unpack indexing and the bucketed == un-bucketed
identity.  Every check is against something other than the checker itself:
exact rational arithmetic, integer arithmetic, library conversions, closed
forms, brute-force Python loops.  No GPU, no GPU library."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2505_10183_amd import workloads as wl


# ------------------------------------------------------------------ bf16 --

def exact_round_to_bf16(fr: Fraction) -> int:
    """Round an exact rational to bf16 (RNE) with integer arithmetic only."""
    if fr == 0:
        return 0
    sign = 0x8000 if fr < 0 else 0
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, -126)
    q = Fraction(2) ** (e - 7)
    m = a / q
    lo = m.numerator // m.denominator
    rem = m - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    # lo is in [0, 256]; 256 means carry into the next binade
    if lo == 256:
        lo, e = 128, e + 1
    if e > 127:
        return sign | 0x7F80
    if lo < 128:                       # subnormal (e == -126)
        return sign | lo
    return sign | ((e + 127) << 7) | (lo - 128)


def test_bf16_widen_exhaustive():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.bf16_widen(int(b)) for b in bits], dtype=np.float32)
    same = (got.view(np.uint32) == ref.view(np.uint32)) | (np.isnan(got) & np.isnan(ref))
    assert same.all()
    assert (oracle.bf16_to_f32_array(bits).view(np.uint32) == (bits.astype(np.uint32) << 16)).all()


def test_bf16_round_every_bf16_value_is_fixed_point():
    for b in range(65536):
        f = oracle.bf16_widen(b)
        r = oracle.bf16_round(f)
        if np.isnan(f):
            assert (r & 0x7F80) == 0x7F80 and (r & 0x7F) != 0
        else:
            assert r == b


def test_bf16_round_against_library_and_integer_rule():
    rng = np.random.default_rng(1)
    u = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64).astype(np.uint32)
    # ties and near-ties: low 16 bits 0x8000, 0x7FFF, 0x8001 on random upper halves
    hi = (rng.integers(0, 2 ** 16, size=3000, dtype=np.uint64).astype(np.uint32)) << 16
    special = np.array([0x00000000, 0x80000000, 0x7F800000, 0xFF800000, 0x7F7FFFFF,
                        0x7F7F8000, 0x7F7F7FFF, 0x00000001, 0x00008000, 0x00008001,
                        0x00018000, 0x007FFFFF, 0x00800000, 0x3F808000, 0x3F818000,
                        0x7FC00000, 0x7F800001, 0xFFC12345], dtype=np.uint32)
    allbits = np.concatenate([u, hi | 0x8000, hi | 0x7FFF, hi | 0x8001, special])
    f = allbits.view(np.float32)
    lib = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    # second formulation: add-and-shift on the binary32 bits
    lsb = (allbits >> 16) & 1
    shifted = ((allbits.astype(np.uint64) + 0x7FFF + lsb) >> 16).astype(np.uint16)
    for i in range(allbits.size):
        x = float(f[i])
        r = oracle.bf16_round(x)
        if np.isnan(x):
            assert (r & 0x7F80) == 0x7F80 and (r & 0x7F) != 0
            continue
        assert r == int(lib[i]), hex(int(allbits[i]))
        assert r == int(shifted[i]), hex(int(allbits[i]))
        if i % 37 == 0:
            assert r == exact_round_to_bf16(Fraction(x))


def test_bf16_round_from_double_is_single_rounding():
    # 1 + 2^-8 + 2^-40 lies just above a bf16 tie: one rounding goes up, but
    # rounding to binary32 first (-> exactly the tie) and then to bf16 goes down.
    d = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert oracle.bf16_round(d) == 0x3F81
    assert oracle.bf16_round(float(np.float32(d))) == 0x3F80
    assert oracle.bf16_round(d) == exact_round_to_bf16(Fraction(d))
    rng = np.random.default_rng(5)
    for x in rng.standard_normal(500) * 10.0 ** rng.integers(-42, 39, size=500):
        assert oracle.bf16_round(float(x)) == exact_round_to_bf16(Fraction(float(x)))


# ---------------------------------------------------------------- reduce --

def frac_round_f32(fr: Fraction) -> np.float32:
    """Exact rational -> nearest binary32 (numpy rounds int/int division
    correctly through Python's exact Fraction -> float -> float32 only when no
    double rounding occurs; so do it with integers)."""
    if fr == 0:
        return np.float32(0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    e = max(e, -126)
    q = Fraction(2) ** (e - 23)
    m = a / q
    lo = m.numerator // m.denominator
    rem = m - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return np.float32(sign * float(Fraction(lo) * q))


def test_reduce_bruteforce_exact_rationals():
    rng = np.random.default_rng(0)
    for K in (1, 2, 3, 5, 8):
        n = 64
        xs = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(K)]
        b = oracle.plan_shares(list(rng.uniform(0.3, 1.0, K)), 96)   # B not a power of two
        w = oracle.share_weights(b, 96)
        outD = oracle.weighted_reduce(xs, w, "f32", "D")
        outS = oracle.weighted_reduce(xs, w, "f32", "S")
        for i in range(n):
            exact = sum(Fraction(float(w[k])) * Fraction(float(xs[k][i])) for k in range(K))
            ref = frac_round_f32(exact)
            bound = sum(abs(float(w[k]) * float(xs[k][i])) for k in range(K))
            ulp = np.spacing(np.float32(abs(ref)))
            # mode D: double accumulation then one rounding: within a hair of exact RN
            assert abs(float(outD[i]) - float(ref)) <= ulp
            assert abs(Fraction(float(outD[i])) - exact) <= Fraction(float(ulp)) * Fraction(51, 100)
            # mode S: K roundings of at most half an ulp of a partial sum each
            assert abs(float(outS[i]) - float(exact)) <= K * 2.0 ** -24 * bound + 1e-45


def test_reduce_identical_peers_returns_input():
    # sum_k b_k = B and a power-of-two B: (sum_k b_k x)/B = x exactly in mode D
    rng = np.random.default_rng(2)
    x = (rng.standard_normal(5000) * 1e-3).astype(np.float32)
    for name in ("mlp", "resnet18", "vit_b16"):
        w_ = wl.WORKLOADS[name]
        b = oracle.plan_shares(w_.throughputs, w_.global_batch)
        w = oracle.share_weights(b, w_.global_batch)
        out = oracle.weighted_reduce([x] * w_.K, w, "f32", "D")
        assert (out.view(np.uint32) == x.view(np.uint32)).all()
    # bf16 data: 8-bit significands times <=12-bit shares never round, either mode
    xb = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    w_ = wl.WORKLOADS["decoder_1p3b"]
    w = oracle.share_weights(oracle.plan_shares(w_.throughputs, w_.global_batch), w_.global_batch)
    for mode in "DS":
        out = oracle.weighted_reduce([xb] * 8, w, "bf16", mode)
        assert (out == xb).all()


def test_reduce_integer_sums_exact():
    rng = np.random.default_rng(3)
    K, n = 8, 4096
    xi = rng.integers(-64, 65, size=(K, n))
    xs = [xi[k].astype(np.float32) for k in range(K)]
    ones = np.ones(K, dtype=np.float32)
    for mode in "DS":
        out = oracle.weighted_reduce(xs, ones, "f32", mode)
        assert (out.astype(np.int64) == xi.sum(axis=0)).all()
    # w = b_k / B with B = 1024: exactly (sum_k b_k x_k) / B
    thr = wl.WORKLOADS["vit_b16"].throughputs
    b = oracle.plan_shares(thr, 1024)
    w = oracle.share_weights(b, 1024)
    num = (np.array(b)[:, None] * xi).sum(axis=0)
    for mode in "DS":
        out = oracle.weighted_reduce(xs, w, "f32", mode)
        assert (out.astype(np.float64) * 1024 == num).all()
    # a dropped or doubled term, or weights applied in the wrong order, would
    # change these sums: shares are distinct across pairs and x_k independent
    assert len(set(b)) > 1


def test_reduce_one_hot_and_copy():
    rng = np.random.default_rng(4)
    K, n = 5, 1000
    xs = [rng.standard_normal(n).astype(np.float32) for _ in range(K)]
    for j in range(K):
        w = np.zeros(K, dtype=np.float32)
        w[j] = 1.0
        for mode in "DS":
            out = oracle.weighted_reduce(xs, w, "f32", mode)
            assert (out == xs[j]).all()
    out = oracle.weighted_reduce([xs[0]], np.ones(1, np.float32), "f32", "D")
    assert (out.view(np.uint32) == xs[0].view(np.uint32)).all()


def test_reduce_mean_special_case_matches_library():
    rng = np.random.default_rng(6)
    K, n = 8, 20000
    xs = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(K)]
    w = np.full(K, 1.0 / K, dtype=np.float32)     # 0.125 exact
    ref = np.mean(np.stack(xs).astype(np.float64), axis=0)
    out = oracle.weighted_reduce(xs, w, "f32", "D")
    assert (out == ref.astype(np.float32)).all()
    tref = torch.stack([torch.from_numpy(x) for x in xs]).double().mean(0).float().numpy()
    assert (out == tref).all()
    outS = oracle.weighted_reduce(xs, w, "f32", "S")
    gmax = max(float(np.abs(x).max()) for x in xs)
    assert np.abs(outS.astype(np.float64) - ref).max() <= 1e-6 * gmax + 1e-9


def test_reduce_linearity_and_mode_gap():
    rng = np.random.default_rng(7)
    K, n = 4, 3000
    xs = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(K)]
    ys = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(K)]
    w = oracle.share_weights([91, 73, 46, 46], 256)
    a = oracle.weighted_reduce(xs, w, "f32", "D").astype(np.float64)
    b = oracle.weighted_reduce(ys, w, "f32", "D").astype(np.float64)
    c = oracle.weighted_reduce([x + y for x, y in zip(xs, ys)], w, "f32", "D").astype(np.float64)
    assert np.abs(c - (a + b)).max() <= 4e-6 * 4e-3
    s = oracle.weighted_reduce(xs, w, "f32", "S").astype(np.float64)
    gmax = max(float(np.abs(x).max()) for x in xs)
    assert np.abs(s - a).max() <= 1e-6 * gmax + 1e-9


def test_reduce_bf16_against_exact():
    rng = np.random.default_rng(8)
    K, n = 8, 300
    xs = [torch.from_numpy((rng.standard_normal(n) * 1e-4).astype(np.float32))
          .to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16) for _ in range(K)]
    w = oracle.share_weights([409, 409, 287, 287, 205, 205, 123, 123], 2048)
    outD = oracle.weighted_reduce(xs, w, "bf16", "D")
    outS = oracle.weighted_reduce(xs, w, "bf16", "S")
    for i in range(n):
        exact = sum(Fraction(float(w[k])) * Fraction(oracle.bf16_widen(int(xs[k][i])))
                    for k in range(K))
        # 12-bit shares x 8-bit significands: all partial sums fit a double exactly
        assert int(outD[i]) == exact_round_to_bf16(exact)
        assert abs(int(outS[i]) - int(outD[i])) <= 1


# ----------------------------------------------------------------- scale --

def test_scale_pins():
    rng = np.random.default_rng(9)
    x = (rng.standard_normal(2000) * 1e-3).astype(np.float32)
    assert (oracle.scale_array(x, 1.0, "f32").view(np.uint32) == x.view(np.uint32)).all()
    assert (oracle.scale_array(x, 0.5, "f32") == x * np.float32(0.5)).all()
    sc = np.float32(1.0 / 3.0)
    got = oracle.scale_array(x, float(sc), "f32")
    for i in range(0, 2000, 50):
        assert got[i] == frac_round_f32(Fraction(float(sc)) * Fraction(float(x[i])))
    xb = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    for mode in "DS":
        assert (oracle.scale_array(xb, 1.0, "bf16", mode) == xb).all()
    gotD = oracle.scale_array(xb, float(sc), "bf16", "D")
    gotS = oracle.scale_array(xb, float(sc), "bf16", "S")
    for i in range(0, 2000, 20):
        ex = Fraction(float(sc)) * Fraction(oracle.bf16_widen(int(xb[i])))
        assert int(gotD[i]) == exact_round_to_bf16(ex)
        assert int(gotS[i]) == exact_round_to_bf16(Fraction(float(frac_round_f32(ex))))
    lib = (torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).float() * float(sc)) \
        .to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (gotS == lib).all()


# ----------------------------------------------------------- pack/unpack --

@pytest.mark.parametrize("dtype,align", [("f32", 16), ("f32", 4), ("bf16", 16),
                                         ("bf16", 2), ("f32", 256)])
def test_pack_unpack_bruteforce(dtype, align):
    numels = [1, 3, 5, 7, 0, 4, 8, 9, 1, 1, 1, 17, 2, 30]
    es = 4 if dtype == "f32" else 2
    L = oracle.assign_buckets(numels, es, 96, align)
    nd = np.float32 if dtype == "f32" else np.uint16
    tensors, g = [], 1
    for n in numels:
        if dtype == "f32":
            tensors.append(np.arange(g, g + n, dtype=np.float32))
        else:   # finite bf16 patterns, all distinct
            tensors.append((0x3F00 + np.arange(g, g + n)).astype(np.uint16))
        g += n
    buckets = oracle.pack(L, tensors, dtype)
    # brute force: walk every bucket element and find its owner by scanning
    for b, buf in enumerate(buckets):
        assert buf.dtype == nd and buf.size == L["bucket_elems"][b]
        for e in range(buf.size):
            owner = None
            for t, n in enumerate(numels):
                if L["tensor_bucket"][t] == b and L["tensor_offset"][t] <= e < L["tensor_offset"][t] + n:
                    assert owner is None          # tensors never overlap
                    owner = (t, e - L["tensor_offset"][t])
            if owner is None:
                assert buf.view(np.uint32 if dtype == "f32" else np.uint16)[e] == 0
            else:
                assert buf[e] == tensors[owner[0]][owner[1]]
    back = oracle.unpack_scale(L, buckets, numels, 1.0, dtype)
    for a, c in zip(tensors, back):
        assert a.size == c.size and (a == c).all()


def test_pack_preserves_bit_patterns():
    bits = np.array([0x7FC00001, 0xFFFFFFFF, 0x00000001, 0x80000000, 0x7F800001], dtype=np.uint32)
    L = oracle.assign_buckets([5], 4, 0, 16)
    out = oracle.pack(L, [bits.view(np.float32)], "f32")[0]
    assert (out.view(np.uint32)[:5] == bits).all() and (out.view(np.uint32)[5:] == 0).all()


# ------------------------------------------------------------- end to end --

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", ["D", "S"])
def test_bucketed_equals_unbucketed(dtype, mode):
    w_ = wl.ragged_workload(dtype=dtype, K=3, seed=11)
    peers = [[wl.to_host_array(t) for t in wl.gradient_set(w_, k)] for k in range(w_.K)]
    L = oracle.assign_buckets(w_.numels, w_.elem_size, w_.bucket_cap_bytes, 16)
    assert len(L["bucket_elems"]) > 3
    b = oracle.plan_shares(w_.throughputs, w_.global_batch)
    w = oracle.share_weights(b, w_.global_batch)
    packed = [oracle.pack(L, p, dtype) for p in peers]
    red = [oracle.weighted_reduce([packed[k][bi] for k in range(w_.K)], w, dtype, mode)
           for bi in range(len(L["bucket_elems"]))]
    scale = 0.37
    got = oracle.unpack_scale(L, red, w_.numels, scale, dtype, mode)
    ref = oracle.direct(peers, w, scale, dtype, mode)
    for a, c in zip(got, ref):
        assert a.tobytes() == c.tobytes()
    # and against plain numpy float64 on the un-bucketed tensors
    for t in range(len(w_.numels)):
        if dtype == "f32":
            xs = [peers[k][t].astype(np.float64) for k in range(w_.K)]
        else:
            xs = [oracle.bf16_to_f32_array(peers[k][t]).astype(np.float64) for k in range(w_.K)]
        want = scale * sum(float(w[k]) * xs[k] for k in range(w_.K))
        have = got[t].astype(np.float64) if dtype == "f32" else \
            oracle.bf16_to_f32_array(got[t]).astype(np.float64)
        tol = 2e-6 if dtype == "f32" else 2.0 ** -7
        mag = scale * sum(abs(float(w[k])) * np.abs(xs[k]) for k in range(w_.K))
        assert np.all(np.abs(have - want) <= tol * mag + 1e-12)


# ------------------------------------------------------------- two level --

def test_group_weights_and_two_level_pins():
    shares = [183, 183, 146, 146, 110, 110, 73, 73]            # ViT workload, B = 1024
    group_of = [0, 0, 0, 0, 1, 1, 1, 1]
    w1, w2, Bg = oracle.group_weights(shares, group_of, 2)
    assert Bg == [658, 366] and sum(Bg) == 1024
    flat = oracle.share_weights(shares, 1024)
    for k in range(8):   # (b_k/B_g)(B_g/B) = b_k/B up to two roundings
        assert abs(float(w1[k]) * float(w2[group_of[k]]) - float(flat[k])) <= 2.0 ** -23 * float(flat[k])
    for g in range(2):   # level-1 weights of a group sum to one
        assert abs(sum(float(w1[k]) for k in range(8) if group_of[k] == g) - 1.0) <= 4 * 2.0 ** -24
    rng = np.random.default_rng(12)
    xs = [(rng.standard_normal(5000) * 1e-3).astype(np.float32) for _ in range(8)]
    flatD = oracle.weighted_reduce(xs, flat, "f32", "D").astype(np.float64)
    gmax = max(float(np.abs(x).max()) for x in xs)
    for mode in "DS":
        two = oracle.two_level_reduce(xs, shares, group_of, 2, "f32", mode).astype(np.float64)
        assert np.abs(two - flatD).max() <= 1e-6 * gmax + 1e-9
    # identical peers: every level returns the input up to one rounding per level
    two = oracle.two_level_reduce([xs[0]] * 8, shares, group_of, 2, "f32", "D")
    assert np.abs(two.astype(np.float64) - xs[0]).max() <= 2 * 2.0 ** -24 * gmax
    # power-of-two group sizes and integer data: exact
    sh2 = [96, 32, 64, 64]
    xi = rng.integers(-64, 65, size=(4, 2000))
    got = oracle.two_level_reduce([xi[k].astype(np.float32) for k in range(4)], sh2, [0, 0, 1, 1], 2, "f32", "S")
    num = (np.array(sh2)[:, None] * xi).sum(axis=0)
    assert (got.astype(np.float64) * 256 == num).all()
    # one group holding everything is the flat reduce
    one = oracle.two_level_reduce(xs, shares, [0] * 8, 1, "f32", "S")
    assert (one == oracle.weighted_reduce(xs, flat, "f32", "S")).all()
    with pytest.raises(ValueError):
        oracle.group_weights([1, 2], [0, 2], 2)
    with pytest.raises(ValueError):
        oracle.group_weights([1, 2], [0, 0], 2)


# ------------------------------------------------------------------- SGD --

def _one_tensor_layout(n):
    return {"tensor_bucket": [0], "tensor_offset": [0], "bucket_elems": [n]}


def test_sgd_against_torch_optimizer():
    """Three steps of torch.optim.SGD(momentum=0.9, weight_decay=5e-4) on the CPU."""
    rng = np.random.default_rng(21)
    n = 4000
    p0 = rng.standard_normal(n).astype(np.float32)
    grads = [(rng.standard_normal(n) * 1e-2).astype(np.float32) for _ in range(3)]
    lr, mu, wd = 0.1, 0.9, 5e-4
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()))
    opt = torch.optim.SGD([tp], lr=lr, momentum=mu, weight_decay=wd)
    for mode in "DS":
        tp.data.copy_(torch.from_numpy(p0))
        opt.state.clear()
        p, v = [p0.copy()], [np.zeros(n, np.float32)]
        for step, g in enumerate(grads):
            tp.grad = torch.from_numpy(g.copy())
            opt.step()
            p, v = oracle.unpack_sgd(_one_tensor_layout(n), [g], [n], 1.0, p, v, lr, mu, wd, step == 0, "f32", mode)
            ref_p = tp.detach().numpy()
            ref_v = opt.state[tp]["momentum_buffer"].numpy()
            assert np.abs(v[0] - ref_v).max() <= 4 * 2.0 ** -24 * np.abs(ref_v).max()
            assert np.abs(p[0] - ref_p).max() <= 2 * 2.0 ** -24 * np.abs(ref_p).max()


def test_sgd_exact_on_dyadic_data():
    """Small integers and power-of-two constants: every operation is exact, so
    both modes equal rational arithmetic."""
    rng = np.random.default_rng(22)
    n = 500
    x = rng.integers(-8, 9, n).astype(np.float32)
    p0 = rng.integers(-8, 9, n).astype(np.float32)
    v0 = rng.integers(-8, 9, n).astype(np.float32)
    scale, lr, mu, wd = 0.5, 0.25, 0.5, 0.125
    for first in (False, True):
        for mode in "DS":
            p, v = oracle.unpack_sgd(_one_tensor_layout(n), [x], [n], scale, [p0], [v0], lr, mu, wd, first, "f32", mode)
            for i in range(n):
                g = Fraction(scale) * Fraction(float(x[i])) + Fraction(wd) * Fraction(float(p0[i]))
                vv = g if first else Fraction(mu) * Fraction(float(v0[i])) + g
                pp = Fraction(float(p0[i])) - Fraction(lr) * vv
                assert Fraction(float(v[0][i])) == vv and Fraction(float(p[0][i])) == pp


def test_sgd_special_cases_and_modes():
    rng = np.random.default_rng(23)
    n = 3000
    x = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    p0 = rng.standard_normal(n).astype(np.float32)
    v0 = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    lay = _one_tensor_layout(n)
    # no momentum, no decay: p' = p - lr * scale * x
    p, v = oracle.unpack_sgd(lay, [x], [n], 2.0, [p0], [v0], 0.5, 0.0, 0.0, False, "f32", "D")
    assert (v[0] == x * np.float32(2.0)).all()
    assert (p[0] == (p0.astype(np.float64) - 0.5 * (2.0 * x.astype(np.float64))).astype(np.float32)).all()
    # first step ignores the old momentum
    a = oracle.unpack_sgd(lay, [x], [n], 1.0, [p0], [v0], 0.1, 0.9, 5e-4, True, "f32", "D")
    b = oracle.unpack_sgd(lay, [x], [n], 1.0, [p0], [np.zeros(n, np.float32)], 0.1, 0.9, 5e-4, False, "f32", "D")
    assert (a[0][0] == b[0][0]).all() and (a[1][0] == b[1][0]).all()
    # inputs are not modified; D and S stay within a few roundings of each other
    assert (p0 == p0.copy()).all()
    d = oracle.unpack_sgd(lay, [x], [n], 0.37, [p0], [v0], 0.1, 0.9, 5e-4, False, "f32", "D")
    s = oracle.unpack_sgd(lay, [x], [n], 0.37, [p0], [v0], 0.1, 0.9, 5e-4, False, "f32", "S")
    assert np.abs(d[1][0] - s[1][0]).max() <= 3 * 2.0 ** -24 * np.abs(d[1][0]).max()
    assert np.abs(d[0][0] - s[0][0]).max() <= 2 * 2.0 ** -24 * np.abs(d[0][0]).max()
    # bf16 gradients are widened exactly: same as feeding the widened values as fp32
    xb = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    for mode in "DS":
        r16 = oracle.unpack_sgd(lay, [xb], [n], 0.37, [p0], [v0], 0.1, 0.9, 5e-4, False, "bf16", mode)
        r32 = oracle.unpack_sgd(lay, [oracle.bf16_to_f32_array(xb)], [n], 0.37, [p0], [v0], 0.1, 0.9, 5e-4, False, "f32", mode)
        assert (r16[0][0] == r32[0][0]).all() and (r16[1][0] == r32[1][0]).all()
    # offsets: a tensor in the middle of a bucket reads its own slice
    lay2 = {"tensor_bucket": [0, 0], "tensor_offset": [0, 8], "bucket_elems": [16]}
    bucket = np.arange(16, dtype=np.float32)
    pp, vv = oracle.unpack_sgd(lay2, [bucket], [5, 3], 1.0, [np.zeros(5, np.float32), np.zeros(3, np.float32)],
                               [np.zeros(5, np.float32), np.zeros(3, np.float32)], 1.0, 0.0, 0.0, True, "f32", "S")
    assert list(vv[0]) == [0, 1, 2, 3, 4] and list(vv[1]) == [8, 9, 10] and list(pp[1]) == [-8, -9, -10]


def test_sgd_master_model_copy_is_the_library_bf16_rounding():
    """Mixed precision: the bf16 model copy equals torch's float32 -> bfloat16
    conversion (round to nearest-even) of the updated master parameters, which
    themselves equal the plain update; ties, overflow to infinity, NaN, signed
    zeros and subnormals included."""
    rng = np.random.default_rng(24)
    n = 200000
    x = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    p0 = rng.standard_normal(n).astype(np.float32)
    v0 = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    lay = _one_tensor_layout(n)
    for mode in "DS":
        p, v = oracle.unpack_sgd(lay, [x], [n], 0.37, [p0], [v0], 0.1, 0.9, 5e-4, False, "f32", mode)
        pm, vm, mm = oracle.unpack_sgd_master(lay, [x], [n], 0.37, [p0], [v0], 0.1, 0.9, 5e-4, False, "f32", mode)
        assert (pm[0] == p[0]).all() and (vm[0] == v[0]).all()
        want = torch.from_numpy(p[0]).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert (mm[0] == want).all()
    # chosen master values through the model-copy step alone
    bits = np.array([0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF,      # ties to even (down, up), just above, just below
                     0x7F7FFFFF, 0xFF7FFFFF,                              # largest finite -> +-infinity
                     0x7F800000, 0xFF800000, 0x7FC00001, 0x7F800001,      # infinities, quiet and signalling NaN
                     0x00000000, 0x80000000, 0x00000001, 0x00008000, 0x00018000, 0x007FFFFF],   # zeros, subnormals
                    dtype=np.uint32)
    p_special = bits.view(np.float32).copy()
    m = len(bits)
    out = np.empty(m, np.uint16)
    oracle._c().kto_f32_to_bf16(p_special.ctypes.data, m, out.ctypes.data)
    mm = [out]
    expect = [0x3F80, 0x3F82, 0x3F81, 0x3F80, 0x7F80, 0xFF80, 0x7F80, 0xFF80, None, None,
              0x0000, 0x8000, 0x0000, 0x0000, 0x0002, 0x0080]
    for got, want, b in zip(mm[0], expect, bits):
        if want is None:
            assert (got & 0x7F80) == 0x7F80 and (got & 0x007F) != 0 and (got & 0x0040), hex(b)    # a quiet NaN
        else:
            assert got == want, (hex(b), hex(got), hex(want))
