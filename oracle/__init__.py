"""CPU checker ("oracle") for the gradient bucket reduction stage.

TEST INFRASTRUCTURE ONLY: used by the tests, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library never imports, links or calls
anything in this directory, and nothing here imports the GPU package.

What it computes (KAITIAN, Sec. III and III-C):

* ``plan_shares``      -- per-device batch sizes b_i proportional to the device
                          score, rounded to integers that sum to B_global
                          (Sec. III-C, phase 2 and its display equation);
* ``share_weights``    -- w_k = b_k / B, the weights under which per-device mean
                          gradients combine into the global-batch mean;
* ``assign_buckets``   -- which flat bucket each gradient tensor is copied into
                          and at which element offset (the flattening DDP does
                          before the gradient AllReduce, Sec. III);
* ``pack``             -- bucket[off_t + i] = g_t[i];
* ``weighted_reduce``  -- out[i] = sum_k w_k * x_k[i], ascending k;
* ``unpack_scale``     -- g_t[i] = scale * bucket[off_t + i];
* ``direct``           -- the same end result with no buckets at all:
                          g_t[i] = scale * sum_k w_k g_t^(k)[i];
* ``sampler_epoch``    -- the dataset indices a device processes in an epoch when
                          every global batch is split by the shares (Sec. III-C
                          phase 2, Sec. IV-A);
* ``group_weights``, ``two_level_reduce`` -- reduction inside groups, then
                          across groups (Sec. III-A);
* ``unpack_sgd``       -- unpack fused with SGD momentum / weight decay (the
                          optimizer of Sec. IV-B); ``unpack_sgd_master`` adds
                          the bf16 model copy of mixed-precision training;
* ``replan_shares``    -- online adaptation of the shares from measured step
                          times (Sec. III-C phase 1).

Element arithmetic lives in ``kt_oracle.c`` (plain C, doubles); integer
planning is plain Python below.  Arrays are numpy: float32 for fp32 data,
uint16 raw bits for bf16 data.

Parity pins: every function here is pinned by tests/test_oracle_*.py against
closed forms, invariants, exact rational arithmetic, brute force on tiny
inputs and library special cases; none is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from typing import Dict, List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kt_oracle.c")
_LIB = os.path.join(_HERE, "libkt_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile kt_oracle.c with gcc (no fused contraction, no fast-math)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math",
             "-Wall", "-Wextra", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _c():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        pp = ctypes.POINTER(ctypes.c_void_p)
        i64, f32, vp = ctypes.c_int64, ctypes.c_float, ctypes.c_void_p
        for name in ("kto_reduce_f32_D", "kto_reduce_f32_S",
                     "kto_reduce_bf16_D", "kto_reduce_bf16_S"):
            fn = getattr(lib, name)
            fn.argtypes = [pp, vp, ctypes.c_int, i64, vp]
            fn.restype = None
        for name in ("kto_scale_f32", "kto_scale_bf16_D", "kto_scale_bf16_S"):
            fn = getattr(lib, name)
            fn.argtypes = [vp, i64, f32, vp]
            fn.restype = None
        for name in ("kto_sgd_f32_D", "kto_sgd_f32_S", "kto_sgd_bf16_D", "kto_sgd_bf16_S"):
            fn = getattr(lib, name)
            fn.argtypes = [vp, i64, f32, vp, vp, f32, f32, f32, ctypes.c_int]
            fn.restype = None
        lib.kto_f32_to_bf16.argtypes = [vp, i64, vp]
        lib.kto_f32_to_bf16.restype = None
        lib.kto_bf16_widen.argtypes = [ctypes.c_uint16]
        lib.kto_bf16_widen.restype = ctypes.c_float
        lib.kto_bf16_round.argtypes = [ctypes.c_double]
        lib.kto_bf16_round.restype = ctypes.c_uint16
        _lib = lib
    return _lib


# --------------------------------------------------------------------------
# Sec. III-C: scores -> integer batch shares -> combine weights
# --------------------------------------------------------------------------

def plan_shares(thr: Sequence[float], B: int) -> List[int]:
    """Integer batch shares b_i with b_i ~ score_i / sum_j score_j * B and
    sum_i b_i = B (Sec. III-C display equation and the sentence after it).

    ``thr`` are device throughputs (samples per unit time); score_i =
    time_fastest / time_i = thr_i / max thr, and the common factor cancels in
    score_i / sum_j score_j, so throughputs are used directly.

    Reading of the integer-rounding rule stated after the Sec. III-C display
    equation (which gives no tie or fix-up rule): largest remainder.  Take the floor of every quota, then give one extra
    sample to the R = B - sum floor entries with the largest fractional parts
    (ties to the lowest index).  Whenever plain rounding already sums to B
    this is plain rounding.

    Quotas are IEEE doubles: S = left-to-right sum, q_i = (thr_i / S) * B.
    """
    K = len(thr)
    if K < 1 or B < 0 or B > (1 << 40):
        raise ValueError("need K >= 1 and 0 <= B <= 2^40")
    for t in thr:
        if not (math.isfinite(t) and t > 0.0):
            raise ValueError("throughputs must be finite and > 0")
    S = 0.0
    for t in thr:
        S = S + float(t)
    if not math.isfinite(S):
        raise ValueError("throughput sum overflows")
    q = [(float(t) / S) * float(B) for t in thr]
    fl = [math.floor(x) for x in q]
    frac = [x - f for x, f in zip(q, fl)]
    b = [int(f) for f in fl]
    R = B - sum(b)
    if R < 0 or R > K:
        raise ArithmeticError("remainder out of range")
    order = sorted(range(K), key=lambda i: (-frac[i], i))
    for i in order[:R]:
        b[i] += 1
    return b


def share_weights(shares: Sequence[int], B: int) -> np.ndarray:
    """w_k = b_k / B as one binary32 division of the two converted integers."""
    if B <= 0:
        raise ValueError("B must be positive to form weights")
    return np.array([np.float32(b) / np.float32(B) for b in shares],
                    dtype=np.float32)


# --------------------------------------------------------------------------
# Bucket layout (the flattening step of DDP's gradient AllReduce, Sec. III)
# --------------------------------------------------------------------------

def assign_buckets(numels: Sequence[int], elem_size: int, cap_bytes: int,
                   align_bytes: int) -> Dict[str, List[int]]:
    """Greedy bucket layout in the caller's tensor order.

    Each tensor starts at the next multiple of ``align_bytes`` inside its
    bucket.  A bucket is closed before a tensor whose (aligned) end would make
    the bucket longer than ``cap_bytes``; tensors are never split, so a tensor
    larger than the cap sits alone.  ``cap_bytes == 0`` means a single bucket.
    A bucket's length is its last tensor's end rounded up to the alignment.
    """
    if elem_size not in (2, 4):
        raise ValueError("elem_size")
    if (align_bytes < elem_size or align_bytes % elem_size
            or align_bytes & (align_bytes - 1) or align_bytes > 16384):
        raise ValueError("align_bytes")
    if cap_bytes < 0:
        raise ValueError("cap_bytes")
    A = align_bytes // elem_size

    def up(x):
        return (x + A - 1) // A * A

    t_bucket, t_off = [], []
    b_first, b_count, b_elems = [], [], []
    cur_end = 0          # end (elements) of the last tensor in the open bucket
    open_count = 0
    for t, n in enumerate(numels):
        if n < 0:
            raise ValueError("numel")
        start = up(cur_end)
        if (open_count > 0 and cap_bytes > 0
                and up(start + n) * elem_size > cap_bytes):
            b_count.append(open_count)
            b_elems.append(up(cur_end))
            cur_end, open_count, start = 0, 0, 0
        if open_count == 0:
            b_first.append(t)
        t_bucket.append(len(b_first) - 1)
        t_off.append(start)
        cur_end = start + n
        open_count += 1
    if open_count > 0:
        b_count.append(open_count)
        b_elems.append(up(cur_end))
    return {"tensor_bucket": t_bucket, "tensor_offset": t_off,
            "bucket_first": b_first, "bucket_count": b_count,
            "bucket_elems": b_elems}


# --------------------------------------------------------------------------
# pack / reduce / unpack
# --------------------------------------------------------------------------

def _np_dtype(dtype: str):
    return {"f32": np.float32, "bf16": np.uint16}[dtype]


def pack(layout, tensors: Sequence[np.ndarray], dtype: str) -> List[np.ndarray]:
    """bucket[off_t + i] = g_t[i]; every padding element is +0 (all bits 0).
    Raw copies: bit patterns are preserved."""
    nd = _np_dtype(dtype)
    raw = np.uint32 if dtype == "f32" else np.uint16
    buckets = [np.zeros(n, dtype=raw) for n in layout["bucket_elems"]]
    for t, g in enumerate(tensors):
        g = np.ascontiguousarray(g, dtype=nd).reshape(-1)
        o = layout["tensor_offset"][t]
        buckets[layout["tensor_bucket"][t]][o:o + g.size] = g.view(raw)
    return [b.view(nd) for b in buckets]


def weighted_reduce(peers: Sequence[np.ndarray], w: np.ndarray, dtype: str,
                    mode: str = "D") -> np.ndarray:
    """out[i] = sum_{k=0}^{K-1} w_k * x_k[i], ascending k (mode D: double
    accumulation, one final rounding; mode S: binary32 product then fused
    multiply-adds)."""
    nd = _np_dtype(dtype)
    K = len(peers)
    if K < 1 or len(w) != K:
        raise ValueError("K")
    xs = [np.ascontiguousarray(p, dtype=nd).reshape(-1) for p in peers]
    n = xs[0].size
    if any(x.size != n for x in xs):
        raise ValueError("peer sizes differ")
    wv = np.ascontiguousarray(w, dtype=np.float32)
    out = np.empty(n, dtype=nd)
    ptrs = (ctypes.c_void_p * K)(*[x.ctypes.data for x in xs])
    fn = getattr(_c(), "kto_reduce_%s_%s" % (dtype, mode))
    fn(ptrs, wv.ctypes.data, K, n, out.ctypes.data)
    return out


def scale_array(x: np.ndarray, scale: float, dtype: str, mode: str = "D") -> np.ndarray:
    nd = _np_dtype(dtype)
    x = np.ascontiguousarray(x, dtype=nd).reshape(-1)
    out = np.empty_like(x)
    name = "kto_scale_f32" if dtype == "f32" else "kto_scale_bf16_" + mode
    getattr(_c(), name)(x.ctypes.data, x.size, ctypes.c_float(scale), out.ctypes.data)
    return out


def unpack_scale(layout, buckets: Sequence[np.ndarray], numels: Sequence[int],
                 scale: float, dtype: str, mode: str = "D") -> List[np.ndarray]:
    """g_t[i] = scale * bucket[off_t + i]; padding is never read."""
    out = []
    for t, n in enumerate(numels):
        o = layout["tensor_offset"][t]
        b = buckets[layout["tensor_bucket"][t]]
        out.append(scale_array(b[o:o + n], scale, dtype, mode))
    return out


def direct(peer_tensors: Sequence[Sequence[np.ndarray]], w: np.ndarray,
           scale: float, dtype: str, mode: str = "D") -> List[np.ndarray]:
    """The end result with no buckets: for every tensor t,
    g_t = scale * sum_k w_k g_t^(k) (two roundings to the storage type, one
    after the sum and one after the scale, like the bucketed path)."""
    K = len(peer_tensors)
    T = len(peer_tensors[0])
    res = []
    for t in range(T):
        s = weighted_reduce([peer_tensors[k][t] for k in range(K)], w, dtype, mode)
        res.append(scale_array(s, scale, dtype, mode))
    return res


# --------------------------------------------------------------------------
# bf16 helpers (scalar, for tests)
# --------------------------------------------------------------------------

def bf16_widen(bits: int) -> float:
    return float(_c().kto_bf16_widen(int(bits)))


def bf16_round(x: float) -> int:
    return int(_c().kto_bf16_round(float(x)))


def bf16_to_f32_array(bits: np.ndarray) -> np.ndarray:
    """Exact widening of an array of bf16 bit patterns (numpy, no C)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# Load-adaptive sampler partition (Sec. III-C phase 2: every device receives a
# portion of each global mini-batch sized by its score; Sec. IV-A says only
# that the sampler override splits the dataset indices by the scores)
# --------------------------------------------------------------------------

_M64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15


class SplitMix64:
    """SplitMix64 (Steele, Lea, Flood 2014): state += gamma; output = mix(state)."""

    def __init__(self, state: int):
        self.state = state & _M64

    def next(self) -> int:
        self.state = (self.state + _GAMMA) & _M64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
        return z ^ (z >> 31)


def _bounded(rng: SplitMix64, n: int) -> int:
    """Unbiased integer in [0, n) from 64-bit draws (Lemire 2019: multiply,
    take the high word, reject the few low words that would bias)."""
    m = rng.next() * n
    low = m & _M64
    if low < n:
        t = ((1 << 64) - n) % n
        while low < t:
            m = rng.next() * n
            low = m & _M64
    return m >> 64


def epoch_permutation(N: int, seed: int, epoch: int, shuffle: bool = True) -> List[int]:
    """The epoch's ordering of dataset indices: identity, or a Fisher-Yates
    shuffle (i = N-1 .. 1, swap with a uniform j <= i) driven by SplitMix64
    started at state seed + epoch * gamma."""
    a = list(range(N))
    if shuffle:
        rng = SplitMix64(seed + epoch * _GAMMA)
        for i in range(N - 1, 0, -1):
            j = _bounded(rng, i + 1)
            a[i], a[j] = a[j], a[i]
    return a


def sampler_epoch(N: int, B: int, shares: Sequence[int], seed: int, epoch: int,
                  rank: int, shuffle: bool = True, drop_last: bool = False) -> List[int]:
    """Dataset indices device ``rank`` processes in one epoch.

    The epoch ordering is cut into global mini-batches of B indices; inside
    every global batch device k takes the contiguous slice of b_k indices that
    starts at b_0 + ... + b_{k-1}.  If N is not a multiple of B the last batch
    is dropped (drop_last) or completed by wrapping around to the start of the
    ordering (as torch's DistributedSampler pads)."""
    K = len(shares)
    if N < 0 or B < 1 or sum(shares) != B or any(b < 0 for b in shares) or not 0 <= rank < K:
        raise ValueError("bad sampler arguments")
    perm = epoch_permutation(N, seed, epoch, shuffle)
    steps = N // B if drop_last else (N + B - 1) // B
    start = sum(shares[:rank])
    out = []
    for s in range(steps):
        for i in range(shares[rank]):
            out.append(perm[(s * B + start + i) % N])
    return out


# --------------------------------------------------------------------------
# Two-level combination (Sec. III-A: gradients are first reduced inside each
# group of homogeneous accelerators, then the group results are combined
# across groups through host memory)
# --------------------------------------------------------------------------

def group_weights(shares: Sequence[int], group_of: Sequence[int], G: int):
    """Level 1: device k of group g weighs b_k / B_g (B_g = the group's samples),
    so a group's result is the mean gradient over the group's samples.
    Level 2: group g weighs B_g / B.  Both as single binary32 divisions.
    The product (b_k/B_g)(B_g/B) = b_k/B is the flat weight."""
    K = len(shares)
    if len(group_of) != K or G < 1 or any(not 0 <= g < G for g in group_of):
        raise ValueError("group_of")
    Bg = [0] * G
    for b, g in zip(shares, group_of):
        Bg[g] += b
    B = sum(shares)
    if B <= 0 or any(x <= 0 for x in Bg):
        raise ValueError("every group needs a positive share")
    w1 = np.array([np.float32(b) / np.float32(Bg[g]) for b, g in zip(shares, group_of)], dtype=np.float32)
    w2 = np.array([np.float32(x) / np.float32(B) for x in Bg], dtype=np.float32)
    return w1, w2, Bg


def two_level_reduce(peers: Sequence[np.ndarray], shares: Sequence[int], group_of: Sequence[int],
                     G: int, dtype: str, mode: str = "D") -> np.ndarray:
    """out = sum_g (B_g/B) * y_g with y_g = sum_{k in g} (b_k/B_g) x_k; each
    level is a weighted_reduce (group members in ascending k, groups in
    ascending g) and y_g is stored in the bucket's element type in between."""
    w1, w2, _ = group_weights(shares, group_of, G)
    ys = []
    for g in range(G):
        idx = [k for k in range(len(peers)) if group_of[k] == g]
        ys.append(weighted_reduce([peers[k] for k in idx], w1[idx], dtype, mode))
    return weighted_reduce(ys, w2, dtype, mode)


# --------------------------------------------------------------------------
# SGD with momentum and weight decay while unpacking (Sec. IV-B: the optimizer
# of the paper's runs: momentum 0.9, weight decay 5e-4)
# --------------------------------------------------------------------------

def unpack_sgd(layout, buckets: Sequence[np.ndarray], numels: Sequence[int], scale: float,
               params: Sequence[np.ndarray], momenta: Sequence[np.ndarray], lr: float, momentum: float,
               weight_decay: float, first_step: bool, dtype: str, mode: str = "D"):
    """For every tensor t and element i, with g = scale * bucket[off_t + i]:
    g' = g + wd * p;  v' = g' on the first step, else mu * v + g';  p' = p - lr * v'.
    Returns new (params, momenta) lists; inputs are not modified."""
    new_p, new_v = [], []
    fn = getattr(_c(), "kto_sgd_%s_%s" % (dtype, mode))
    nd = _np_dtype(dtype)
    for t, n in enumerate(numels):
        o = layout["tensor_offset"][t]
        x = np.ascontiguousarray(buckets[layout["tensor_bucket"][t]][o:o + n], dtype=nd)
        p = np.array(params[t], dtype=np.float32).reshape(-1).copy()
        v = np.array(momenta[t], dtype=np.float32).reshape(-1).copy()
        assert p.size == n and v.size == n
        fn(x.ctypes.data, n, ctypes.c_float(scale), p.ctypes.data, v.ctypes.data, ctypes.c_float(lr),
           ctypes.c_float(momentum), ctypes.c_float(weight_decay), int(bool(first_step)))
        new_p.append(p)
        new_v.append(v)
    return new_p, new_v


def unpack_sgd_master(layout, buckets: Sequence[np.ndarray], numels: Sequence[int], scale: float,
                      masters: Sequence[np.ndarray], momenta: Sequence[np.ndarray], lr: float, momentum: float,
                      weight_decay: float, first_step: bool, dtype: str, mode: str = "D"):
    """unpack_sgd for mixed-precision training: the binary32 parameters are the
    master copy and the model that forward / backward use holds each updated
    value rounded once, to nearest-even, to bf16.  Returns (masters, momenta,
    models); models are uint16 bit patterns."""
    new_p, new_v = unpack_sgd(layout, buckets, numels, scale, masters, momenta, lr, momentum, weight_decay,
                              first_step, dtype, mode)
    models = []
    for p in new_p:
        m = np.empty(p.size, dtype=np.uint16)
        _c().kto_f32_to_bf16(p.ctypes.data, p.size, m.ctypes.data)
        models.append(m)
    return new_p, new_v, models


# --------------------------------------------------------------------------
# Online adaptation of the scores (Sec. III-C phase 1, "Online Adaptation":
# monitor computation time per batch during training and adjust the scores)
# --------------------------------------------------------------------------

def replan_shares(step_time: Sequence[float], shares_used: Sequence[int],
                  ema: Sequence[float], alpha: float, B: int):
    """One adaptation step.  Device k processed shares_used[k] samples in
    step_time[k]; its time per sample tau_k = t_k / b_k enters an exponential
    moving average  ema_k <- alpha * tau_k + (1 - alpha) * ema_k  (ema_k <= 0
    means "no estimate yet" and is replaced by tau_k; a device that processed
    no samples keeps its estimate).  The score is the speed 1 / ema_k and the
    new shares are plan_shares(1 / ema, B).  Returns (new_ema, shares)."""
    K = len(step_time)
    if len(shares_used) != K or len(ema) != K or not (0.0 < alpha <= 1.0):
        raise ValueError("bad arguments")
    new = []
    for t, b, e in zip(step_time, shares_used, ema):
        e = float(e)
        if b > 0:
            if not (math.isfinite(t) and t > 0.0):
                raise ValueError("step times must be finite and > 0")
            tau = float(t) / float(b)
            e = tau if not e > 0.0 else alpha * tau + (1.0 - alpha) * e
        if not (e > 0.0 and math.isfinite(e)):
            raise ValueError("no speed estimate for a device")
        new.append(e)
    thr = [1.0 / e for e in new]
    return new, plan_shares(thr, B)
