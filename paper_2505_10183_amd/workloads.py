"""Seeded synthetic gradient sets shaped like the training workloads.

This module only *describes* inputs: tensor shape lists of five published
network architectures, the per-device throughputs / global batch size that go
with each, and seeded Gaussian value generators.  It holds none of the
method's arithmetic (no share planning, no bucket layout, no reduction) and is
the one module that both the GPU path's callers and the CPU checker's callers
may use, so that both sides see the same inputs.

The paper trains MobileNetV2 on CIFAR-10 with a global batch of 256 (Sec. IV-B);
the ``mobilenetv2`` workload takes that network's parameter-tensor shapes
(tensor count and size mix), not its data.  The other four extend the same idea
to a tiny MLP, ResNet-18 (CIFAR head), ViT-B/16 and a 1.3B-parameter decoder.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from functools import cached_property
from typing import List, Sequence, Tuple

import numpy as np

Shape = Tuple[int, ...]


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                      # "f32" or "bf16"
    shapes: Tuple[Shape, ...]       # parameter tensors, forward order
    throughputs: Tuple[float, ...]  # samples/ms per peer device (K entries)
    global_batch: int               # B
    bucket_cap_bytes: int           # 0 = one bucket holding everything
    sigma: float                    # std of the Gaussian gradient values
    seed: int
    labels: Tuple[str, ...] = field(default=(), compare=False)

    @property
    def K(self) -> int:
        return len(self.throughputs)

    @cached_property
    def numels(self) -> List[int]:
        return [int(np.prod(s, dtype=np.int64)) for s in self.shapes]

    @cached_property
    def total_elems(self) -> int:
        return int(sum(self.numels))

    @property
    def elem_size(self) -> int:
        return 4 if self.dtype == "f32" else 2


MiB = 1 << 20


def _mlp_shapes():
    return [(784, 256), (256,), (256, 128), (128,), (128, 10), (10,)]


def _bn(c):
    return [(c,), (c,)]


def _resnet18_cifar_shapes():
    s: List[Shape] = [(64, 3, 3, 3)] + _bn(64)
    cin = 64
    for cout in (64, 128, 256, 512):
        for blk in range(2):
            s += [(cout, cin if blk == 0 else cout, 3, 3)] + _bn(cout)
            s += [(cout, cout, 3, 3)] + _bn(cout)
            if blk == 0 and cout != cin:
                s += [(cout, cin, 1, 1)] + _bn(cout)
        cin = cout
    s += [(10, 512), (10,)]
    return s


def _mobilenetv2_shapes():
    s: List[Shape] = [(32, 3, 3, 3)] + _bn(32)
    cin = 32
    for t, c, n in ((1, 16, 1), (6, 24, 2), (6, 32, 3), (6, 64, 4),
                    (6, 96, 3), (6, 160, 3), (6, 320, 1)):
        for _ in range(n):
            hidden = cin * t
            if t != 1:
                s += [(hidden, cin, 1, 1)] + _bn(hidden)
            s += [(hidden, 1, 3, 3)] + _bn(hidden)
            s += [(c, hidden, 1, 1)] + _bn(c)
            cin = c
    s += [(1280, 320, 1, 1)] + _bn(1280)
    s += [(10, 1280), (10,)]
    return s


def _vit_b16_shapes():
    d = 768
    s: List[Shape] = [(1, 1, d), (1, 197, d), (d, 3, 16, 16), (d,)]
    for _ in range(12):
        s += [(d,), (d,), (3 * d, d), (3 * d,), (d, d), (d,),
              (d,), (d,), (4 * d, d), (4 * d,), (d, 4 * d), (d,)]
    s += [(d,), (d,), (1000, d), (1000,)]
    return s


def _decoder_1p3b_shapes():
    d = 2048
    s: List[Shape] = [(50304, d), (2048, d)]
    for _ in range(24):
        s += [(d,), (d,), (3 * d, d), (3 * d,), (d, d), (d,),
              (d,), (d,), (4 * d, d), (4 * d,), (d, 4 * d), (d,)]
    s += [(d,), (d,)]
    return s


WORKLOADS = {
    w.name: w for w in (
        Workload("mlp", "f32", tuple(_mlp_shapes()), (1.0, 0.6), 128, 0, 1e-2,
                 20250510),
        Workload("resnet18", "f32", tuple(_resnet18_cifar_shapes()),
                 (1.0, 1.0, 0.55, 0.55), 512, 25 * MiB, 1e-3, 20250511),
        Workload("mobilenetv2", "f32", tuple(_mobilenetv2_shapes()),
                 (1.0, 0.8, 0.5, 0.5), 256, 25 * MiB, 1e-3, 20250512),
        Workload("vit_b16", "f32", tuple(_vit_b16_shapes()),
                 (1.0, 1.0, 0.8, 0.8, 0.6, 0.6, 0.4, 0.4), 1024, 25 * MiB,
                 1e-3, 20250513),
        Workload("decoder_1p3b", "bf16", tuple(_decoder_1p3b_shapes()),
                 (1.0, 1.0, 0.7, 0.7, 0.5, 0.5, 0.3, 0.3), 2048, 64 * MiB,
                 1e-4, 20250514),
    )
}

WORKLOAD_ORDER = ("mlp", "resnet18", "mobilenetv2", "vit_b16", "decoder_1p3b")


def sized_workload(name: str) -> Workload:
    """`sized_<dtype>_<tiles>`: 24 equal tensors that fill `tiles` 16 KiB tiles per peer, K = 8,
    25 MiB (f32) or 64 MiB (bf16) buckets: gradient sets of any size for measurements that depend
    on the launch size."""
    _, dtype, tiles = name.split("_")
    es = 4 if dtype == "f32" else 2
    n = int(tiles) * (16384 // es)
    return Workload(name, dtype, tuple(((n // 24),) for _ in range(24)), (1.0, 1.0, 0.8, 0.8, 0.6, 0.6, 0.4, 0.4),
                    1024, (25 if dtype == "f32" else 64) * MiB, 1e-3, 99)


def get(name: str) -> Workload:
    """A named workload of the table, or a `sized_<dtype>_<tiles>` one."""
    if name in WORKLOADS:
        return WORKLOADS[name]
    if name.startswith("sized_"):
        return sized_workload(name)
    raise KeyError(name)


def ragged_workload(name: str = "ragged", dtype: str = "f32", K: int = 3,
                    seed: int = 7, n_tensors: int = 40,
                    cap_bytes: int = 96 * 1024) -> Workload:
    """A small, deliberately awkward gradient set for parity tests.

    Sizes mix 1/3/5/7-element tensors, sizes straddling 16-byte vectors, sizes
    a little above/below a kernel tile, and a few tensors larger than the
    bucket cap, so that a plan built from it spans several tiles per bucket,
    several buckets, ragged tails and an oversize bucket.
    """
    rng = np.random.default_rng(seed)
    fixed = [1, 3, 5, 7, 2, 4, 8, 9, 15, 16, 17, 31, 33, 127, 129, 1000, 1023,
             1025, 8191, 8192, 8193, 16385, 40000, 70001]
    extra = [int(x) for x in rng.integers(1, 5000, size=max(0, n_tensors - len(fixed)))]
    sizes = fixed + extra
    order = rng.permutation(len(sizes))
    shapes = tuple((sizes[i],) for i in order)
    thr = tuple(float(x) for x in np.round(rng.uniform(0.3, 1.0, size=K), 2))
    return Workload(name, dtype, shapes, thr, 96, cap_bytes, 1e-3, seed)


# --------------------------------------------------------------------------
# Value generators.  torch is used only as a seeded random-number source and a
# container; the same tensors are handed to the GPU path (on device) and, as
# host copies, to the CPU checker.
# --------------------------------------------------------------------------

def _torch():
    import torch
    return torch


def torch_dtype(dtype: str):
    torch = _torch()
    return torch.float32 if dtype == "f32" else torch.bfloat16


def gradient_set(w: Workload, peer: int, device="cpu", kind: str = "normal"):
    """One peer's gradients: a list of contiguous tensors, one per shape.

    kind = "normal": i.i.d. N(0, sigma^2) drawn in fp32 (then rounded to bf16
    by torch for the bf16 workload); "ints": integers uniform in [-64, 64];
    "same": like "normal" but identical for every peer.
    """
    torch = _torch()
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    p = 0 if kind == "same" else peer
    gen.manual_seed(w.seed * 1000 + p)
    out = []
    dt = torch_dtype(w.dtype)
    for shp in w.shapes:
        if kind == "ints":
            t = torch.randint(-64, 65, shp, generator=gen, device=dev,
                              dtype=torch.int32).to(torch.float32)
        else:
            t = torch.randn(shp, generator=gen, device=dev,
                            dtype=torch.float32) * w.sigma
        out.append(t.to(dt).contiguous())
    return out


def flat_normal(n: int, dtype: str, sigma: float, seed: int, device="cpu"):
    """A flat buffer of n Gaussian values (a peer's bucket as it would arrive
    from another device)."""
    torch = _torch()
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    t = torch.randn(n, generator=gen, device=dev, dtype=torch.float32) * sigma
    return t.to(torch_dtype(dtype))


def to_host_array(t) -> np.ndarray:
    """Host numpy copy of a tensor; bf16 is returned as its raw uint16 bits."""
    torch = _torch()
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).reshape(-1).copy()
    return t.numpy().reshape(-1).copy()
