"""Thin ctypes binding over libkt.so: argument marshalling only.

Every step of the path (share planning, bucket layout, pack, reduce, unpack)
runs inside the C-ABI library; this module converts Python lists / torch
tensors to the pointers and sizes the C functions take and raises on a non-zero
status.  There is no fallback: if the library is missing, loading fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkt.so")

KT_F32, KT_BF16 = 0, 1
KT_ALL_BUCKETS = -1
KT_MAX_PEERS = 64
_DTYPES = {"f32": KT_F32, "bf16": KT_BF16}

_lib = None


class KtError(RuntimeError):
    def __init__(self, status: int, name: str, msg: str):
        super().__init__("%s: %s" % (name, msg))
        self.status = status
        self.status_name = name


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libkt.so is not built (%s); run __graft_entry__.build() or "
                "python paper_2505_10183_amd/build.py" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        c = ctypes
        vp, i64, i32 = c.c_void_p, c.c_int64, c.c_int
        L.kt_version.restype = c.c_char_p
        L.kt_status_string.restype = c.c_char_p
        L.kt_status_string.argtypes = [i32]
        L.kt_last_error.restype = c.c_char_p
        L.kt_plan_shares.argtypes = [c.POINTER(c.c_double), i32, i64, c.POINTER(i64), c.POINTER(c.c_float)]
        L.kt_plan_create.argtypes = [c.POINTER(i64), i32, i32, i64, i32, c.POINTER(vp)]
        L.kt_plan_destroy.argtypes = [vp]
        L.kt_plan_num_buckets.argtypes = [vp]
        L.kt_plan_num_tensors.argtypes = [vp]
        L.kt_plan_bucket_info.argtypes = [vp, i32, c.POINTER(i64), c.POINTER(i32), c.POINTER(i32)]
        L.kt_plan_tensor_info.argtypes = [vp, i32, c.POINTER(i32), c.POINTER(i64)]
        L.kt_plan_num_tiles.argtypes = [vp]
        L.kt_plan_num_tiles.restype = i64
        L.kt_plan_tile_info.argtypes = [vp, i64, c.POINTER(i32), c.POINTER(i64), c.POINTER(i32), c.POINTER(i32)]
        L.kt_plan_tile_info.restype = i32
        L.kt_bucket_pack.argtypes = [vp, i32, c.POINTER(vp), c.POINTER(vp), vp]
        L.kt_weighted_reduce.argtypes = [vp, i32, c.POINTER(vp), i32, c.POINTER(c.c_float), c.POINTER(vp), vp]
        L.kt_bucket_unpack_scale.argtypes = [vp, i32, c.POINTER(vp), c.c_float, c.POINTER(vp), vp]
        L.kt_replan_shares.argtypes = [c.POINTER(c.c_double), c.POINTER(i64), c.POINTER(c.c_double), c.c_double, i32,
                                       i64, c.POINTER(i64), c.POINTER(c.c_float)]
        L.kt_replan_shares.restype = i32
        L.kt_plan_group_weights.argtypes = [c.POINTER(i64), i32, c.POINTER(i32), i32, c.POINTER(c.c_float),
                                            c.POINTER(c.c_float), c.POINTER(i64)]
        L.kt_plan_group_weights.restype = i32
        L.kt_sampler_epoch_size.argtypes = [i64, i64, c.POINTER(i64), i32, i32, i32, c.POINTER(i64)]
        L.kt_sampler_epoch_size.restype = i32
        L.kt_sampler_epoch.argtypes = [i64, i64, c.POINTER(i64), i32, c.c_uint64, c.c_uint64, i32, i32, i32,
                                       c.POINTER(i64), i64, c.POINTER(i64)]
        L.kt_sampler_epoch.restype = i32
        L.kt_bucket_unpack_sgd.argtypes = [vp, i32, c.POINTER(vp), c.c_float, c.POINTER(vp), c.POINTER(vp), c.c_float,
                                           c.c_float, c.c_float, i32, vp]
        L.kt_bucket_unpack_sgd.restype = i32
        L.kt_bucket_unpack_sgd_master.argtypes = [vp, i32, c.POINTER(vp), c.c_float, c.POINTER(vp), c.POINTER(vp),
                                                  c.POINTER(vp), c.c_float, c.c_float, c.c_float, i32, vp]
        L.kt_bucket_unpack_sgd_master.restype = i32
        L.kt_plan_set_weights.argtypes = [vp, c.POINTER(c.c_float), i32, vp]
        L.kt_plan_set_weights.restype = i32
        L.kt_plan_set_sgd.argtypes = [vp, c.c_float, c.c_float, c.c_float, c.c_float, vp]
        L.kt_plan_set_sgd.restype = i32
        L.kt_bucket_unpack_sgd_resident.argtypes = [vp, i32, c.POINTER(vp), c.POINTER(vp), c.POINTER(vp), c.POINTER(vp),
                                                    i32, vp]
        L.kt_bucket_unpack_sgd_resident.restype = i32
        L.kt_fused_step_sgd.argtypes = [vp, i32, c.POINTER(vp), c.POINTER(vp), i32, c.POINTER(c.c_float), c.c_float,
                                        c.POINTER(vp), c.POINTER(vp), c.POINTER(vp), c.c_float, c.c_float, c.c_float,
                                        i32, vp]
        L.kt_fused_step_sgd.restype = i32
        L.kt_fused_step_sgd_resident.argtypes = [vp, i32, c.POINTER(vp), c.POINTER(vp), i32, c.POINTER(vp), c.POINTER(vp),
                                                 c.POINTER(vp), i32, vp]
        L.kt_fused_step_sgd_resident.restype = i32
        L.kt_fused_step.argtypes = [vp, i32, c.POINTER(vp), c.POINTER(vp), i32, c.POINTER(c.c_float), c.c_float,
                                    c.POINTER(vp), vp]
        L.kt_fused_step.restype = i32
        L.kt_fused_step_noalloc.argtypes = L.kt_fused_step.argtypes
        L.kt_fused_step_noalloc.restype = i32
        for n in ("kt_plan_shares", "kt_plan_create", "kt_plan_destroy", "kt_plan_bucket_info",
                  "kt_plan_tensor_info", "kt_bucket_pack", "kt_weighted_reduce", "kt_bucket_unpack_scale",
                  "kt_plan_num_buckets", "kt_plan_num_tensors"):
            getattr(L, n).restype = i32
        _lib = L
    return _lib


def _check(status: int):
    if status != 0:
        L = lib()
        raise KtError(status, L.kt_status_string(status).decode(), L.kt_last_error().decode())


def _ptr(x) -> int:
    """Device address of a torch tensor, or an int address as is."""
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _ptr_array(items: Sequence) -> ctypes.Array:
    arr = (ctypes.c_void_p * max(1, len(items)))()
    for i, x in enumerate(items):
        arr[i] = _ptr(x)
    return arr


def _stream(stream) -> int:
    if stream is None:
        # torch's current stream on the current device, as a raw hipStream_t
        import torch
        try:
            return torch._C._cuda_getCurrentRawStream(torch._C._cuda_getDevice())
        except AttributeError:
            return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def kt_plan_shares(thr: Sequence[float], B: int, want_weights: bool = True) -> Tuple[List[int], Optional[List[float]]]:
    """Integer batch shares (and optionally the combine weights w_k = b_k/B)."""
    K = len(thr)
    t = (ctypes.c_double * max(1, K))(*[float(x) for x in thr])
    b = (ctypes.c_int64 * max(1, K))()
    w = (ctypes.c_float * max(1, K))() if want_weights else None
    _check(lib().kt_plan_shares(t, K, int(B), b, w))
    return [int(b[i]) for i in range(K)], ([float(w[i]) for i in range(K)] if want_weights else None)


def kt_replan_shares(step_time: Sequence[float], shares_used: Sequence[int], ema: Sequence[float], alpha: float,
                     B: int):
    """One online-adaptation step: (new_ema, shares, weights)."""
    K = len(step_time)
    if len(shares_used) != K or len(ema) != K:
        raise ValueError("need K entries each")
    t = (ctypes.c_double * max(1, K))(*[float(x) for x in step_time])
    u = (ctypes.c_int64 * max(1, K))(*[int(x) for x in shares_used])
    e = (ctypes.c_double * max(1, K))(*[float(x) for x in ema])
    b = (ctypes.c_int64 * max(1, K))()
    w = (ctypes.c_float * max(1, K))()
    _check(lib().kt_replan_shares(t, u, e, float(alpha), K, int(B), b, w if B > 0 else None))
    return [float(e[i]) for i in range(K)], [int(b[i]) for i in range(K)], [float(w[i]) for i in range(K)]


def kt_plan_group_weights(shares: Sequence[int], group_of: Sequence[int], G: int):
    """(w_intra[K], w_inter[G], group_batch[G]) for a two-level combination."""
    K = len(shares)
    sh = (ctypes.c_int64 * max(1, K))(*[int(x) for x in shares])
    go = (ctypes.c_int * max(1, K))(*[int(x) for x in group_of])
    w1 = (ctypes.c_float * max(1, K))()
    w2 = (ctypes.c_float * max(1, G))()
    gb = (ctypes.c_int64 * max(1, G))()
    if len(group_of) != K:
        raise ValueError("group_of needs K entries")
    _check(lib().kt_plan_group_weights(sh, K, go, int(G), w1, w2, gb))
    return [float(w1[i]) for i in range(K)], [float(w2[i]) for i in range(G)], [int(gb[i]) for i in range(G)]


def kt_sampler_epoch(N: int, B: int, shares: Sequence[int], seed: int, epoch: int, rank: int,
                     shuffle: bool = True, drop_last: bool = False) -> List[int]:
    """Dataset indices of device `rank` for one epoch."""
    K = len(shares)
    sh = (ctypes.c_int64 * max(1, K))(*[int(x) for x in shares])
    n = ctypes.c_int64()
    _check(lib().kt_sampler_epoch_size(int(N), int(B), sh, K, int(rank), int(drop_last), ctypes.byref(n)))
    out = (ctypes.c_int64 * max(1, n.value))()
    got = ctypes.c_int64()
    _check(lib().kt_sampler_epoch(int(N), int(B), sh, K, int(seed) & ((1 << 64) - 1), int(epoch), int(shuffle),
                                  int(rank), int(drop_last), out, n.value, ctypes.byref(got)))
    return list(out[:got.value])


class Plan:
    """Owner of a kt_plan handle."""

    def __init__(self, numels: Sequence[int], dtype: str, cap_bytes: int, align_bytes: int = 16):
        self.dtype = dtype
        self.numels = [int(n) for n in numels]
        T = len(self.numels)
        arr = (ctypes.c_int64 * max(1, T))(*self.numels)
        h = ctypes.c_void_p()
        _check(lib().kt_plan_create(arr, T, _DTYPES[dtype], int(cap_bytes), int(align_bytes), ctypes.byref(h)))
        self._h = h
        self._nb = lib().kt_plan_num_buckets(h)

    def close(self):
        if getattr(self, "_h", None):
            _check(lib().kt_plan_destroy(self._h))
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def num_buckets(self) -> int:
        return self._nb

    @property
    def num_tensors(self) -> int:
        return lib().kt_plan_num_tensors(self._h)

    def bucket_info(self, b: int) -> Tuple[int, int, int]:
        n, f, c = ctypes.c_int64(), ctypes.c_int(), ctypes.c_int()
        _check(lib().kt_plan_bucket_info(self._h, b, ctypes.byref(n), ctypes.byref(f), ctypes.byref(c)))
        return n.value, f.value, c.value

    def tensor_info(self, t: int) -> Tuple[int, int]:
        b, o = ctypes.c_int(), ctypes.c_int64()
        _check(lib().kt_plan_tensor_info(self._h, t, ctypes.byref(b), ctypes.byref(o)))
        return b.value, o.value

    @property
    def num_tiles(self) -> int:
        return lib().kt_plan_num_tiles(self._h)

    def tile_info(self, i: int) -> Tuple[int, int, int, int]:
        b, k, f, c = ctypes.c_int(), ctypes.c_int64(), ctypes.c_int(), ctypes.c_int()
        _check(lib().kt_plan_tile_info(self._h, i, ctypes.byref(b), ctypes.byref(k), ctypes.byref(f), ctypes.byref(c)))
        return b.value, k.value, f.value, c.value

    def bucket_elems(self) -> List[int]:
        return [self.bucket_info(b)[0] for b in range(self.num_buckets)]

    # -- device calls: marshal pointers, call, raise on error ---------------
    # The library copies whole arrays (T tensor pointers, num_buckets bucket
    # pointers, num_buckets * K peer pointers) whatever bucket is selected, so
    # every array's length is checked here before its address crosses the ABI.

    def marshal(self, items: Sequence) -> ctypes.Array:
        """Pre-marshalled pointer array (reusable across calls)."""
        return _ptr_array(items)

    def _arr(self, items, want: int, what: str):
        pre = isinstance(items, ctypes.Array)
        # marshal() pads an empty list to one (unused) entry
        if len(items) != (max(1, want) if pre else want):
            raise ValueError("%s: need %d entries (the library copies the whole array whatever bucket is "
                             "selected), got %d" % (what, want, len(items)))
        return items if pre else _ptr_array(items)

    def _weights(self, weights, K: int):
        if weights is None:         # the plan's device-resident weights (kt_plan_set_weights)
            return None
        if len(weights) != K:
            raise ValueError("need K = %d weights, got %d" % (K, len(weights)))
        if isinstance(weights, ctypes.Array):
            return weights
        return (ctypes.c_float * max(1, K))(*[float(x) for x in weights])

    def kt_plan_set_weights(self, weights, stream=None):
        """Copy the weights into the plan's device memory; device calls with weights=None read them there."""
        K = len(weights)
        w = weights if isinstance(weights, ctypes.Array) else (ctypes.c_float * max(1, K))(*[float(x) for x in weights])
        _check(lib().kt_plan_set_weights(self._h, w, K, _stream(stream)))

    def kt_bucket_pack(self, bucket: int, tensors, bucket_bufs, stream=None):
        T, nb = len(self.numels), self.num_buckets
        _check(lib().kt_bucket_pack(self._h, bucket, self._arr(tensors, T, "tensor_ptrs"),
                                    self._arr(bucket_bufs, nb, "bucket_bufs"), _stream(stream)))

    def kt_weighted_reduce(self, bucket: int, peer_bufs, K: int, weights, out_bufs, stream=None):
        """peer_bufs: flat sequence, entry [b * K + k]."""
        nb = self.num_buckets
        if not 1 <= K <= KT_MAX_PEERS:      # the library rejects K before it reads any array
            _check(lib().kt_weighted_reduce(self._h, bucket, None, K, None, None, _stream(stream)))
        _check(lib().kt_weighted_reduce(self._h, bucket, self._arr(peer_bufs, nb * K, "peer_bufs"), K,
                                        self._weights(weights, K), self._arr(out_bufs, nb, "bucket_bufs (outputs)"),
                                        _stream(stream)))

    def kt_bucket_unpack_scale(self, bucket: int, bucket_bufs, scale: float, tensors, stream=None):
        T, nb = len(self.numels), self.num_buckets
        _check(lib().kt_bucket_unpack_scale(self._h, bucket, self._arr(bucket_bufs, nb, "bucket_bufs"), float(scale),
                                            self._arr(tensors, T, "tensor_ptrs"), _stream(stream)))

    def _fused(self, fn, bucket, local_tensors, peer_bufs, K, weights, scale, out_tensors, stream):
        T, nb = len(self.numels), self.num_buckets
        if not 1 <= K <= KT_MAX_PEERS:      # the library rejects K before it reads any array
            _check(fn(self._h, bucket, None, None, K, None, float(scale), None, _stream(stream)))
        _check(fn(self._h, bucket, self._arr(local_tensors, T, "tensor_ptrs (local)"),
                  self._arr(peer_bufs, nb * (K - 1), "peer_bufs"), K, self._weights(weights, K), float(scale),
                  self._arr(out_tensors, T, "tensor_ptrs (outputs)"), _stream(stream)))

    def kt_fused_step(self, bucket: int, local_tensors, peer_bufs, K: int, weights, scale: float, out_tensors,
                      stream=None):
        """peer_bufs: flat sequence over peers 1..K-1, entry [b * (K-1) + (k-1)]."""
        self._fused(lib().kt_fused_step, bucket, local_tensors, peer_bufs, K, weights, scale, out_tensors, stream)

    def kt_fused_step_noalloc(self, bucket: int, local_tensors, peer_bufs, K: int, weights, scale: float,
                              out_tensors, stream=None):
        """kt_fused_step through the entry point that allocates nothing."""
        self._fused(lib().kt_fused_step_noalloc, bucket, local_tensors, peer_bufs, K, weights, scale, out_tensors,
                    stream)

    def kt_bucket_unpack_sgd(self, bucket: int, bucket_bufs, scale: float, params, momenta, lr: float,
                             momentum: float, weight_decay: float, first_step: bool, stream=None):
        T, nb = len(self.numels), self.num_buckets
        _check(lib().kt_bucket_unpack_sgd(self._h, bucket, self._arr(bucket_bufs, nb, "bucket_bufs"), float(scale),
                                          self._arr(params, T, "tensor_ptrs (parameters)"),
                                          self._arr(momenta, T, "tensor_ptrs (momentum)"), float(lr),
                                          float(momentum), float(weight_decay), int(bool(first_step)),
                                          _stream(stream)))

    def kt_bucket_unpack_sgd_master(self, bucket: int, bucket_bufs, scale: float, masters, momenta, models,
                                    lr: float, momentum: float, weight_decay: float, first_step: bool, stream=None):
        """Mixed precision: binary32 master parameters and momentum updated in place, bf16 model copy written."""
        T, nb = len(self.numels), self.num_buckets
        _check(lib().kt_bucket_unpack_sgd_master(self._h, bucket, self._arr(bucket_bufs, nb, "bucket_bufs"),
                                                 float(scale), self._arr(masters, T, "tensor_ptrs (master parameters)"),
                                                 self._arr(momenta, T, "tensor_ptrs (momentum)"),
                                                 self._arr(models, T, "tensor_ptrs (model parameters)"), float(lr),
                                                 float(momentum), float(weight_decay), int(bool(first_step)),
                                                 _stream(stream)))

    def kt_fused_step_sgd(self, bucket: int, local_tensors, peer_bufs, K: int, weights, scale: float, params, momenta,
                          models, lr: float, momentum: float, weight_decay: float, first_step: bool, stream=None):
        """K gradient copies -> updated parameters in one pass.  peer_bufs: flat sequence, entry
        [b * (K-1) + (k-1)] for k = 1..K-1; models=None: no bf16 model copy."""
        T, nb = len(self.numels), self.num_buckets
        if not 1 <= K <= KT_MAX_PEERS:
            _check(lib().kt_fused_step_sgd(self._h, bucket, None, None, K, None, 1.0, None, None, None, 0.0, 0.0, 0.0, 0,
                                           _stream(stream)))
        m = None if models is None else self._arr(models, T, "tensor_ptrs (model parameters)")
        _check(lib().kt_fused_step_sgd(self._h, bucket, self._arr(local_tensors, T, "tensor_ptrs (local gradients)"),
                                       self._arr(peer_bufs, nb * (K - 1), "peer_bufs"), K, self._weights(weights, K),
                                       float(scale), self._arr(params, T, "tensor_ptrs (parameters)"),
                                       self._arr(momenta, T, "tensor_ptrs (momentum)"), m, float(lr), float(momentum),
                                       float(weight_decay), int(bool(first_step)), _stream(stream)))

    def kt_fused_step_sgd_resident(self, bucket: int, local_tensors, peer_bufs, K: int, params, momenta, models,
                                   first_step: bool, stream=None):
        """kt_fused_step_sgd with the weights of kt_plan_set_weights and the scalars of kt_plan_set_sgd."""
        T, nb = len(self.numels), self.num_buckets
        if not 1 <= K <= KT_MAX_PEERS:
            _check(lib().kt_fused_step_sgd_resident(self._h, bucket, None, None, K, None, None, None, 0, _stream(stream)))
        m = None if models is None else self._arr(models, T, "tensor_ptrs (model parameters)")
        _check(lib().kt_fused_step_sgd_resident(self._h, bucket,
                                                self._arr(local_tensors, T, "tensor_ptrs (local gradients)"),
                                                self._arr(peer_bufs, nb * (K - 1), "peer_bufs"), K,
                                                self._arr(params, T, "tensor_ptrs (parameters)"),
                                                self._arr(momenta, T, "tensor_ptrs (momentum)"), m,
                                                int(bool(first_step)), _stream(stream)))

    def kt_plan_set_sgd(self, scale: float, lr: float, momentum: float, weight_decay: float, stream=None):
        """Copy the optimizer scalars into the plan's device memory (read by kt_bucket_unpack_sgd_resident)."""
        _check(lib().kt_plan_set_sgd(self._h, float(scale), float(lr), float(momentum), float(weight_decay),
                                     _stream(stream)))

    def kt_bucket_unpack_sgd_resident(self, bucket: int, bucket_bufs, params, momenta, models, first_step: bool,
                                      stream=None):
        """SGD on unpack with scale, lr, momentum and weight decay as set by kt_plan_set_sgd; models=None: no
        bf16 model copy."""
        T, nb = len(self.numels), self.num_buckets
        m = None if models is None else self._arr(models, T, "tensor_ptrs (model parameters)")
        _check(lib().kt_bucket_unpack_sgd_resident(self._h, bucket, self._arr(bucket_bufs, nb, "bucket_bufs"),
                                                   self._arr(params, T, "tensor_ptrs (parameters)"),
                                                   self._arr(momenta, T, "tensor_ptrs (momentum)"), m,
                                                   int(bool(first_step)), _stream(stream)))
