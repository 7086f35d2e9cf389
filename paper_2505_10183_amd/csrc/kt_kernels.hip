// HIP kernels for gfx950: multi-tensor pack / unpack-scale driven by a
// device-side tile + tensor-offset table, and the K-way weighted reduce.
//
// All three are streaming, zero-reuse, HBM-bound kernels.  One workgroup of
// 256 lanes (4 wavefronts) processes one tile of KT_TILE_BYTES of a bucket;
// each lane moves 16-byte vectors, several in flight before the first use.
// Nothing here is a contraction, so no MFMA.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kt_internal.h"

#ifndef KT_NT_LOAD
#define KT_NT_LOAD 1
#endif
#ifndef KT_NT_STORE
#define KT_NT_STORE 1
#endif

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int VE = 4; };
template <> struct Elem<uint16_t> { static constexpr int VE = 8; };

// Every data pointer reaches the kernels through a pointer table in memory,
// so the compiler cannot tell that it addresses global memory and would emit
// flat loads/stores.  The data is always in global memory: say so.
#define KT_GLOBAL __attribute__((address_space(1)))

__device__ __forceinline__ u32x4 ld_vec(const void *p)
{
    const KT_GLOBAL u32x4 *g = (const KT_GLOBAL u32x4 *)p;
#if KT_NT_LOAD
    return __builtin_nontemporal_load(g);
#else
    return *g;
#endif
}

__device__ __forceinline__ void st_vec(void *p, u32x4 v)
{
    KT_GLOBAL u32x4 *g = (KT_GLOBAL u32x4 *)p;
#if KT_NT_STORE
    __builtin_nontemporal_store(v, g);
#else
    *g = v;
#endif
}

template <typename T> __device__ __forceinline__ T ld_elem(const T *p) { return *(const KT_GLOBAL T *)p; }
template <typename T> __device__ __forceinline__ void st_elem(T *p, T v) { *(KT_GLOBAL T *)p = v; }

// bf16 <-> binary32.  Widening is exact (the bits become the upper half);
// narrowing is round-to-nearest-even on the bit pattern, NaN stays quiet NaN.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// scale * x for one element of either storage type
__device__ __forceinline__ float scale_elem(float x, float s) { return __fmul_rn(s, x); }
__device__ __forceinline__ uint16_t scale_elem(uint16_t x, float s)
{
    return (uint16_t)f32_to_bf16(__fmul_rn(s, __uint_as_float((uint32_t)x << 16)));
}

template <typename T> __device__ __forceinline__ u32x4 scale_vec(u32x4 v, float s);
template <> __device__ __forceinline__ u32x4 scale_vec<float>(u32x4 v, float s)
{
    u32x4 r;
#pragma unroll
    for (int c = 0; c < 4; ++c) r[c] = __float_as_uint(__fmul_rn(s, __uint_as_float(v[c])));
    return r;
}
template <> __device__ __forceinline__ u32x4 scale_vec<uint16_t>(u32x4 v, float s)
{
    u32x4 r;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        uint32_t lo = f32_to_bf16(__fmul_rn(s, bf16_lo(v[c])));
        uint32_t hi = f32_to_bf16(__fmul_rn(s, bf16_hi(v[c])));
        r[c] = lo | (hi << 16);
    }
    return r;
}

struct TileGeom {
    int bucket;
    int64_t start;   // first element of the tile inside the bucket
    int64_t end;     // one past the last element (clipped to the bucket length)
};

__device__ __forceinline__ TileGeom tile_geom(const KtTile &tl, const int64_t *b_elems, int64_t tile_elems)
{
    TileGeom g;
    g.bucket = tl.bucket;
    g.start = (int64_t)tl.tile_in_bucket * tile_elems;
    int64_t n = b_elems[tl.bucket];
    g.end = g.start + tile_elems < n ? g.start + tile_elems : n;
    return g;
}

// The tile's slice of the tensor table is staged in LDS when it fits, so that
// the per-vector owner search runs on LDS instead of global memory.
struct LdsTable {
    int64_t off[KT_LDS_TENSORS];     // element offset of the tensor in its bucket
    int64_t numel[KT_LDS_TENSORS];   // element count
    uintptr_t ptr[KT_LDS_TENSORS];   // base address (source or destination tensor)
    uintptr_t ptr2[KT_LDS_TENSORS];  // second base address for kernels with two tensor sets
};

// Typed views of the table slice of a mixed tile: in LDS (the usual case) or in
// global memory (more than KT_LDS_TENSORS tensors in one tile).  Keeping the
// address space in the type lets the owner search use LDS instructions.
#define KT_LDS __attribute__((address_space(3)))
struct LdsView {
    const KT_LDS int64_t *off;
    const KT_LDS int64_t *numel;
    const KT_LDS uintptr_t *ptr;
    const KT_LDS uintptr_t *ptr2;
};
struct GlobalView {
    const KT_GLOBAL int64_t *off;
    const KT_GLOBAL int64_t *numel;
    const KT_GLOBAL uintptr_t *ptr;
    const KT_GLOBAL uintptr_t *ptr2;
};

template <typename V> __device__ __forceinline__ int find_owner_v(const V &tv, int nt, int64_t e)
{
    int lo = 0, hi = nt;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (tv.off[mid] <= e) lo = mid + 1; else hi = mid;
    }
    return lo - 1;
}

// `second` may be NULL for kernels with one tensor set (ptr2 then mirrors ptr).
__device__ __forceinline__ LdsView stage_lds(LdsTable &lds, const KtDeviceTables &tb, const void *const *first,
                                             const void *const *second, int t0, int nt)
{
    for (int i = threadIdx.x; i < nt; i += KT_BLOCK) {
        lds.off[i] = tb.t_off[t0 + i];
        lds.numel[i] = tb.t_numel[t0 + i];
        lds.ptr[i] = reinterpret_cast<uintptr_t>(first[t0 + i]);
        lds.ptr2[i] = reinterpret_cast<uintptr_t>(second ? second[t0 + i] : first[t0 + i]);
    }
    __syncthreads();
    LdsView v;
    v.off = (const KT_LDS int64_t *)lds.off;
    v.numel = (const KT_LDS int64_t *)lds.numel;
    v.ptr = (const KT_LDS uintptr_t *)lds.ptr;
    v.ptr2 = (const KT_LDS uintptr_t *)lds.ptr2;
    return v;
}

__device__ __forceinline__ GlobalView global_view(const KtDeviceTables &tb, const void *const *first,
                                                  const void *const *second, int t0)
{
    GlobalView v;
    v.off = (const KT_GLOBAL int64_t *)(tb.t_off + t0);
    v.numel = (const KT_GLOBAL int64_t *)(tb.t_numel + t0);
    v.ptr = (const KT_GLOBAL uintptr_t *)(reinterpret_cast<const uintptr_t *>(first) + t0);
    v.ptr2 = (const KT_GLOBAL uintptr_t *)(reinterpret_cast<const uintptr_t *>(second ? second : first) + t0);
    return v;
}

// ---- pack ----------------------------------------------------------------

// One vector of a mixed tile, element by element: tensor tails, padding,
// misaligned sources, vectors straddling tensors, the last partial vector of a
// densely packed bucket.
template <typename T, typename V>
__device__ __forceinline__ void pack_slow(const V &tv, int nt, int64_t e0, int64_t b_n, T *dst)
{
    constexpr int VE = Elem<T>::VE;
    int i = find_owner_v(tv, nt, e0);
#pragma unroll 1
    for (int q = 0; q < VE; ++q) {
        const int64_t e = e0 + q;
        if (e >= b_n) break;
        while (i + 1 < nt && tv.off[i + 1] <= e) ++i;
        T x = 0;
        if (i >= 0 && e - tv.off[i] < tv.numel[i])
            x = ld_elem(reinterpret_cast<const T *>(tv.ptr[i]) + (e - tv.off[i]));
        st_elem(dst + e, x);
    }
}

// Mixed tile, 16-byte path.  Two phases so that the loads of all of a lane's
// vectors are in flight together: (1) find each vector's owner in the staged
// table and issue its load, (2) store; stragglers go element by element.
template <typename T, typename V>
__device__ __forceinline__ void pack_mixed(const V &tv, int nt, const TileGeom &g, int64_t b_n, T *dst)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int VPT = KT_TILE_VECS / KT_BLOCK;
    const int nvec = (int)((g.end - g.start + VE - 1) / VE);
    u32x4 val[VPT];
    int how[VPT];      // 0 = nothing, 1 = whole vector loaded, 2 = element-wise
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const int v = j * KT_BLOCK + threadIdx.x;
        how[j] = 0;
        if (v < nvec) {
            const int64_t e0 = g.start + (int64_t)v * VE;
            how[j] = 2;
            const int i = find_owner_v(tv, nt, e0);
            if (i >= 0 && e0 + VE <= b_n) {
                const int64_t r = e0 - tv.off[i];
                if (r + VE <= tv.numel[i]) {
                    const uintptr_t p = tv.ptr[i] + (uintptr_t)r * sizeof(T);
                    if ((p & 15u) == 0) {
                        val[j] = ld_vec(reinterpret_cast<const void *>(p));
                        how[j] = 1;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const int64_t e0 = g.start + (int64_t)(j * KT_BLOCK + threadIdx.x) * VE;
        if (how[j] == 1) st_vec(dst + e0, val[j]);
        else if (how[j] == 2) pack_slow<T>(tv, nt, e0, b_n, dst);
    }
}

// Any alignment: one element per lane per step, coalesced.
template <typename T, typename V>
__device__ __forceinline__ void pack_elems(const V &tv, int nt, const TileGeom &g, T *dst)
{
    for (int64_t e = g.start + threadIdx.x; e < g.end; e += KT_BLOCK) {
        const int i = find_owner_v(tv, nt, e);
        T x = 0;
        if (i >= 0 && e - tv.off[i] < tv.numel[i])
            x = ld_elem(reinterpret_cast<const T *>(tv.ptr[i]) + (e - tv.off[i]));
        st_elem(dst + e, x);
    }
}

template <typename T, bool VEC>
__global__ __launch_bounds__(KT_BLOCK) void kt_pack_kernel(KtDeviceTables tb, int64_t tile0,
                                                           const void *const *tensor_ptrs,
                                                           void *const *bucket_ptrs)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    constexpr int VPT = KT_TILE_VECS / KT_BLOCK;
    __shared__ LdsTable lds;

    const KtTile tl = tb.tiles[tile0 + blockIdx.x];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    T *dst = reinterpret_cast<T *>(bucket_ptrs[g.bucket]);
    const int tid = threadIdx.x;

    if (VEC && tl.nt == 0) {
        // Solid tile: one tensor owns everything; straight 16-byte copy when
        // the source address is 16-byte aligned.
        const T *src = reinterpret_cast<const T *>(tensor_ptrs[tl.t0]) + (g.start - tb.t_off[tl.t0]);
        if ((reinterpret_cast<uintptr_t>(src) & 15u) == 0) {
            const u32x4 *s4 = reinterpret_cast<const u32x4 *>(src);
            u32x4 *d4 = reinterpret_cast<u32x4 *>(dst + g.start);
            const int nvec = (int)((g.end - g.start) / VE);
            if (nvec == KT_TILE_VECS) {
                u32x4 r[VPT];
#pragma unroll
                for (int j = 0; j < VPT; ++j) r[j] = ld_vec(s4 + j * KT_BLOCK + tid);
#pragma unroll
                for (int j = 0; j < VPT; ++j) st_vec(d4 + j * KT_BLOCK + tid, r[j]);
            } else {
#pragma unroll 1
                for (int v = tid; v < nvec; v += KT_BLOCK) st_vec(d4 + v, ld_vec(s4 + v));
            }
            return;
        }
    }

    const int nt = tl.nt == 0 ? 1 : tl.nt;
    const int64_t b_n = tb.b_elems[g.bucket];
    if (nt <= KT_LDS_TENSORS) {
        const LdsView tv = stage_lds(lds, tb, tensor_ptrs, nullptr, tl.t0, nt);
        if (VEC) pack_mixed<T>(tv, nt, g, b_n, dst); else pack_elems<T>(tv, nt, g, dst);
    } else {
        const GlobalView tv = global_view(tb, tensor_ptrs, nullptr, tl.t0);
        if (VEC) pack_mixed<T>(tv, nt, g, b_n, dst); else pack_elems<T>(tv, nt, g, dst);
    }
}

// ---- unpack with scale ----------------------------------------------------

template <typename T, typename V>
__device__ __forceinline__ void unpack_slow(const V &tv, int nt, int64_t e0, int64_t b_n, const T *src, float scale)
{
    constexpr int VE = Elem<T>::VE;
    int i = find_owner_v(tv, nt, e0);
#pragma unroll 1
    for (int q = 0; q < VE; ++q) {
        const int64_t e = e0 + q;
        if (e >= b_n) break;
        while (i + 1 < nt && tv.off[i + 1] <= e) ++i;
        if (i >= 0 && e - tv.off[i] < tv.numel[i])
            st_elem(reinterpret_cast<T *>(tv.ptr[i]) + (e - tv.off[i]), scale_elem(ld_elem(src + e), scale));
    }
}

template <typename T, typename V>
__device__ __forceinline__ void unpack_mixed(const V &tv, int nt, const TileGeom &g, int64_t b_n, const T *src,
                                             float scale)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int VPT = KT_TILE_VECS / KT_BLOCK;
    const int nvec = (int)((g.end - g.start + VE - 1) / VE);
    u32x4 val[VPT];
    uintptr_t where[VPT];   // destination of a whole vector, 0 = none, 1 = element-wise
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const int v = j * KT_BLOCK + threadIdx.x;
        where[j] = 0;
        if (v < nvec) {
            const int64_t e0 = g.start + (int64_t)v * VE;
            where[j] = 1;
            const int i = find_owner_v(tv, nt, e0);
            if (i >= 0 && e0 + VE <= b_n) {
                const int64_t r = e0 - tv.off[i];
                if (r + VE <= tv.numel[i]) {
                    const uintptr_t p = tv.ptr[i] + (uintptr_t)r * sizeof(T);
                    if ((p & 15u) == 0) {
                        val[j] = ld_vec(src + e0);
                        where[j] = p;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        if (where[j] > 1) st_vec(reinterpret_cast<void *>(where[j]), scale_vec<T>(val[j], scale));
        else if (where[j] == 1)
            unpack_slow<T>(tv, nt, g.start + (int64_t)(j * KT_BLOCK + threadIdx.x) * VE, b_n, src, scale);
    }
}

template <typename T, typename V>
__device__ __forceinline__ void unpack_elems(const V &tv, int nt, const TileGeom &g, const T *src, float scale)
{
    for (int64_t e = g.start + threadIdx.x; e < g.end; e += KT_BLOCK) {
        const int i = find_owner_v(tv, nt, e);
        if (i >= 0 && e - tv.off[i] < tv.numel[i])
            st_elem(reinterpret_cast<T *>(tv.ptr[i]) + (e - tv.off[i]), scale_elem(ld_elem(src + e), scale));
    }
}

template <typename T, bool VEC>
__global__ __launch_bounds__(KT_BLOCK) void kt_unpack_kernel(KtDeviceTables tb, int64_t tile0,
                                                             const void *const *bucket_ptrs, float scale,
                                                             void *const *tensor_ptrs)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    constexpr int VPT = KT_TILE_VECS / KT_BLOCK;
    __shared__ LdsTable lds;

    const KtTile tl = tb.tiles[tile0 + blockIdx.x];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const T *src = reinterpret_cast<const T *>(bucket_ptrs[g.bucket]);
    const int tid = threadIdx.x;

    if (VEC && tl.nt == 0) {
        T *dst = reinterpret_cast<T *>(tensor_ptrs[tl.t0]) + (g.start - tb.t_off[tl.t0]);
        if ((reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
            const u32x4 *s4 = reinterpret_cast<const u32x4 *>(src + g.start);
            u32x4 *d4 = reinterpret_cast<u32x4 *>(dst);
            const int nvec = (int)((g.end - g.start) / VE);
            if (nvec == KT_TILE_VECS) {
                u32x4 r[VPT];
#pragma unroll
                for (int j = 0; j < VPT; ++j) r[j] = ld_vec(s4 + j * KT_BLOCK + tid);
#pragma unroll
                for (int j = 0; j < VPT; ++j) st_vec(d4 + j * KT_BLOCK + tid, scale_vec<T>(r[j], scale));
            } else {
#pragma unroll 1
                for (int v = tid; v < nvec; v += KT_BLOCK) st_vec(d4 + v, scale_vec<T>(ld_vec(s4 + v), scale));
            }
            return;
        }
    }

    const int nt = tl.nt == 0 ? 1 : tl.nt;
    const int64_t b_n = tb.b_elems[g.bucket];
    const void *const *tp = reinterpret_cast<const void *const *>(tensor_ptrs);
    if (nt <= KT_LDS_TENSORS) {
        const LdsView tv = stage_lds(lds, tb, tp, nullptr, tl.t0, nt);
        if (VEC) unpack_mixed<T>(tv, nt, g, b_n, src, scale); else unpack_elems<T>(tv, nt, g, src, scale);
    } else {
        const GlobalView tv = global_view(tb, tp, nullptr, tl.t0);
        if (VEC) unpack_mixed<T>(tv, nt, g, b_n, src, scale); else unpack_elems<T>(tv, nt, g, src, scale);
    }
}

// ---- K-way weighted reduce ------------------------------------------------
// Per element: acc = w0*x0 (rounded), then acc = fma(wk, xk, acc), ascending k.

template <typename T> struct Acc;
template <> struct Acc<float> {
    float a[4];
    __device__ __forceinline__ void first(u32x4 x, float w)
    {
#pragma unroll
        for (int c = 0; c < 4; ++c) a[c] = __fmul_rn(w, __uint_as_float(x[c]));
    }
    __device__ __forceinline__ void add(u32x4 x, float w)
    {
#pragma unroll
        for (int c = 0; c < 4; ++c) a[c] = __fmaf_rn(w, __uint_as_float(x[c]), a[c]);
    }
    __device__ __forceinline__ u32x4 finish() const
    {
        u32x4 r;
#pragma unroll
        for (int c = 0; c < 4; ++c) r[c] = __float_as_uint(a[c]);
        return r;
    }
};
template <> struct Acc<uint16_t> {
    float a[8];
    __device__ __forceinline__ void first(u32x4 x, float w)
    {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            a[2 * c] = __fmul_rn(w, bf16_lo(x[c]));
            a[2 * c + 1] = __fmul_rn(w, bf16_hi(x[c]));
        }
    }
    __device__ __forceinline__ void add(u32x4 x, float w)
    {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            a[2 * c] = __fmaf_rn(w, bf16_lo(x[c]), a[2 * c]);
            a[2 * c + 1] = __fmaf_rn(w, bf16_hi(x[c]), a[2 * c + 1]);
        }
    }
    __device__ __forceinline__ u32x4 finish() const
    {
        u32x4 r;
#pragma unroll
        for (int c = 0; c < 4; ++c) r[c] = f32_to_bf16(a[2 * c]) | (f32_to_bf16(a[2 * c + 1]) << 16);
        return r;
    }
};

__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }
template <typename T> __device__ __forceinline__ T narrow(float a);
template <> __device__ __forceinline__ float narrow<float>(float a) { return a; }
template <> __device__ __forceinline__ uint16_t narrow<uint16_t>(float a) { return (uint16_t)f32_to_bf16(a); }

// Vectors in flight per lane before the first use (K loads each).
template <int K> struct Unroll { static constexpr int U = KT_TILE_VECS / KT_BLOCK; };

template <typename T, int K>
__global__ __launch_bounds__(KT_BLOCK) void kt_reduce_kernel(KtDeviceTables tb, int64_t tile0,
                                                             const void *const *peer_ptrs, KtWeights wts,
                                                             void *const *out_ptrs)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    constexpr int VPT = KT_TILE_VECS / KT_BLOCK;
    constexpr int U = Unroll<K>::U;
    static_assert(VPT % U == 0, "unroll must divide vectors per lane");

    const KtTile tl = tb.tiles[tile0 + blockIdx.x];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const int tid = threadIdx.x;

    const T *x[K];
#pragma unroll
    for (int k = 0; k < K; ++k) x[k] = reinterpret_cast<const T *>(peer_ptrs[(int64_t)g.bucket * K + k]) + g.start;
    T *out = reinterpret_cast<T *>(out_ptrs[g.bucket]) + g.start;
    float w[K];
#pragma unroll
    for (int k = 0; k < K; ++k) w[k] = wts.w[k];

    const int64_t n = g.end - g.start;
    const int nvec = (int)(n / VE);

    if (nvec == KT_TILE_VECS) {
#pragma unroll 1
        for (int j = 0; j < VPT; j += U) {
            u32x4 r[U][K];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int k = 0; k < K; ++k)
                    r[u][k] = ld_vec(reinterpret_cast<const u32x4 *>(x[k]) + (j + u) * KT_BLOCK + tid);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                Acc<T> acc;
                acc.first(r[u][0], w[0]);
#pragma unroll
                for (int k = 1; k < K; ++k) acc.add(r[u][k], w[k]);
                st_vec(reinterpret_cast<u32x4 *>(out) + (j + u) * KT_BLOCK + tid, acc.finish());
            }
        }
    } else {
        for (int v = tid; v < nvec; v += KT_BLOCK) {
            u32x4 r[K];
#pragma unroll
            for (int k = 0; k < K; ++k) r[k] = ld_vec(reinterpret_cast<const u32x4 *>(x[k]) + v);
            Acc<T> acc;
            acc.first(r[0], w[0]);
#pragma unroll
            for (int k = 1; k < K; ++k) acc.add(r[k], w[k]);
            st_vec(reinterpret_cast<u32x4 *>(out) + v, acc.finish());
        }
        // tail of a densely packed bucket (fewer than VE elements)
        const int64_t e = (int64_t)nvec * VE + tid;
        if (e < n) {
            float a = __fmul_rn(w[0], widen(ld_elem(x[0] + e)));
#pragma unroll
            for (int k = 1; k < K; ++k) a = __fmaf_rn(w[k], widen(ld_elem(x[k] + e)), a);
            st_elem(out + e, narrow<T>(a));
        }
    }
}

// Any K (weights in the kernel argument block), 16-byte vectors.
template <typename T>
__global__ __launch_bounds__(KT_BLOCK) void kt_reduce_anyk_kernel(KtDeviceTables tb, int64_t tile0,
                                                                  const void *const *peer_ptrs, int K,
                                                                  KtWeights wts, void *const *out_ptrs)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    const KtTile tl = tb.tiles[tile0 + blockIdx.x];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const int tid = threadIdx.x;
    const void *const *pp = peer_ptrs + (int64_t)g.bucket * K;
    T *out = reinterpret_cast<T *>(out_ptrs[g.bucket]) + g.start;
    const int64_t n = g.end - g.start;
    const int nvec = (int)(n / VE);
    for (int v = tid; v < nvec; v += KT_BLOCK) {
        Acc<T> acc;
        acc.first(ld_vec(reinterpret_cast<const u32x4 *>(reinterpret_cast<const T *>(pp[0]) + g.start) + v), wts.w[0]);
#pragma unroll 4
        for (int k = 1; k < K; ++k)
            acc.add(ld_vec(reinterpret_cast<const u32x4 *>(reinterpret_cast<const T *>(pp[k]) + g.start) + v), wts.w[k]);
        st_vec(reinterpret_cast<u32x4 *>(out) + v, acc.finish());
    }
    const int64_t e = (int64_t)nvec * VE + tid;
    if (e < n) {
        float a = __fmul_rn(wts.w[0], widen(ld_elem(reinterpret_cast<const T *>(pp[0]) + g.start + e)));
        for (int k = 1; k < K; ++k)
            a = __fmaf_rn(wts.w[k], widen(ld_elem(reinterpret_cast<const T *>(pp[k]) + g.start + e)), a);
        st_elem(out + e, narrow<T>(a));
    }
}

// Any K, any alignment: one element per lane per step.
template <typename T>
__global__ __launch_bounds__(KT_BLOCK) void kt_reduce_elem_kernel(KtDeviceTables tb, int64_t tile0,
                                                                  const void *const *peer_ptrs, int K,
                                                                  KtWeights wts, void *const *out_ptrs)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    const KtTile tl = tb.tiles[tile0 + blockIdx.x];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const void *const *pp = peer_ptrs + (int64_t)g.bucket * K;
    T *out = reinterpret_cast<T *>(out_ptrs[g.bucket]);
    for (int64_t e = g.start + threadIdx.x; e < g.end; e += KT_BLOCK) {
        float a = __fmul_rn(wts.w[0], widen(ld_elem(reinterpret_cast<const T *>(pp[0]) + e)));
        for (int k = 1; k < K; ++k) a = __fmaf_rn(wts.w[k], widen(ld_elem(reinterpret_cast<const T *>(pp[k]) + e)), a);
        st_elem(out + e, narrow<T>(a));
    }
}

template <typename T>
hipError_t launch_reduce_t(const KtDeviceTables &tb, int64_t tile0, int64_t ntiles, const void *const *peers,
                           int K, const KtWeights &w, void *const *outs, bool vector_ok, hipStream_t s)
{
    dim3 grid((unsigned)ntiles), block(KT_BLOCK);
    if (!vector_ok) {
        kt_reduce_elem_kernel<T><<<grid, block, 0, s>>>(tb, tile0, peers, K, w, outs);
        return hipGetLastError();
    }
    switch (K) {
#define KT_CASE(KK) \
    case KK: kt_reduce_kernel<T, KK><<<grid, block, 0, s>>>(tb, tile0, peers, w, outs); break;
        KT_CASE(1) KT_CASE(2) KT_CASE(3) KT_CASE(4) KT_CASE(5) KT_CASE(6) KT_CASE(7) KT_CASE(8)
#undef KT_CASE
    default: kt_reduce_anyk_kernel<T><<<grid, block, 0, s>>>(tb, tile0, peers, K, w, outs); break;
    }
    return hipGetLastError();
}

// ---- fused single pass: tensors + peer buckets -> scaled tensors ------------
// out_t[i] = scale * round(sum_k w_k x_k), where x_0 is read straight from the
// local gradient tensor and x_1..x_{K-1} from the peer buckets.  The rounding
// sequence equals pack -> reduce -> unpack-scale (sum rounded to the storage
// type, then one multiplication), so the results are bit-identical to the
// chained path while moving (K+1) instead of (K+5) element sizes per element.

// Mixed tile of the fused pass: per vector, peer 0 comes from the owning tensor
// (tv.ptr = local gradients), the result goes to the same position of tv.ptr2.
template <typename T, int K, typename V>
__device__ __forceinline__ void fused_mixed(const V &tv, int nt, const TileGeom &g, int64_t b_n,
                                            const T *const *x, const float *w, float scale)
{
    constexpr int VE = Elem<T>::VE;
    const int nvec = (int)((g.end - g.start + VE - 1) / VE);
#pragma unroll 1
    for (int v = threadIdx.x; v < nvec; v += KT_BLOCK) {
        const int64_t e0 = g.start + (int64_t)v * VE;
        int i = find_owner_v(tv, nt, e0);
        if (i >= 0 && e0 + VE <= b_n) {
            const int64_t r = e0 - tv.off[i];
            if (r + VE <= tv.numel[i]) {
                const uintptr_t ps = tv.ptr[i] + (uintptr_t)r * sizeof(T);
                const uintptr_t pd = tv.ptr2[i] + (uintptr_t)r * sizeof(T);
                if (((ps | pd) & 15u) == 0) {
                    Acc<T> acc;
                    acc.first(ld_vec(reinterpret_cast<const void *>(ps)), w[0]);
#pragma unroll
                    for (int k = 1; k < K; ++k)
                        acc.add(ld_vec(reinterpret_cast<const u32x4 *>(x[k - 1]) + v), w[k]);
                    st_vec(reinterpret_cast<void *>(pd), scale_vec<T>(acc.finish(), scale));
                    continue;
                }
            }
        }
#pragma unroll 1
        for (int q = 0; q < VE; ++q) {
            const int64_t e = e0 + q;
            if (e >= b_n) break;
            while (i + 1 < nt && tv.off[i + 1] <= e) ++i;
            if (i >= 0 && e - tv.off[i] < tv.numel[i]) {
                const int64_t r = e - tv.off[i];
                float a = __fmul_rn(w[0], widen(ld_elem(reinterpret_cast<const T *>(tv.ptr[i]) + r)));
#pragma unroll
                for (int k = 1; k < K; ++k) a = __fmaf_rn(w[k], widen(ld_elem(x[k - 1] + (e - g.start))), a);
                st_elem(reinterpret_cast<T *>(tv.ptr2[i]) + r, scale_elem(narrow<T>(a), scale));
            }
        }
    }
}

template <typename T, int K>
__global__ __launch_bounds__(KT_BLOCK) void kt_fused_kernel(KtDeviceTables tb, int64_t tile0,
                                                            const void *const *local_ptrs,
                                                            const void *const *peer_ptrs, KtWeights wts,
                                                            float scale, void *const *out_ptrs)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    constexpr int VPT = KT_TILE_VECS / KT_BLOCK;
    constexpr int KP = K > 1 ? K - 1 : 1;
    __shared__ LdsTable lds;

    const KtTile tl = tb.tiles[tile0 + blockIdx.x];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const int tid = threadIdx.x;

    const T *x[KP];   // peers 1..K-1, already advanced to the tile start
#pragma unroll
    for (int k = 1; k < K; ++k)
        x[k - 1] = reinterpret_cast<const T *>(peer_ptrs[(int64_t)g.bucket * (K - 1) + (k - 1)]) + g.start;
    float w[K];
#pragma unroll
    for (int k = 0; k < K; ++k) w[k] = wts.w[k];

    if (tl.nt == 0) {
        const int64_t rel = g.start - tb.t_off[tl.t0];
        const T *src = reinterpret_cast<const T *>(local_ptrs[tl.t0]) + rel;
        T *dst = reinterpret_cast<T *>(out_ptrs[tl.t0]) + rel;
        if (((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) == 0) {
            const int nvec = (int)((g.end - g.start) / VE);
            if (nvec == KT_TILE_VECS) {
                u32x4 r[VPT][K];
#pragma unroll
                for (int u = 0; u < VPT; ++u) {
                    r[u][0] = ld_vec(reinterpret_cast<const u32x4 *>(src) + u * KT_BLOCK + tid);
#pragma unroll
                    for (int k = 1; k < K; ++k)
                        r[u][k] = ld_vec(reinterpret_cast<const u32x4 *>(x[k - 1]) + u * KT_BLOCK + tid);
                }
#pragma unroll
                for (int u = 0; u < VPT; ++u) {
                    Acc<T> acc;
                    acc.first(r[u][0], w[0]);
#pragma unroll
                    for (int k = 1; k < K; ++k) acc.add(r[u][k], w[k]);
                    st_vec(reinterpret_cast<u32x4 *>(dst) + u * KT_BLOCK + tid, scale_vec<T>(acc.finish(), scale));
                }
            } else {
#pragma unroll 1
                for (int v = tid; v < nvec; v += KT_BLOCK) {
                    Acc<T> acc;
                    acc.first(ld_vec(reinterpret_cast<const u32x4 *>(src) + v), w[0]);
#pragma unroll
                    for (int k = 1; k < K; ++k) acc.add(ld_vec(reinterpret_cast<const u32x4 *>(x[k - 1]) + v), w[k]);
                    st_vec(reinterpret_cast<u32x4 *>(dst) + v, scale_vec<T>(acc.finish(), scale));
                }
            }
            return;
        }
    }

    // mixed tile: stage (offset, size, source, destination) of its tensors in LDS
    const int nt = tl.nt == 0 ? 1 : tl.nt;
    const int64_t b_n = tb.b_elems[g.bucket];
    const void *const *op = reinterpret_cast<const void *const *>(out_ptrs);
    if (nt <= KT_LDS_TENSORS) {
        const LdsView tv = stage_lds(lds, tb, local_ptrs, op, tl.t0, nt);
        fused_mixed<T, K>(tv, nt, g, b_n, x, w, scale);
    } else {
        const GlobalView tv = global_view(tb, local_ptrs, op, tl.t0);
        fused_mixed<T, K>(tv, nt, g, b_n, x, w, scale);
    }
}

// Any K, any alignment: one element per lane per step.
template <typename T>
__global__ __launch_bounds__(KT_BLOCK) void kt_fused_elem_kernel(KtDeviceTables tb, int64_t tile0,
                                                                 const void *const *local_ptrs,
                                                                 const void *const *peer_ptrs, int K,
                                                                 KtWeights wts, float scale, void *const *out_ptrs)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    const KtTile tl = tb.tiles[tile0 + blockIdx.x];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const int nt = tl.nt == 0 ? 1 : tl.nt;
    const GlobalView tv = global_view(tb, local_ptrs, reinterpret_cast<const void *const *>(out_ptrs), tl.t0);
    const void *const *pp = peer_ptrs + (int64_t)g.bucket * (K - 1);
    for (int64_t e = g.start + threadIdx.x; e < g.end; e += KT_BLOCK) {
        const int i = find_owner_v(tv, nt, e);
        if (i >= 0 && e - tv.off[i] < tv.numel[i]) {
            const int64_t r = e - tv.off[i];
            float a = __fmul_rn(wts.w[0], widen(ld_elem(reinterpret_cast<const T *>(tv.ptr[i]) + r)));
            for (int k = 1; k < K; ++k)
                a = __fmaf_rn(wts.w[k], widen(ld_elem(reinterpret_cast<const T *>(pp[k - 1]) + e)), a);
            st_elem(reinterpret_cast<T *>(tv.ptr2[i]) + r, scale_elem(narrow<T>(a), scale));
        }
    }
}

template <typename T>
hipError_t launch_fused_t(const KtDeviceTables &tb, int64_t tile0, int64_t ntiles, const void *const *locals,
                          const void *const *peers, int K, const KtWeights &w, float scale, void *const *outs,
                          bool vector_ok, hipStream_t s)
{
    dim3 grid((unsigned)ntiles), block(KT_BLOCK);
    if (!vector_ok || K > 8) {
        kt_fused_elem_kernel<T><<<grid, block, 0, s>>>(tb, tile0, locals, peers, K, w, scale, outs);
        return hipGetLastError();
    }
    switch (K) {
#define KT_CASE(KK) \
    case KK: kt_fused_kernel<T, KK><<<grid, block, 0, s>>>(tb, tile0, locals, peers, w, scale, outs); break;
        KT_CASE(1) KT_CASE(2) KT_CASE(3) KT_CASE(4) KT_CASE(5) KT_CASE(6) KT_CASE(7) KT_CASE(8)
#undef KT_CASE
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ---- unpack fused with SGD (momentum, weight decay) -------------------------
// With g = scale * bucket value:  g' = fma(wd, p, g);  v' = g' on the first
// step, else fma(mu, v, g');  p' = fma(-lr, v', p).  p and v are binary32,
// updated in place; the gradient itself is never written.

__device__ __forceinline__ void sgd_elem(float x, float &p, float &v, const KtSgd &a)
{
    const float g = __fmul_rn(a.scale, x);
    const float g2 = __fmaf_rn(a.wd, p, g);
    const float vn = a.first ? g2 : __fmaf_rn(a.mu, v, g2);
    p = __fmaf_rn(-a.lr, vn, p);
    v = vn;
}

// four consecutive gradient elements
template <typename T> struct Quad;
template <> struct Quad<float> { u32x4 d; };
template <> struct Quad<uint16_t> { uint32_t d[2]; };
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ Quad<float> ld_quad(const Quad<float> *p)
{
    Quad<float> q;
    q.d = ld_vec(p);
    return q;
}
__device__ __forceinline__ Quad<uint16_t> ld_quad(const Quad<uint16_t> *p)
{
    const u32x2 t = __builtin_nontemporal_load((const KT_GLOBAL u32x2 *)p);
    Quad<uint16_t> q;
    q.d[0] = t[0];
    q.d[1] = t[1];
    return q;
}
__device__ __forceinline__ void sgd_quad(const Quad<float> &g, u32x4 &p, u32x4 &v, const KtSgd &a)
{
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        float pp = __uint_as_float(p[c]), vv = __uint_as_float(v[c]);
        sgd_elem(__uint_as_float(g.d[c]), pp, vv, a);
        p[c] = __float_as_uint(pp);
        v[c] = __float_as_uint(vv);
    }
}
__device__ __forceinline__ void sgd_quad(const Quad<uint16_t> &g, u32x4 &p, u32x4 &v, const KtSgd &a)
{
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        float p0 = __uint_as_float(p[2 * c]), v0 = __uint_as_float(v[2 * c]);
        float p1 = __uint_as_float(p[2 * c + 1]), v1 = __uint_as_float(v[2 * c + 1]);
        sgd_elem(bf16_lo(g.d[c]), p0, v0, a);
        sgd_elem(bf16_hi(g.d[c]), p1, v1, a);
        p[2 * c] = __float_as_uint(p0); v[2 * c] = __float_as_uint(v0);
        p[2 * c + 1] = __float_as_uint(p1); v[2 * c + 1] = __float_as_uint(v1);
    }
}

// one 16-byte gradient vector against its 4 (fp32) or 8 (bf16) parameters
template <typename T> struct SgdVec;
template <> struct SgdVec<float> {
    static constexpr int PV = 1;
    static __device__ __forceinline__ void apply(u32x4 g, u32x4 *p, u32x4 *v, const KtSgd &a)
    {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float pp = __uint_as_float(p[0][c]), vv = __uint_as_float(v[0][c]);
            sgd_elem(__uint_as_float(g[c]), pp, vv, a);
            p[0][c] = __float_as_uint(pp);
            v[0][c] = __float_as_uint(vv);
        }
    }
};
template <> struct SgdVec<uint16_t> {
    static constexpr int PV = 2;
    static __device__ __forceinline__ void apply(u32x4 g, u32x4 *p, u32x4 *v, const KtSgd &a)
    {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int h = c >> 1, o = (c & 1) * 2;
            float p0 = __uint_as_float(p[h][o]), v0 = __uint_as_float(v[h][o]);
            float p1 = __uint_as_float(p[h][o + 1]), v1 = __uint_as_float(v[h][o + 1]);
            sgd_elem(bf16_lo(g[c]), p0, v0, a);
            sgd_elem(bf16_hi(g[c]), p1, v1, a);
            p[h][o] = __float_as_uint(p0); v[h][o] = __float_as_uint(v0);
            p[h][o + 1] = __float_as_uint(p1); v[h][o + 1] = __float_as_uint(v1);
        }
    }
};

// Mixed tile: tv.ptr = parameters, tv.ptr2 = momentum of the owning tensor.
template <typename T, typename V>
__device__ __forceinline__ void sgd_mixed(const V &tv, int nt, const TileGeom &g, int64_t b_n, const T *src,
                                          const KtSgd &a, int vec_ok)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int PV = SgdVec<T>::PV;
    const int nvec = (int)((g.end - g.start + VE - 1) / VE);
#pragma unroll 1
    for (int v = threadIdx.x; v < nvec; v += KT_BLOCK) {
        const int64_t e0 = g.start + (int64_t)v * VE;
        int i = find_owner_v(tv, nt, e0);
        if (vec_ok && i >= 0 && e0 + VE <= b_n) {
            const int64_t r = e0 - tv.off[i];
            if (r + VE <= tv.numel[i]) {
                const uintptr_t pa = tv.ptr[i] + (uintptr_t)r * 4, va = tv.ptr2[i] + (uintptr_t)r * 4;
                if (((pa | va) & 15u) == 0) {
                    u32x4 pr[PV], vr[PV];
                    const u32x4 gr = ld_vec(src + e0);
#pragma unroll
                    for (int h = 0; h < PV; ++h) {
                        pr[h] = ld_vec(reinterpret_cast<const u32x4 *>(pa) + h);
                        vr[h] = u32x4{0, 0, 0, 0};
                        if (!a.first) vr[h] = ld_vec(reinterpret_cast<const u32x4 *>(va) + h);
                    }
                    SgdVec<T>::apply(gr, pr, vr, a);
#pragma unroll
                    for (int h = 0; h < PV; ++h) {
                        st_vec(reinterpret_cast<u32x4 *>(pa) + h, pr[h]);
                        st_vec(reinterpret_cast<u32x4 *>(va) + h, vr[h]);
                    }
                    continue;
                }
            }
        }
#pragma unroll 1
        for (int q = 0; q < VE; ++q) {
            const int64_t e = e0 + q;
            if (e >= b_n) break;
            while (i + 1 < nt && tv.off[i + 1] <= e) ++i;
            if (i >= 0 && e - tv.off[i] < tv.numel[i]) {
                const int64_t r = e - tv.off[i];
                float *pe = reinterpret_cast<float *>(tv.ptr[i]) + r;
                float *ve = reinterpret_cast<float *>(tv.ptr2[i]) + r;
                float pv = ld_elem(pe), vv = a.first ? 0.0f : ld_elem(ve);
                sgd_elem(widen(ld_elem(src + e)), pv, vv, a);
                st_elem(pe, pv);
                st_elem(ve, vv);
            }
        }
    }
}

template <typename T>
__global__ __launch_bounds__(KT_BLOCK) void kt_unpack_sgd_kernel(KtDeviceTables tb, int64_t tile0,
                                                                 const void *const *bucket_ptrs,
                                                                 void *const *param_ptrs, void *const *mom_ptrs,
                                                                 KtSgd a, int vec_ok)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    __shared__ LdsTable lds;

    const KtTile tl = tb.tiles[tile0 + blockIdx.x];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const T *src = reinterpret_cast<const T *>(bucket_ptrs[g.bucket]);
    const int tid = threadIdx.x;

    if (vec_ok && tl.nt == 0) {
        // Solid tile, processed in quads of 4 elements so that every access is
        // coalesced: 16 bytes of p and of v per lane, 16 (fp32) or 8 (bf16)
        // bytes of gradient.
        const int64_t rel = g.start - tb.t_off[tl.t0];
        float *pp = reinterpret_cast<float *>(param_ptrs[tl.t0]) + rel;
        float *vp = reinterpret_cast<float *>(mom_ptrs[tl.t0]) + rel;
        if (((reinterpret_cast<uintptr_t>(pp) | reinterpret_cast<uintptr_t>(vp)) & 15u) == 0) {
            constexpr int QPT = (int)(TILE_ELEMS / 4 / KT_BLOCK);     // quads per lane in a full tile
            const Quad<T> *s4 = reinterpret_cast<const Quad<T> *>(src + g.start);
            u32x4 *p4 = reinterpret_cast<u32x4 *>(pp);
            u32x4 *v4 = reinterpret_cast<u32x4 *>(vp);
            const int nq = (int)((g.end - g.start) / 4);
            if (nq == QPT * KT_BLOCK) {
                constexpr int QB = 4;          // quads in flight per lane
                static_assert(QPT % QB == 0, "quads per lane");
#pragma unroll 1
                for (int u0 = 0; u0 < QPT; u0 += QB) {
                    Quad<T> gr[QB];
                    u32x4 pr[QB], vr[QB];
#pragma unroll
                    for (int u = 0; u < QB; ++u) {
                        const int idx = (u0 + u) * KT_BLOCK + tid;
                        gr[u] = ld_quad(s4 + idx);
                        pr[u] = ld_vec(p4 + idx);
                        vr[u] = u32x4{0, 0, 0, 0};
                        if (!a.first) vr[u] = ld_vec(v4 + idx);
                    }
#pragma unroll
                    for (int u = 0; u < QB; ++u) {
                        const int idx = (u0 + u) * KT_BLOCK + tid;
                        sgd_quad(gr[u], pr[u], vr[u], a);
                        st_vec(p4 + idx, pr[u]);
                        st_vec(v4 + idx, vr[u]);
                    }
                }
            } else {
#pragma unroll 1
                for (int idx = tid; idx < nq; idx += KT_BLOCK) {
                    const Quad<T> gq = ld_quad(s4 + idx);
                    u32x4 pr = ld_vec(p4 + idx), vr = u32x4{0, 0, 0, 0};
                    if (!a.first) vr = ld_vec(v4 + idx);
                    sgd_quad(gq, pr, vr, a);
                    st_vec(p4 + idx, pr);
                    st_vec(v4 + idx, vr);
                }
            }
            return;
        }
    }

    const int nt = tl.nt == 0 ? 1 : tl.nt;
    const int64_t b_n = tb.b_elems[g.bucket];
    const void *const *pp = reinterpret_cast<const void *const *>(param_ptrs);
    const void *const *mp = reinterpret_cast<const void *const *>(mom_ptrs);
    if (nt <= KT_LDS_TENSORS) {
        const LdsView tv = stage_lds(lds, tb, pp, mp, tl.t0, nt);
        sgd_mixed<T>(tv, nt, g, b_n, src, a, vec_ok);
    } else {
        const GlobalView tv = global_view(tb, pp, mp, tl.t0);
        sgd_mixed<T>(tv, nt, g, b_n, src, a, vec_ok);
    }
}

}  // namespace

int kt_launch_pack(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0, int64_t ntiles,
                   const void *const *d_tensor_ptrs, void *const *d_bucket_ptrs, bool vector_ok, void *stream)
{
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    dim3 grid((unsigned)ntiles), block(KT_BLOCK);
    if (dt == KT_F32) {
        if (vector_ok) kt_pack_kernel<float, true><<<grid, block, 0, s>>>(tb, tile0, d_tensor_ptrs, d_bucket_ptrs);
        else kt_pack_kernel<float, false><<<grid, block, 0, s>>>(tb, tile0, d_tensor_ptrs, d_bucket_ptrs);
    } else {
        if (vector_ok) kt_pack_kernel<uint16_t, true><<<grid, block, 0, s>>>(tb, tile0, d_tensor_ptrs, d_bucket_ptrs);
        else kt_pack_kernel<uint16_t, false><<<grid, block, 0, s>>>(tb, tile0, d_tensor_ptrs, d_bucket_ptrs);
    }
    return (int)hipGetLastError();
}

int kt_launch_unpack(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0, int64_t ntiles,
                     const void *const *d_bucket_ptrs, float scale, void *const *d_tensor_ptrs, bool vector_ok,
                     void *stream)
{
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    dim3 grid((unsigned)ntiles), block(KT_BLOCK);
    if (dt == KT_F32) {
        if (vector_ok) kt_unpack_kernel<float, true><<<grid, block, 0, s>>>(tb, tile0, d_bucket_ptrs, scale, d_tensor_ptrs);
        else kt_unpack_kernel<float, false><<<grid, block, 0, s>>>(tb, tile0, d_bucket_ptrs, scale, d_tensor_ptrs);
    } else {
        if (vector_ok) kt_unpack_kernel<uint16_t, true><<<grid, block, 0, s>>>(tb, tile0, d_bucket_ptrs, scale, d_tensor_ptrs);
        else kt_unpack_kernel<uint16_t, false><<<grid, block, 0, s>>>(tb, tile0, d_bucket_ptrs, scale, d_tensor_ptrs);
    }
    return (int)hipGetLastError();
}

int kt_launch_reduce(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0, int64_t ntiles,
                     const void *const *d_peer_ptrs, int K, const KtWeights &w, void *const *d_out_ptrs,
                     bool vector_ok, void *stream)
{
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (dt == KT_F32) return (int)launch_reduce_t<float>(tb, tile0, ntiles, d_peer_ptrs, K, w, d_out_ptrs, vector_ok, s);
    return (int)launch_reduce_t<uint16_t>(tb, tile0, ntiles, d_peer_ptrs, K, w, d_out_ptrs, vector_ok, s);
}

int kt_launch_fused(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0, int64_t ntiles,
                    const void *const *d_local_ptrs, const void *const *d_peer_ptrs, int K, const KtWeights &w,
                    float scale, void *const *d_out_ptrs, bool vector_ok, void *stream)
{
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (dt == KT_F32)
        return (int)launch_fused_t<float>(tb, tile0, ntiles, d_local_ptrs, d_peer_ptrs, K, w, scale, d_out_ptrs, vector_ok, s);
    return (int)launch_fused_t<uint16_t>(tb, tile0, ntiles, d_local_ptrs, d_peer_ptrs, K, w, scale, d_out_ptrs, vector_ok, s);
}

int kt_launch_unpack_sgd(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0, int64_t ntiles,
                         const void *const *d_bucket_ptrs, void *const *d_param_ptrs, void *const *d_mom_ptrs,
                         const KtSgd &a, bool vector_ok, void *stream)
{
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    dim3 grid((unsigned)ntiles), block(KT_BLOCK);
    if (dt == KT_F32)
        kt_unpack_sgd_kernel<float><<<grid, block, 0, s>>>(tb, tile0, d_bucket_ptrs, d_param_ptrs, d_mom_ptrs, a, vector_ok ? 1 : 0);
    else
        kt_unpack_sgd_kernel<uint16_t><<<grid, block, 0, s>>>(tb, tile0, d_bucket_ptrs, d_param_ptrs, d_mom_ptrs, a, vector_ok ? 1 : 0);
    return (int)hipGetLastError();
}
