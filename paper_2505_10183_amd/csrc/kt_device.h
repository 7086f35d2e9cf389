// Device-side helpers shared by the kernels: 16-byte global loads/stores,
// bf16 conversion, tile geometry, the tensor-table views of mixed tiles and the
// per-element accumulation of the weighted sum.  Everything is internal to a
// translation unit (anonymous namespace).
#ifndef KT_DEVICE_H
#define KT_DEVICE_H

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
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

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
#if KT_NT_LOAD == 2
    return *(const volatile KT_GLOBAL u32x4 *)g;      // system scope (sc0 sc1), for measurement
#elif KT_NT_LOAD
    return __builtin_nontemporal_load(g);
#else
    return *g;
#endif
}

__device__ __forceinline__ void st_vec(void *p, u32x4 v)
{
    KT_GLOBAL u32x4 *g = (KT_GLOBAL u32x4 *)p;
#if KT_NT_STORE == 2
    *(volatile KT_GLOBAL u32x4 *)g = v;                // system scope (sc0 sc1), for measurement
#elif KT_NT_STORE
    __builtin_nontemporal_store(v, g);
#else
    *g = v;
#endif
}

// Store policy of the kernels that write about as much as they read (pack, unpack, SGD on
// unpack with bf16 gradients: 44-50 % of their bytes are written): a system-scope store, which
// the L2 writes through at once instead of holding the line, measured 1-4 points of 8 TB/s
// better there than the non-temporal store, and 1-3 points worse in the kernels that write a
// quarter of their bytes or less (reduce, fused pass, K copies -> parameters), which keep
// st_vec.  KT_WT_STORE=0 builds these kernels with st_vec as well, for measurement.
#ifndef KT_WT_STORE
#define KT_WT_STORE 1
#endif
template <bool WT> __device__ __forceinline__ void st_vec_copy(void *p, u32x4 v)
{
#if KT_WT_STORE && KT_NT_STORE == 1
    if (WT) {
        *(volatile KT_GLOBAL u32x4 *)p = v;
        return;
    }
#endif
    st_vec(p, v);
}

// Holds a wave back until the store window opens (KtWindow).  Bounded twice over: the clock
// always advances, so the condition comes true within one period (about 12 us), and the
// iteration count ends the loop in any case.  (The low 32 bits of the clock wrap every 43 s at
// 100 MHz; one period is then irregular.)
__device__ __forceinline__ void kt_wait_store_window(const KtWindow &w)
{
    if (w.width) {
        for (int spin = 0; spin < 4096; ++spin) {
            if ((uint32_t)wall_clock64() % w.period < w.width) break;
            __builtin_amdgcn_s_sleep(4);
        }
    }
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

// Weight of peer k: from the kernel-argument block, or, when the caller asked for
// the plan's device-resident weights, from device memory (uniform scalar reads).
// (a template parameter, so that launches with weights by value run exactly the code they
// would without this choice.)
template <bool DEVW> __device__ __forceinline__ float kt_weight(const KtWeights &wts, int k)
{
    if (DEVW) return wts.dev[k];
    return wts.w[k];
}

// ---- weighted sum of one 16-byte vector per peer ---------------------------
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

// ---- K > 8 -------------------------------------------------------------------
// The peers are taken in chunks of at most Chunk<T>::N, ascending, with the
// accumulators of the tile's vectors kept in registers across chunks, so that a
// lane still has (vectors per lane) x (chunk) loads in flight at a time and the
// per-element order of operations is the one of the definition (product for
// k = 0, then one fused multiply-add per peer in ascending k).  `ptr(k)` gives
// peer k's data at the tile start.
template <typename T> struct Chunk;
template <> struct Chunk<float> { static constexpr int N = 8; };       // 148 VGPRs, 3 waves per SIMD
template <> struct Chunk<uint16_t> { static constexpr int N = 6; };    // 8 accumulators per vector: 6 keeps 3 waves per SIMD

template <typename T, int KC, bool DEVW, typename P>
__device__ __forceinline__ void sum_chunk(Acc<T> *acc, P ptr, const KtWeights &wts, int k0, int tid)
{
    constexpr int VPT = KT_TILE_VECS / KT_BLOCK;
    u32x4 r[VPT][KC];
#pragma unroll
    for (int j = 0; j < KC; ++j) {
        const u32x4 *x = reinterpret_cast<const u32x4 *>(ptr(k0 + j));
#pragma unroll
        for (int u = 0; u < VPT; ++u) r[u][j] = ld_vec(x + u * KT_BLOCK + tid);
    }
#pragma unroll
    for (int j = 0; j < KC; ++j) {
        const float w = kt_weight<DEVW>(wts, k0 + j);
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            if (j == 0 && k0 == 0) acc[u].first(r[u][j], w); else acc[u].add(r[u][j], w);
        }
    }
}

// acc[u] = sum over all K peers of vector u of a full tile.
template <typename T, bool DEVW, typename P>
__device__ __forceinline__ void sum_in_chunks(Acc<T> *acc, P ptr, const KtWeights &wts, int K, int tid)
{
    constexpr int CH = Chunk<T>::N;
    int k0 = 0;
#pragma unroll 1
    for (; k0 + CH <= K; k0 += CH) sum_chunk<T, CH, DEVW>(acc, ptr, wts, k0, tid);
    switch (K - k0) {      // the last, shorter chunk (uniform over the grid)
    case 1: sum_chunk<T, 1, DEVW>(acc, ptr, wts, k0, tid); break;
    case 2: sum_chunk<T, 2, DEVW>(acc, ptr, wts, k0, tid); break;
    case 3: sum_chunk<T, 3, DEVW>(acc, ptr, wts, k0, tid); break;
    case 4: sum_chunk<T, 4, DEVW>(acc, ptr, wts, k0, tid); break;
    case 5: sum_chunk<T, 5, DEVW>(acc, ptr, wts, k0, tid); break;
    case 6: if (CH > 6) sum_chunk<T, 6, DEVW>(acc, ptr, wts, k0, tid); break;
    case 7: if (CH > 7) sum_chunk<T, 7, DEVW>(acc, ptr, wts, k0, tid); break;
    default: break;
    }
}

__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }
template <typename T> __device__ __forceinline__ T narrow(float a);
template <> __device__ __forceinline__ float narrow<float>(float a) { return a; }
template <> __device__ __forceinline__ uint16_t narrow<uint16_t>(float a) { return (uint16_t)f32_to_bf16(a); }

}  // namespace

#endif
