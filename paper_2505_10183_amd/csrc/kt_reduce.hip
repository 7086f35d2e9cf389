// HIP kernels for gfx950: the K-way weighted reduce.  HBM-bound (K reads, one write per
// element); nothing here is a contraction, so no MFMA.
#include "kt_device.h"

// Occupancy the compiler must reach for the main kernel (waves per SIMD); 0 leaves it alone.
#ifndef KT_REDUCE_WAVES
#define KT_REDUCE_WAVES 0
#endif
#if KT_REDUCE_WAVES > 0
#define KT_REDUCE_OCC __attribute__((amdgpu_waves_per_eu(KT_REDUCE_WAVES, KT_REDUCE_WAVES)))
#else
#define KT_REDUCE_OCC
#endif

// Design-choice knobs of the main kernel (defaults are what measured best; the others are kept
// so that the comparison can be repeated).
//   KT_REDUCE_LAYOUT  0: vector u of lane t is u*256 + t (a workgroup's load covers 4 KiB)
//                     1: each wavefront owns 4 KiB of the tile (vector wave*256 + u*64 + lane)
//   KT_REDUCE_ISSUE   0: loads issued vector by vector, the K peers of a vector together
//                     1: peer by peer, the 4 vectors of a peer together
//   KT_REDUCE_XCD     0: tile = blockIdx.x (neighbouring tiles on different XCDs)
//                     1: each of the 8 XCDs walks its own contiguous eighth of the tiles
#ifndef KT_REDUCE_LAYOUT
#define KT_REDUCE_LAYOUT 0
#endif
#ifndef KT_REDUCE_ISSUE
#define KT_REDUCE_ISSUE 0
#endif
#ifndef KT_REDUCE_XCD
#define KT_REDUCE_XCD 0
#endif
//   KT_REDUCE_CHUNK   0: all K copies of the lane's 4 vectors in flight together
//                     c: the copies taken c at a time, accumulators kept in registers (fewer
//                        registers, more workgroups per CU, fewer loads in flight per lane)
#ifndef KT_REDUCE_CHUNK
#define KT_REDUCE_CHUNK 0
#endif
//   KT_REDUCE_LD_AUX  -1: the loads of a full tile are non-temporal global loads
//                     a >= 0: buffer loads through a descriptor of the tile (16 KiB per copy)
//                        with cache-policy bits a (1 = sc0, 2 = nt, 16 = sc1), for measurement
#ifndef KT_REDUCE_LD_AUX
#define KT_REDUCE_LD_AUX -1
#endif

namespace {

__device__ __forceinline__ int64_t reduce_tile_index()
{
#if KT_REDUCE_XCD
    // workgroups are dealt round-robin to the XCDs: blockIdx.x % 8 names the XCD
    const uint32_t x = blockIdx.x & 7u, i = blockIdx.x >> 3, q = gridDim.x >> 3, r = gridDim.x & 7u;
    return (int64_t)x * q + (x < r ? x : r) + i;
#else
    return blockIdx.x;
#endif
}

__device__ __forceinline__ int reduce_vec_index(int u, int tid)
{
#if KT_REDUCE_LAYOUT == 1
    constexpr int VPT = KT_TILE_VECS / KT_BLOCK;
    return (tid >> 6) * (VPT * 64) + u * 64 + (tid & 63);
#else
    return u * KT_BLOCK + tid;
#endif
}

template <typename T, int K, bool DEVW>
__global__ __launch_bounds__(KT_BLOCK) KT_REDUCE_OCC void kt_reduce_kernel(KtDeviceTables tb, int64_t tile0,
                                                             const void *const *peer_ptrs, KtWeights wts,
                                                             void *const *out_ptrs, KtWindow win)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    constexpr int VPT = KT_TILE_VECS / KT_BLOCK;   // vectors per lane, K loads each, all in flight at once

    const KtTile tl = tb.tiles[tile0 + reduce_tile_index()];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const int tid = threadIdx.x;

    const T *x[K];
#pragma unroll
    for (int k = 0; k < K; ++k) x[k] = reinterpret_cast<const T *>(peer_ptrs[(int64_t)g.bucket * K + k]) + g.start;
    T *out = reinterpret_cast<T *>(out_ptrs[g.bucket]) + g.start;
    float w[K];
#pragma unroll
    for (int k = 0; k < K; ++k) w[k] = kt_weight<DEVW>(wts, k);

    const int64_t n = g.end - g.start;
    const int nvec = (int)(n / VE);

#if KT_REDUCE_CHUNK > 0
    if (nvec == KT_TILE_VECS && K > KT_REDUCE_CHUNK) {
        constexpr int C = KT_REDUCE_CHUNK;
        Acc<T> acc[VPT];
#pragma unroll
        for (int k0 = 0; k0 < K; k0 += C) {
            u32x4 r[VPT][C];
#pragma unroll
            for (int u = 0; u < VPT; ++u)
#pragma unroll
                for (int j = 0; j < C; ++j)
                    if (k0 + j < K) r[u][j] = ld_vec(reinterpret_cast<const u32x4 *>(x[k0 + j < K ? k0 + j : 0]) + u * KT_BLOCK + tid);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < VPT; ++u)
#pragma unroll
                for (int j = 0; j < C; ++j)
                    if (k0 + j < K) {
                        if (k0 + j == 0) acc[u].first(r[u][j], w[0]); else acc[u].add(r[u][j], w[k0 + j < K ? k0 + j : 0]);
                    }
#pragma unroll
            for (int u = 0; u < VPT; ++u)
#pragma unroll
                for (int c = 0; c < (int)(sizeof(acc[u].a) / sizeof(float)); ++c) asm volatile("" : "+v"(acc[u].a[c]));
            __builtin_amdgcn_sched_barrier(0);
        }
        kt_wait_store_window(win);
#pragma unroll
        for (int u = 0; u < VPT; ++u) st_vec(reinterpret_cast<u32x4 *>(out) + u * KT_BLOCK + tid, acc[u].finish());
    } else
#endif
    if (nvec == KT_TILE_VECS) {
        u32x4 r[VPT][K];
#if KT_REDUCE_LD_AUX >= 0
        __amdgpu_buffer_rsrc_t rs[K];
#pragma unroll
        for (int k = 0; k < K; ++k)
            rs[k] = __builtin_amdgcn_make_buffer_rsrc(const_cast<T *>(x[k]), 0, KT_TILE_BYTES, 0x00020000);
#pragma unroll
        for (int u = 0; u < VPT; ++u)
#pragma unroll
            for (int k = 0; k < K; ++k)
                r[u][k] = __builtin_amdgcn_raw_buffer_load_b128(rs[k], reduce_vec_index(u, tid) * 16, 0, KT_REDUCE_LD_AUX);
#elif KT_REDUCE_ISSUE == 1
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
            for (int u = 0; u < VPT; ++u)
                r[u][k] = ld_vec(reinterpret_cast<const u32x4 *>(x[k]) + reduce_vec_index(u, tid));
#else
#pragma unroll
        for (int u = 0; u < VPT; ++u)
#pragma unroll
            for (int k = 0; k < K; ++k)
                r[u][k] = ld_vec(reinterpret_cast<const u32x4 *>(x[k]) + reduce_vec_index(u, tid));
#endif
        u32x4 res[VPT];
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            Acc<T> acc;
            acc.first(r[u][0], w[0]);
#pragma unroll
            for (int k = 1; k < K; ++k) acc.add(r[u][k], w[k]);
            res[u] = acc.finish();
        }
        kt_wait_store_window(win);     // large launches: the chip writes in bursts (KtWindow)
#pragma unroll
        for (int u = 0; u < VPT; ++u) st_vec(reinterpret_cast<u32x4 *>(out) + reduce_vec_index(u, tid), res[u]);
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

// K > 8: peers in chunks, accumulators in registers across chunks (sum_in_chunks).
template <typename T, bool DEVW>
__global__ __launch_bounds__(KT_BLOCK) void kt_reduce_manyk_kernel(KtDeviceTables tb, int64_t tile0,
                                                                   const void *const *peer_ptrs, int K,
                                                                   KtWeights wts, void *const *out_ptrs, KtWindow win)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    constexpr int VPT = KT_TILE_VECS / KT_BLOCK;
    const KtTile tl = tb.tiles[tile0 + blockIdx.x];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const int tid = threadIdx.x;
    const void *const *pp = peer_ptrs + (int64_t)g.bucket * K;
    T *out = reinterpret_cast<T *>(out_ptrs[g.bucket]) + g.start;
    const int64_t n = g.end - g.start;
    const int nvec = (int)(n / VE);
    if (nvec == KT_TILE_VECS) {
        Acc<T> acc[VPT];
        sum_in_chunks<T, DEVW>(acc, [&](int k) { return reinterpret_cast<const T *>(pp[k]) + g.start; }, wts, K, tid);
        u32x4 res[VPT];
#pragma unroll
        for (int u = 0; u < VPT; ++u) res[u] = acc[u].finish();
        kt_wait_store_window(win);
#pragma unroll
        for (int u = 0; u < VPT; ++u) st_vec(reinterpret_cast<u32x4 *>(out) + u * KT_BLOCK + tid, res[u]);
        return;
    }
    // the ragged last tile of a bucket: one vector at a time
    for (int v = tid; v < nvec; v += KT_BLOCK) {
        Acc<T> acc;
        acc.first(ld_vec(reinterpret_cast<const u32x4 *>(reinterpret_cast<const T *>(pp[0]) + g.start) + v), kt_weight<DEVW>(wts, 0));
#pragma unroll 4
        for (int k = 1; k < K; ++k)
            acc.add(ld_vec(reinterpret_cast<const u32x4 *>(reinterpret_cast<const T *>(pp[k]) + g.start) + v), kt_weight<DEVW>(wts, k));
        st_vec(reinterpret_cast<u32x4 *>(out) + v, acc.finish());
    }
    const int64_t e = (int64_t)nvec * VE + tid;
    if (e < n) {
        float a = __fmul_rn(kt_weight<DEVW>(wts, 0), widen(ld_elem(reinterpret_cast<const T *>(pp[0]) + g.start + e)));
        for (int k = 1; k < K; ++k)
            a = __fmaf_rn(kt_weight<DEVW>(wts, k), widen(ld_elem(reinterpret_cast<const T *>(pp[k]) + g.start + e)), a);
        st_elem(out + e, narrow<T>(a));
    }
}

// Any K, any alignment: one element per lane per step.
template <typename T, bool DEVW>
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
        float a = __fmul_rn(kt_weight<DEVW>(wts, 0), widen(ld_elem(reinterpret_cast<const T *>(pp[0]) + e)));
        for (int k = 1; k < K; ++k) a = __fmaf_rn(kt_weight<DEVW>(wts, k), widen(ld_elem(reinterpret_cast<const T *>(pp[k]) + e)), a);
        st_elem(out + e, narrow<T>(a));
    }
}

template <typename T, bool DEVW>
hipError_t launch_reduce_t(const KtDeviceTables &tb, int64_t tile0, int64_t ntiles, const void *const *peers,
                           int K, const KtWeights &w, void *const *outs, bool vector_ok, hipStream_t s)
{
    dim3 grid((unsigned)ntiles), block(KT_BLOCK);
    if (!vector_ok) {
        kt_reduce_elem_kernel<T, DEVW><<<grid, block, 0, s>>>(tb, tile0, peers, K, w, outs);
        return hipGetLastError();
    }
    const KtWindow win = kt_store_window(K, ntiles, KT_WINDOW_MIN_TILES_REDUCE);
    switch (K) {
#define KT_CASE(KK) \
    case KK: kt_reduce_kernel<T, KK, DEVW><<<grid, block, 0, s>>>(tb, tile0, peers, w, outs, win); break;
        KT_CASE(1) KT_CASE(2) KT_CASE(3) KT_CASE(4) KT_CASE(5) KT_CASE(6) KT_CASE(7) KT_CASE(8)
#undef KT_CASE
    default: kt_reduce_manyk_kernel<T, DEVW><<<grid, block, 0, s>>>(tb, tile0, peers, K, w, outs, win); break;
    }
    return hipGetLastError();
}

}  // namespace

int kt_launch_reduce(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0, int64_t ntiles,
                     const void *const *d_peer_ptrs, int K, const KtWeights &w, void *const *d_out_ptrs,
                     bool vector_ok, void *stream)
{
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    // weights by value (the usual case) and weights read from device memory are separate instantiations
    if (dt == KT_F32)
        return (int)(w.dev ? launch_reduce_t<float, true>(tb, tile0, ntiles, d_peer_ptrs, K, w, d_out_ptrs, vector_ok, s)
                           : launch_reduce_t<float, false>(tb, tile0, ntiles, d_peer_ptrs, K, w, d_out_ptrs, vector_ok, s));
    return (int)(w.dev ? launch_reduce_t<uint16_t, true>(tb, tile0, ntiles, d_peer_ptrs, K, w, d_out_ptrs, vector_ok, s)
                       : launch_reduce_t<uint16_t, false>(tb, tile0, ntiles, d_peer_ptrs, K, w, d_out_ptrs, vector_ok, s));
}
