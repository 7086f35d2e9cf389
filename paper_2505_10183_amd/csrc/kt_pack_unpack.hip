// HIP kernels for gfx950: multi-tensor pack and unpack-scale driven by the device-side
// tile + tensor-offset table.  Streaming, zero-reuse, HBM-bound: workgroups of 256 lanes
// (4 wavefronts), four to a 16 KiB tile, 16-byte vectors (non-temporal loads, system-scope
// stores), all loads of a lane in flight before its first store.
#include "kt_device.h"

// The copy kernels do best with little work per workgroup (unlike the
// read-dominated reduce, which wants many loads in flight per lane): the
// 16 KiB tile of the table is shared by KT_COPY_SPLIT workgroups, each moving
// KT_TILE_VECS / KT_BLOCK / KT_COPY_SPLIT vectors per lane.  With one vector
// per lane and workgroup (the default: 4 workgroups per 16 KiB tile) pack runs
// at 84 % of 8 TB/s on 1.3 G bf16 elements against 76 % with one workgroup per tile.
#ifndef KT_COPY_SPLIT
#define KT_COPY_SPLIT (KT_TILE_VECS / KT_BLOCK)
#endif

namespace {

constexpr int COPY_SPLIT = KT_COPY_SPLIT;
constexpr int COPY_VPT = KT_TILE_VECS / KT_BLOCK / COPY_SPLIT;     // vectors per lane and workgroup
static_assert(COPY_VPT >= 1 && COPY_VPT * COPY_SPLIT * KT_BLOCK == KT_TILE_VECS, "workgroups per tile");

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
__device__ __forceinline__ void pack_mixed(const V &tv, int nt, const TileGeom &g, int64_t b_n, T *dst, int part)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int VPT = COPY_VPT;
    const int nvec = (int)((g.end - g.start + VE - 1) / VE);
    u32x4 val[VPT];
    int how[VPT];      // 0 = nothing, 1 = whole vector loaded, 2 = element-wise
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const int v = (part * VPT + j) * KT_BLOCK + threadIdx.x;
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
        const int64_t e0 = g.start + (int64_t)((part * VPT + j) * KT_BLOCK + threadIdx.x) * VE;
        if (how[j] == 1) st_vec_copy<true>(dst + e0, val[j]);
        else if (how[j] == 2) pack_slow<T>(tv, nt, e0, b_n, dst);
    }
}

// Any alignment: one element per lane per step, coalesced.
template <typename T, typename V>
__device__ __forceinline__ void pack_elems(const V &tv, int nt, const TileGeom &g, T *dst, int part)
{
    for (int64_t e = g.start + part * KT_BLOCK + threadIdx.x; e < g.end; e += COPY_SPLIT * KT_BLOCK) {
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
    constexpr int VPT = COPY_VPT;
    __shared__ LdsTable lds;

    const int part = COPY_SPLIT == 1 ? 0 : (int)(blockIdx.x % COPY_SPLIT);
    const KtTile tl = tb.tiles[tile0 + blockIdx.x / COPY_SPLIT];
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
                for (int j = 0; j < VPT; ++j) r[j] = ld_vec(s4 + (part * VPT + j) * KT_BLOCK + tid);
#pragma unroll
                for (int j = 0; j < VPT; ++j) st_vec_copy<true>(d4 + (part * VPT + j) * KT_BLOCK + tid, r[j]);
            } else {
#pragma unroll 1
                for (int v = part * KT_BLOCK + tid; v < nvec; v += COPY_SPLIT * KT_BLOCK) st_vec_copy<true>(d4 + v, ld_vec(s4 + v));
            }
            return;
        }
    }

    // a short last tile leaves the later workgroups of the tile without vectors
    if (VEC && (int64_t)part * VPT * KT_BLOCK * VE >= g.end - g.start) return;
    const int nt = tl.nt == 0 ? 1 : tl.nt;
    const int64_t b_n = tb.b_elems[g.bucket];
    if (nt <= KT_LDS_TENSORS) {
        const LdsView tv = stage_lds(lds, tb, tensor_ptrs, nullptr, tl.t0, nt);
        if (VEC) pack_mixed<T>(tv, nt, g, b_n, dst, part); else pack_elems<T>(tv, nt, g, dst, part);
    } else {
        const GlobalView tv = global_view(tb, tensor_ptrs, nullptr, tl.t0);
        if (VEC) pack_mixed<T>(tv, nt, g, b_n, dst, part); else pack_elems<T>(tv, nt, g, dst, part);
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
                                             float scale, int part)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int VPT = COPY_VPT;
    const int nvec = (int)((g.end - g.start + VE - 1) / VE);
    u32x4 val[VPT];
    uintptr_t where[VPT];   // destination of a whole vector, 0 = none, 1 = element-wise
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const int v = (part * VPT + j) * KT_BLOCK + threadIdx.x;
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
        if (where[j] > 1) st_vec_copy<true>(reinterpret_cast<void *>(where[j]), scale_vec<T>(val[j], scale));
        else if (where[j] == 1)
            unpack_slow<T>(tv, nt, g.start + (int64_t)((part * VPT + j) * KT_BLOCK + threadIdx.x) * VE, b_n, src, scale);
    }
}

template <typename T, typename V>
__device__ __forceinline__ void unpack_elems(const V &tv, int nt, const TileGeom &g, const T *src, float scale, int part)
{
    for (int64_t e = g.start + part * KT_BLOCK + threadIdx.x; e < g.end; e += COPY_SPLIT * KT_BLOCK) {
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
    constexpr int VPT = COPY_VPT;
    __shared__ LdsTable lds;

    const int part = COPY_SPLIT == 1 ? 0 : (int)(blockIdx.x % COPY_SPLIT);
    const KtTile tl = tb.tiles[tile0 + blockIdx.x / COPY_SPLIT];
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
                for (int j = 0; j < VPT; ++j) r[j] = ld_vec(s4 + (part * VPT + j) * KT_BLOCK + tid);
#pragma unroll
                for (int j = 0; j < VPT; ++j) st_vec_copy<true>(d4 + (part * VPT + j) * KT_BLOCK + tid, scale_vec<T>(r[j], scale));
            } else {
#pragma unroll 1
                for (int v = part * KT_BLOCK + tid; v < nvec; v += COPY_SPLIT * KT_BLOCK)
                    st_vec_copy<true>(d4 + v, scale_vec<T>(ld_vec(s4 + v), scale));
            }
            return;
        }
    }

    if (VEC && (int64_t)part * VPT * KT_BLOCK * VE >= g.end - g.start) return;
    const int nt = tl.nt == 0 ? 1 : tl.nt;
    const int64_t b_n = tb.b_elems[g.bucket];
    const void *const *tp = reinterpret_cast<const void *const *>(tensor_ptrs);
    if (nt <= KT_LDS_TENSORS) {
        const LdsView tv = stage_lds(lds, tb, tp, nullptr, tl.t0, nt);
        if (VEC) unpack_mixed<T>(tv, nt, g, b_n, src, scale, part); else unpack_elems<T>(tv, nt, g, src, scale, part);
    } else {
        const GlobalView tv = global_view(tb, tp, nullptr, tl.t0);
        if (VEC) unpack_mixed<T>(tv, nt, g, b_n, src, scale, part); else unpack_elems<T>(tv, nt, g, src, scale, part);
    }
}

}  // namespace

// A grid may not hold 2^32 or more lanes: very large plans go in several launches.
template <typename F> static int launch_in_chunks(int64_t tile0, int64_t ntiles, F launch)
{
    const int64_t per_launch = (((int64_t)1 << 32) / KT_BLOCK - 1) / COPY_SPLIT;
    for (int64_t done = 0; done < ntiles; done += per_launch) {
        const int64_t now = ntiles - done < per_launch ? ntiles - done : per_launch;
        launch(tile0 + done, dim3((unsigned)(now * COPY_SPLIT)));
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return (int)e;
    }
    return (int)hipSuccess;
}

int kt_launch_pack(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0, int64_t ntiles,
                   const void *const *d_tensor_ptrs, void *const *d_bucket_ptrs, bool vector_ok, void *stream)
{
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const dim3 block(KT_BLOCK);
    return launch_in_chunks(tile0, ntiles, [&](int64_t t0, dim3 grid) {
        if (dt == KT_F32) {
            if (vector_ok) kt_pack_kernel<float, true><<<grid, block, 0, s>>>(tb, t0, d_tensor_ptrs, d_bucket_ptrs);
            else kt_pack_kernel<float, false><<<grid, block, 0, s>>>(tb, t0, d_tensor_ptrs, d_bucket_ptrs);
        } else {
            if (vector_ok) kt_pack_kernel<uint16_t, true><<<grid, block, 0, s>>>(tb, t0, d_tensor_ptrs, d_bucket_ptrs);
            else kt_pack_kernel<uint16_t, false><<<grid, block, 0, s>>>(tb, t0, d_tensor_ptrs, d_bucket_ptrs);
        }
    });
}

int kt_launch_unpack(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0, int64_t ntiles,
                     const void *const *d_bucket_ptrs, float scale, void *const *d_tensor_ptrs, bool vector_ok,
                     void *stream)
{
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const dim3 block(KT_BLOCK);
    return launch_in_chunks(tile0, ntiles, [&](int64_t t0, dim3 grid) {
        if (dt == KT_F32) {
            if (vector_ok) kt_unpack_kernel<float, true><<<grid, block, 0, s>>>(tb, t0, d_bucket_ptrs, scale, d_tensor_ptrs);
            else kt_unpack_kernel<float, false><<<grid, block, 0, s>>>(tb, t0, d_bucket_ptrs, scale, d_tensor_ptrs);
        } else {
            if (vector_ok) kt_unpack_kernel<uint16_t, true><<<grid, block, 0, s>>>(tb, t0, d_bucket_ptrs, scale, d_tensor_ptrs);
            else kt_unpack_kernel<uint16_t, false><<<grid, block, 0, s>>>(tb, t0, d_bucket_ptrs, scale, d_tensor_ptrs);
        }
    });
}
