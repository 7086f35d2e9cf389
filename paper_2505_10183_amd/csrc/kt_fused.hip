// HIP kernels for gfx950: the fused single pass (pack + reduce + unpack-scale in one kernel).
#include "kt_device.h"

// Vectors per lane and workgroup on a tile (KT_TILE_VECS / KT_BLOCK = the whole tile to one
// workgroup); smaller values share the tile between several workgroups.
#ifndef KT_FUSED_VPT
#define KT_FUSED_VPT (KT_TILE_VECS / KT_BLOCK)
#endif

namespace {

constexpr int FUSED_VPT = KT_FUSED_VPT;
constexpr int FUSED_SPLIT = (KT_TILE_VECS / KT_BLOCK) / FUSED_VPT;
static_assert(FUSED_VPT >= 1 && (KT_TILE_VECS / KT_BLOCK) % FUSED_VPT == 0, "a tile is shared out in equal parts");

// ---- fused single pass: tensors + peer buckets -> scaled tensors ------------
// out_t[i] = scale * round(sum_k w_k x_k), where x_0 is read straight from the
// local gradient tensor and x_1..x_{K-1} from the peer buckets.  The rounding
// sequence equals pack -> reduce -> unpack-scale (sum rounded to the storage
// type, then one multiplication), so the results are bit-identical to the
// chained path while moving (K+1) instead of (K+5) element sizes per element.

// Mixed tile of the fused pass: per vector, peer 0 comes from the owning tensor
// (tv.ptr = local gradients), the result goes to the same position of tv.ptr2.
// Vectors are taken MB at a time per lane, in two phases, so that the loads of
// all of them are in flight together: (1) find each vector's owner in the staged
// table and issue its K loads, (2) combine and store; vectors that are not
// wholly inside one tensor at 16-byte aligned addresses go element by element.
template <typename T, int K, typename V>
__device__ __forceinline__ void fused_mixed(const V &tv, int nt, const TileGeom &g, int64_t b_n,
                                            const T *const *x, const float *w, float scale, int part)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int MB = K <= 4 ? 4 : 2;
    constexpr int STEP = FUSED_SPLIT * KT_BLOCK;      // distance between two vectors of one lane
    const int nvec = (int)((g.end - g.start + VE - 1) / VE);
#pragma unroll 1
    for (int v0 = part * KT_BLOCK + threadIdx.x; v0 < nvec; v0 += MB * STEP) {
        u32x4 r[MB][K];
        uintptr_t where[MB];      // destination of a whole vector; 0 = none, 1 = element-wise
#pragma unroll
        for (int j = 0; j < MB; ++j) {
            const int v = v0 + j * STEP;
            where[j] = 0;
            if (v < nvec) {
                where[j] = 1;
                const int64_t e0 = g.start + (int64_t)v * VE;
                const int i = find_owner_v(tv, nt, e0);
                if (i >= 0 && e0 + VE <= b_n) {
                    const int64_t rr = e0 - tv.off[i];
                    if (rr + VE <= tv.numel[i]) {
                        const uintptr_t ps = tv.ptr[i] + (uintptr_t)rr * sizeof(T);
                        const uintptr_t pd = tv.ptr2[i] + (uintptr_t)rr * sizeof(T);
                        if (((ps | pd) & 15u) == 0) {
                            r[j][0] = ld_vec(reinterpret_cast<const void *>(ps));
#pragma unroll
                            for (int k = 1; k < K; ++k) r[j][k] = ld_vec(reinterpret_cast<const u32x4 *>(x[k - 1]) + v);
                            where[j] = pd;
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int j = 0; j < MB; ++j) {
            if (where[j] > 1) {
                Acc<T> acc;
                acc.first(r[j][0], w[0]);
#pragma unroll
                for (int k = 1; k < K; ++k) acc.add(r[j][k], w[k]);
                st_vec(reinterpret_cast<void *>(where[j]), scale_vec<T>(acc.finish(), scale));
            } else if (where[j] == 1) {
                const int64_t e0 = g.start + (int64_t)(v0 + j * STEP) * VE;
                int i = find_owner_v(tv, nt, e0);
#pragma unroll 1
                for (int q = 0; q < VE; ++q) {
                    const int64_t e = e0 + q;
                    if (e >= b_n) break;
                    while (i + 1 < nt && tv.off[i + 1] <= e) ++i;
                    if (i >= 0 && e - tv.off[i] < tv.numel[i]) {
                        const int64_t rr = e - tv.off[i];
                        float a = __fmul_rn(w[0], widen(ld_elem(reinterpret_cast<const T *>(tv.ptr[i]) + rr)));
#pragma unroll
                        for (int k = 1; k < K; ++k) a = __fmaf_rn(w[k], widen(ld_elem(x[k - 1] + (e - g.start))), a);
                        st_elem(reinterpret_cast<T *>(tv.ptr2[i]) + rr, scale_elem(narrow<T>(a), scale));
                    }
                }
            }
        }
    }
}

template <typename T, int K, bool DEVW>
__global__ __launch_bounds__(KT_BLOCK) void kt_fused_kernel(KtDeviceTables tb, int64_t tile0,
                                                            const void *const *local_ptrs,
                                                            const void *const *peer_ptrs, KtWeights wts,
                                                            float scale, void *const *out_ptrs, KtWindow win)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    constexpr int VPT = FUSED_VPT, SPLIT = FUSED_SPLIT;
    constexpr int KP = K > 1 ? K - 1 : 1;
    __shared__ LdsTable lds;

    const int part = SPLIT == 1 ? 0 : (int)(blockIdx.x % SPLIT);
    const KtTile tl = tb.tiles[tile0 + blockIdx.x / SPLIT];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const int tid = threadIdx.x;

    const T *x[KP];   // peers 1..K-1, already advanced to the tile start
#pragma unroll
    for (int k = 1; k < K; ++k)
        x[k - 1] = reinterpret_cast<const T *>(peer_ptrs[(int64_t)g.bucket * (K - 1) + (k - 1)]) + g.start;
    float w[K];
#pragma unroll
    for (int k = 0; k < K; ++k) w[k] = kt_weight<DEVW>(wts, k);

    if (tl.nt == 0) {
        const int64_t rel = g.start - tb.t_off[tl.t0];
        const T *src = reinterpret_cast<const T *>(local_ptrs[tl.t0]) + rel;
        T *dst = reinterpret_cast<T *>(out_ptrs[tl.t0]) + rel;
        if (((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) == 0) {
            const int nvec = (int)((g.end - g.start) / VE);
            if (nvec == KT_TILE_VECS) {
                const int v0 = part * VPT * KT_BLOCK + tid;     // the lane's first vector in the tile
                u32x4 r[VPT][K];
#pragma unroll
                for (int u = 0; u < VPT; ++u) {
                    r[u][0] = ld_vec(reinterpret_cast<const u32x4 *>(src) + v0 + u * KT_BLOCK);
#pragma unroll
                    for (int k = 1; k < K; ++k)
                        r[u][k] = ld_vec(reinterpret_cast<const u32x4 *>(x[k - 1]) + v0 + u * KT_BLOCK);
                }
                u32x4 res[VPT];
#pragma unroll
                for (int u = 0; u < VPT; ++u) {
                    Acc<T> acc;
                    acc.first(r[u][0], w[0]);
#pragma unroll
                    for (int k = 1; k < K; ++k) acc.add(r[u][k], w[k]);
                    res[u] = scale_vec<T>(acc.finish(), scale);
                }
                kt_wait_store_window(win);     // large launches: the chip writes in bursts (KtWindow)
#pragma unroll
                for (int u = 0; u < VPT; ++u) st_vec(reinterpret_cast<u32x4 *>(dst) + v0 + u * KT_BLOCK, res[u]);
            } else {
#pragma unroll 1
                for (int v = part * KT_BLOCK + tid; v < nvec; v += SPLIT * KT_BLOCK) {
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
        fused_mixed<T, K>(tv, nt, g, b_n, x, w, scale, part);
    } else {
        const GlobalView tv = global_view(tb, local_ptrs, op, tl.t0);
        fused_mixed<T, K>(tv, nt, g, b_n, x, w, scale, part);
    }
}

// K > 8, 16-byte vectors: full solid tiles take the peers in chunks with the
// accumulators in registers (sum_in_chunks; peer 0 is the local tensor); every
// other tile goes vector by vector with a loop over the peers.
template <typename T, bool DEVW, typename V>
__device__ __forceinline__ void fused_mixed_manyk(const V &tv, int nt, const TileGeom &g, int64_t b_n,
                                                  const void *const *pp, int K, const KtWeights &wts, float scale)
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
                    acc.first(ld_vec(reinterpret_cast<const void *>(ps)), kt_weight<DEVW>(wts, 0));
#pragma unroll 4
                    for (int k = 1; k < K; ++k)
                        acc.add(ld_vec(reinterpret_cast<const u32x4 *>(reinterpret_cast<const T *>(pp[k - 1]) + g.start) + v), kt_weight<DEVW>(wts, k));
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
                float a = __fmul_rn(kt_weight<DEVW>(wts, 0), widen(ld_elem(reinterpret_cast<const T *>(tv.ptr[i]) + r)));
                for (int k = 1; k < K; ++k) a = __fmaf_rn(kt_weight<DEVW>(wts, k), widen(ld_elem(reinterpret_cast<const T *>(pp[k - 1]) + e)), a);
                st_elem(reinterpret_cast<T *>(tv.ptr2[i]) + r, scale_elem(narrow<T>(a), scale));
            }
        }
    }
}

template <typename T, bool DEVW>
__global__ __launch_bounds__(KT_BLOCK) void kt_fused_manyk_kernel(KtDeviceTables tb, int64_t tile0,
                                                                  const void *const *local_ptrs,
                                                                  const void *const *peer_ptrs, int K,
                                                                  KtWeights wts, float scale, void *const *out_ptrs,
                                                                  KtWindow win)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    constexpr int VPT = KT_TILE_VECS / KT_BLOCK;
    __shared__ LdsTable lds;

    const KtTile tl = tb.tiles[tile0 + blockIdx.x];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const int tid = threadIdx.x;
    const void *const *pp = peer_ptrs + (int64_t)g.bucket * (K - 1);   // peers 1..K-1 of this bucket

    if (tl.nt == 0 && g.end - g.start == TILE_ELEMS) {
        const int64_t rel = g.start - tb.t_off[tl.t0];
        const T *src = reinterpret_cast<const T *>(local_ptrs[tl.t0]) + rel;
        T *dst = reinterpret_cast<T *>(out_ptrs[tl.t0]) + rel;
        if (((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) == 0) {
            Acc<T> acc[VPT];
            sum_in_chunks<T, DEVW>(acc, [&](int k) { return k == 0 ? src : reinterpret_cast<const T *>(pp[k - 1]) + g.start; },
                             wts, K, tid);
            u32x4 res[VPT];
#pragma unroll
            for (int u = 0; u < VPT; ++u) res[u] = scale_vec<T>(acc[u].finish(), scale);
            kt_wait_store_window(win);
#pragma unroll
            for (int u = 0; u < VPT; ++u) st_vec(reinterpret_cast<u32x4 *>(dst) + u * KT_BLOCK + tid, res[u]);
            return;
        }
    }
    const int nt = tl.nt == 0 ? 1 : tl.nt;
    const int64_t b_n = tb.b_elems[g.bucket];
    const void *const *op = reinterpret_cast<const void *const *>(out_ptrs);
    if (nt <= KT_LDS_TENSORS) {
        const LdsView tv = stage_lds(lds, tb, local_ptrs, op, tl.t0, nt);
        fused_mixed_manyk<T, DEVW>(tv, nt, g, b_n, pp, K, wts, scale);
    } else {
        const GlobalView tv = global_view(tb, local_ptrs, op, tl.t0);
        fused_mixed_manyk<T, DEVW>(tv, nt, g, b_n, pp, K, wts, scale);
    }
}

// Any K, any alignment: one element per lane per step.
template <typename T, bool DEVW>
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
            float a = __fmul_rn(kt_weight<DEVW>(wts, 0), widen(ld_elem(reinterpret_cast<const T *>(tv.ptr[i]) + r)));
            for (int k = 1; k < K; ++k)
                a = __fmaf_rn(kt_weight<DEVW>(wts, k), widen(ld_elem(reinterpret_cast<const T *>(pp[k - 1]) + e)), a);
            st_elem(reinterpret_cast<T *>(tv.ptr2[i]) + r, scale_elem(narrow<T>(a), scale));
        }
    }
}

template <typename T, bool DEVW>
hipError_t launch_fused_t(const KtDeviceTables &tb, int64_t tile0, int64_t ntiles, const void *const *locals,
                          const void *const *peers, int K, const KtWeights &w, float scale, void *const *outs,
                          bool vector_ok, hipStream_t s)
{
    dim3 grid((unsigned)ntiles), block(KT_BLOCK);
    if (!vector_ok) {
        kt_fused_elem_kernel<T, DEVW><<<grid, block, 0, s>>>(tb, tile0, locals, peers, K, w, scale, outs);
        return hipGetLastError();
    }
    // the window assumes one workgroup per tile (the time a generation of workgroups reads for)
    const KtWindow win = FUSED_SPLIT == 1 ? kt_store_window(K, ntiles, KT_WINDOW_MIN_TILES_FUSED) : KtWindow{0, 0};
    if (K > 8) {
        kt_fused_manyk_kernel<T, DEVW><<<grid, block, 0, s>>>(tb, tile0, locals, peers, K, w, scale, outs, win);
        return hipGetLastError();
    }
    // FUSED_SPLIT workgroups per tile; a grid may not hold 2^32 or more lanes: very large plans go in several launches
    const int64_t per_launch = (((int64_t)1 << 32) / KT_BLOCK - 1) / FUSED_SPLIT;
    for (int64_t done = 0; done < ntiles; done += per_launch) {
        const int64_t now = ntiles - done < per_launch ? ntiles - done : per_launch;
        const dim3 g2((unsigned)(now * FUSED_SPLIT));
        const int64_t t0 = tile0 + done;
        switch (K) {
#define KT_CASE(KK) \
    case KK: kt_fused_kernel<T, KK, DEVW><<<g2, block, 0, s>>>(tb, t0, locals, peers, w, scale, outs, win); break;
            KT_CASE(1) KT_CASE(2) KT_CASE(3) KT_CASE(4) KT_CASE(5) KT_CASE(6) KT_CASE(7) KT_CASE(8)
#undef KT_CASE
        default: return hipErrorInvalidValue;
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

int kt_launch_fused(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0, int64_t ntiles,
                    const void *const *d_local_ptrs, const void *const *d_peer_ptrs, int K, const KtWeights &w,
                    float scale, void *const *d_out_ptrs, bool vector_ok, void *stream)
{
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
#define KT_FUSED(TT, DD) \
    (int)launch_fused_t<TT, DD>(tb, tile0, ntiles, d_local_ptrs, d_peer_ptrs, K, w, scale, d_out_ptrs, vector_ok, s)
    if (dt == KT_F32) return w.dev ? KT_FUSED(float, true) : KT_FUSED(float, false);
    return w.dev ? KT_FUSED(uint16_t, true) : KT_FUSED(uint16_t, false);
#undef KT_FUSED
}
