// HIP kernels for gfx950: the single pass from K gradient copies to updated parameters
// (fused single pass + SGD momentum / weight decay in one kernel).
#include "kt_sgd_device.h"

namespace {

// ---- tensors + peer buckets -> parameters and momentum ----------------------
// Per element: r = round_T(sum_k w_k x_k) with x_0 read from the local gradient
// tensor and x_1..x_{K-1} from the peer buckets (product for k = 0, then one
// fused multiply-add per peer in ascending k, rounded to the storage type T as
// the reduce does), then the update of unpack-with-SGD on x = widen(r):
// g = scale*x; g' = fma(wd,p,g); v' = g' or fma(mu,v,g'); p' = fma(-lr,v',p).
// The results are bit-identical to pack -> reduce -> unpack-with-SGD; the
// reduced gradient is never written: (K-1)*s + s + 16 bytes per element move
// instead of (K+1)*s + s + 16.

struct FsgdArgs {
    const void *const *local_ptrs;   // T gradient tensors (peer 0)
    const void *const *peer_ptrs;    // nb * (K-1) peer buckets
    void *const *param_ptrs;         // T
    void *const *mom_ptrs;           // T
    void *const *model_ptrs;         // T, or NULL: no bf16 model copy
};

__device__ __forceinline__ KtSgd resolve_sgd(KtSgd a)
{
    if (a.dev) {        // uniform: the optimizer scalars set with kt_plan_set_sgd
        const float *d = a.dev;
        a.scale = d[0];
        a.lr = d[1];
        a.mu = d[2];
        a.wd = d[3];
    }
    return a;
}

// Second half of a full solid tile: the lane's 4 reduced vectors (storage type)
// against the tile's parameters and momentum.  binary32 gradients: a vector is
// a quad of 4 elements, so lane and vector keep their 16 bytes of p and of v.
// bf16: a vector holds 8 elements = 32 bytes of p; the tile's reduced values go
// through LDS (16 KiB) and come back in quads of 4 elements, so that every
// access to p and v is one coalesced 16 bytes per lane.
// FIRST (momentum not read) and MODEL (bf16 copy written) are compile-time here: as run-time
// conditions inside the unrolled loops they split the loads into basic blocks with a wait at
// every join, which serialises them.
template <typename T> struct TileUpdate;
template <> struct TileUpdate<float> {
    template <int VPT, bool FIRST, bool MODEL>
    static __device__ __forceinline__ void run(const u32x4 *g, u32x4 *, u32x4 *p4, u32x4 *v4, u32x2 *m2, const KtSgd &a)
    {
        const int tid = threadIdx.x;
        u32x4 pr[VPT], vr[VPT];
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            pr[u] = ld_vec(p4 + u * KT_BLOCK + tid);
            vr[u] = FIRST ? u32x4{0, 0, 0, 0} : ld_vec(v4 + u * KT_BLOCK + tid);
        }
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            Quad<float> q;
            q.d = g[u];
            sgd_quad(q, pr[u], vr[u], a);
            st_vec(p4 + u * KT_BLOCK + tid, pr[u]);
            st_vec(v4 + u * KT_BLOCK + tid, vr[u]);
            if (MODEL) st_model_quad(m2 + u * KT_BLOCK + tid, pr[u]);
        }
    }
};
template <> struct TileUpdate<uint16_t> {
    template <int VPT, bool FIRST, bool MODEL>
    static __device__ __forceinline__ void run(const u32x4 *g, u32x4 *lds, u32x4 *p4, u32x4 *v4, u32x2 *m2, const KtSgd &a)
    {
        constexpr int QPT = 2 * VPT;          // quads per lane
        const int tid = threadIdx.x;
#pragma unroll
        for (int u = 0; u < VPT; ++u) lds[u * KT_BLOCK + tid] = g[u];
        __syncthreads();
        const u32x2 *l2 = reinterpret_cast<const u32x2 *>(lds);
        u32x4 pr[QPT], vr[QPT];
        Quad<uint16_t> q[QPT];
#pragma unroll
        for (int j = 0; j < QPT; ++j) {
            const int qi = j * KT_BLOCK + tid;
            const u32x2 t = l2[qi];
            q[j].d[0] = t[0];
            q[j].d[1] = t[1];
            pr[j] = ld_vec(p4 + qi);
            vr[j] = FIRST ? u32x4{0, 0, 0, 0} : ld_vec(v4 + qi);
        }
#pragma unroll
        for (int j = 0; j < QPT; ++j) {
            const int qi = j * KT_BLOCK + tid;
            sgd_quad(q[j], pr[j], vr[j], a);
            st_vec(p4 + qi, pr[j]);
            st_vec(v4 + qi, vr[j]);
            if (MODEL) st_model_quad(m2 + qi, pr[j]);
        }
    }
};

// The update of a workgroup's share of a full solid tile (VPT reduced vectors per lane; p4, v4,
// m2 point at the share's first quad), dispatched on the two uniform conditions.
template <typename T, int VPT>
__device__ __forceinline__ void tile_update(const u32x4 *g, u32x4 *lds, u32x4 *p4, u32x4 *v4, u32x2 *m2, const KtSgd &a_in)
{
    KtSgd a = a_in;
    if (a_in.first) {
        a.first = 1;
        if (m2) TileUpdate<T>::template run<VPT, true, true>(g, lds, p4, v4, m2, a);
        else TileUpdate<T>::template run<VPT, true, false>(g, lds, p4, v4, m2, a);
    } else {
        a.first = 0;
        if (m2) TileUpdate<T>::template run<VPT, false, true>(g, lds, p4, v4, m2, a);
        else TileUpdate<T>::template run<VPT, false, false>(g, lds, p4, v4, m2, a);
    }
}

// How a 16 KiB tile is shared out: one 16-byte vector of every copy per lane and workgroup, i.e.
// 4 workgroups per tile.  With the tensors in allocations of their own (not congruent with the
// bucket's tiles) this measured best for both element types: binary32 73 % of 8 TB/s against
// 70 % for half or a whole tile per workgroup, bf16 71.6 % against 71 %.  The second half of the
// kernel writes what it reads and, like the copy kernels, wants little work per workgroup.
// KT_FSGD_VPT_F32 / KT_FSGD_VPT_BF16 override the vectors per lane and workgroup for measurement.
#ifndef KT_FSGD_VPT_F32
#define KT_FSGD_VPT_F32 1
#endif
#ifndef KT_FSGD_VPT_BF16
#define KT_FSGD_VPT_BF16 1
#endif
template <typename T> struct FsgdShape {
    static constexpr int TILE_VPT = KT_TILE_VECS / KT_BLOCK;
    static constexpr int VPT = sizeof(T) == 2 ? KT_FSGD_VPT_BF16 : KT_FSGD_VPT_F32;   // vectors per lane and workgroup
    static constexpr int SPLIT = TILE_VPT / VPT;                                      // workgroups per tile
    static constexpr int QUADS = VPT * KT_BLOCK * Elem<T>::VE / 4;                   // quads per share
    static_assert(VPT >= 1 && TILE_VPT % VPT == 0, "a tile is shared out in equal parts");
};

// Everything that is not a full, aligned solid tile: vector by vector, with a
// loop over the peers; vectors that are not wholly inside one tensor at aligned
// addresses go element by element.  tv.ptr = local gradients, tv.ptr2 =
// parameters; momentum and model pointers come from the global pointer table
// (mom, model: already advanced to the tile's first tensor).
template <typename T, bool DEVW, typename V>
__device__ __forceinline__ void fsgd_generic(const V &tv, int nt, const TileGeom &g, int64_t b_n,
                                             const void *const *pp, int K, const KtWeights &wts, const KtSgd &a,
                                             void *const *mom, void *const *model, int vec_ok, int part, int parts)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int PV = SgdVec<T>::PV;
    const int nvec = (int)((g.end - g.start + VE - 1) / VE);
#pragma unroll 1
    for (int v = part * KT_BLOCK + threadIdx.x; v < nvec; v += parts * KT_BLOCK) {
        const int64_t e0 = g.start + (int64_t)v * VE;
        int i = find_owner_v(tv, nt, e0);
        if (vec_ok && i >= 0 && e0 + VE <= b_n) {
            const int64_t r = e0 - tv.off[i];
            if (r + VE <= tv.numel[i]) {
                const uintptr_t ps = tv.ptr[i] + (uintptr_t)r * sizeof(T);
                const uintptr_t pa = tv.ptr2[i] + (uintptr_t)r * 4;
                const uintptr_t va = reinterpret_cast<uintptr_t>(mom[i]) + (uintptr_t)r * 4;
                const uintptr_t ma = model ? reinterpret_cast<uintptr_t>(model[i]) + (uintptr_t)r * 2 : 0;
                if (((ps | pa | va) & 15u) == 0 && (ma & 7u) == 0) {
                    Acc<T> acc;
                    acc.first(ld_vec(reinterpret_cast<const void *>(ps)), kt_weight<DEVW>(wts, 0));
#pragma unroll 4
                    for (int k = 1; k < K; ++k)
                        acc.add(ld_vec(reinterpret_cast<const u32x4 *>(reinterpret_cast<const T *>(pp[k - 1]) + g.start) + v),
                                kt_weight<DEVW>(wts, k));
                    u32x4 pr[PV], vr[PV];
#pragma unroll
                    for (int h = 0; h < PV; ++h) {
                        pr[h] = ld_vec(reinterpret_cast<const u32x4 *>(pa) + h);
                        vr[h] = u32x4{0, 0, 0, 0};
                        if (!a.first) vr[h] = ld_vec(reinterpret_cast<const u32x4 *>(va) + h);
                    }
                    SgdVec<T>::apply(acc.finish(), pr, vr, a);
#pragma unroll
                    for (int h = 0; h < PV; ++h) {
                        st_vec(reinterpret_cast<u32x4 *>(pa) + h, pr[h]);
                        st_vec(reinterpret_cast<u32x4 *>(va) + h, vr[h]);
                        if (model) st_model_quad(reinterpret_cast<void *>(ma + 8 * h), pr[h]);
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
                float s = __fmul_rn(kt_weight<DEVW>(wts, 0), widen(ld_elem(reinterpret_cast<const T *>(tv.ptr[i]) + r)));
                for (int k = 1; k < K; ++k)
                    s = __fmaf_rn(kt_weight<DEVW>(wts, k), widen(ld_elem(reinterpret_cast<const T *>(pp[k - 1]) + e)), s);
                float *pe = reinterpret_cast<float *>(tv.ptr2[i]) + r;
                float *ve = reinterpret_cast<float *>(mom[i]) + r;
                float pv = ld_elem(pe), vv = a.first ? 0.0f : ld_elem(ve);
                sgd_elem(widen(narrow<T>(s)), pv, vv, a);
                st_elem(pe, pv);
                st_elem(ve, vv);
                if (model) st_elem(reinterpret_cast<uint16_t *>(model[i]) + r, (uint16_t)f32_to_bf16(pv));
            }
        }
    }
}

// The pointers of a full solid tile whose tensor-side addresses allow 16-byte
// accesses (8-byte for the bf16 model copy); `ok` is uniform over the workgroup.
template <typename T> struct SolidTile {
    const T *src;
    u32x4 *p4, *v4;
    u32x2 *m2;
    bool ok;
};
template <typename T>
__device__ __forceinline__ SolidTile<T> solid_tile(const KtDeviceTables &tb, const KtTile &tl, const TileGeom &g,
                                                   const FsgdArgs &f, int vec_ok)
{
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * Elem<T>::VE;
    SolidTile<T> s;
    s.ok = false;
    if (!vec_ok || tl.nt != 0 || g.end - g.start != TILE_ELEMS) return s;
    const int64_t rel = g.start - tb.t_off[tl.t0];
    s.src = reinterpret_cast<const T *>(f.local_ptrs[tl.t0]) + rel;
    float *pp = reinterpret_cast<float *>(f.param_ptrs[tl.t0]) + rel;
    float *vp = reinterpret_cast<float *>(f.mom_ptrs[tl.t0]) + rel;
    uint16_t *mp = f.model_ptrs ? reinterpret_cast<uint16_t *>(f.model_ptrs[tl.t0]) + rel : nullptr;
    s.p4 = reinterpret_cast<u32x4 *>(pp);
    s.v4 = reinterpret_cast<u32x4 *>(vp);
    s.m2 = reinterpret_cast<u32x2 *>(mp);
    s.ok = ((reinterpret_cast<uintptr_t>(s.src) | reinterpret_cast<uintptr_t>(pp) | reinterpret_cast<uintptr_t>(vp)) & 15u) == 0 &&
           (reinterpret_cast<uintptr_t>(mp) & 7u) == 0;
    return s;
}

// LDS of a workgroup: the tensor-table slice of a mixed tile, or the reduced
// values of a full solid bf16 tile on their way from vector to quad order.
union FsgdLds {
    LdsTable table;
    u32x4 red[KT_TILE_VECS];
};

template <typename T, bool DEVW>
__device__ __forceinline__ void fsgd_other_tile(LdsTable &lds, const KtDeviceTables &tb, const KtTile &tl,
                                                const TileGeom &g, const FsgdArgs &f, const void *const *pp, int K,
                                                const KtWeights &wts, const KtSgd &a, int vec_ok, int part, int parts)
{
    const int nt = tl.nt == 0 ? 1 : tl.nt;
    const int64_t b_n = tb.b_elems[g.bucket];
    const void *const *prm = reinterpret_cast<const void *const *>(f.param_ptrs);
    void *const *mom = f.mom_ptrs + tl.t0;
    void *const *model = f.model_ptrs ? f.model_ptrs + tl.t0 : nullptr;
    if (nt <= KT_LDS_TENSORS) {
        const LdsView tv = stage_lds(lds, tb, f.local_ptrs, prm, tl.t0, nt);
        fsgd_generic<T, DEVW>(tv, nt, g, b_n, pp, K, wts, a, mom, model, vec_ok, part, parts);
    } else {
        const GlobalView tv = global_view(tb, f.local_ptrs, prm, tl.t0);
        fsgd_generic<T, DEVW>(tv, nt, g, b_n, pp, K, wts, a, mom, model, vec_ok, part, parts);
    }
}

// K = 1..8, 16-byte aligned buckets.  SPLIT workgroups share a tile; on a full solid tile each
// has VPT vectors x K copies in flight per lane, then the update of its share.
template <typename T, int K, bool DEVW>
__global__ __launch_bounds__(KT_BLOCK) void kt_fused_sgd_kernel(KtDeviceTables tb, int64_t tile0, FsgdArgs f,
                                                                KtWeights wts, KtSgd a_in)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    constexpr int VPT = FsgdShape<T>::VPT, SPLIT = FsgdShape<T>::SPLIT, QUADS = FsgdShape<T>::QUADS;
    __shared__ FsgdLds lds;

    const KtSgd a = resolve_sgd(a_in);
    const int part = SPLIT == 1 ? 0 : (int)(blockIdx.x % SPLIT);
    const KtTile tl = tb.tiles[tile0 + blockIdx.x / SPLIT];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const int tid = threadIdx.x;
    const void *const *pp = f.peer_ptrs + (int64_t)g.bucket * (K - 1);   // peers 1..K-1 of this bucket

    const SolidTile<T> st = solid_tile<T>(tb, tl, g, f, 1);
    if (st.ok) {
        const int v0 = part * VPT * KT_BLOCK + tid;     // the lane's first vector in the tile
        u32x4 r[VPT][K];
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            r[u][0] = ld_vec(reinterpret_cast<const u32x4 *>(st.src) + v0 + u * KT_BLOCK);
#pragma unroll
            for (int k = 1; k < K; ++k)
                r[u][k] = ld_vec(reinterpret_cast<const u32x4 *>(reinterpret_cast<const T *>(pp[k - 1]) + g.start) + v0 + u * KT_BLOCK);
        }
        // keep every load above the arithmetic: all of them are in flight together
        __builtin_amdgcn_sched_barrier(0);
        u32x4 red[VPT];
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            Acc<T> acc;
            acc.first(r[u][0], kt_weight<DEVW>(wts, 0));
#pragma unroll
            for (int k = 1; k < K; ++k) acc.add(r[u][k], kt_weight<DEVW>(wts, k));
            red[u] = acc.finish();
        }
        // ... and the loads of p and v below it.  The empty statements make the reduced values
        // exist at this point, so that the compiler cannot sink the arithmetic among the loads
        // of p and v (which costs a third of the occupancy: 190 VGPRs for binary32).
#pragma unroll
        for (int u = 0; u < VPT; ++u) asm volatile("" : "+v"(red[u]));
        __builtin_amdgcn_sched_barrier(0);
        tile_update<T, VPT>(red, lds.red, st.p4 + part * QUADS, st.v4 + part * QUADS,
                            st.m2 ? st.m2 + part * QUADS : nullptr, a);
        return;
    }
    fsgd_other_tile<T, DEVW>(lds.table, tb, tl, g, f, pp, K, wts, a, 1, part, SPLIT);
}

// Any K (1..64) and any alignment: full solid tiles of aligned buckets take the
// peers in chunks with the accumulators in registers; every other tile goes
// through the generic path (element by element when vec_ok == 0).
template <typename T, bool DEVW>
__global__ __launch_bounds__(KT_BLOCK) void kt_fused_sgd_any_kernel(KtDeviceTables tb, int64_t tile0, FsgdArgs f,
                                                                    int K, KtWeights wts, KtSgd a_in, int vec_ok)
{
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    constexpr int VPT = KT_TILE_VECS / KT_BLOCK;
    __shared__ FsgdLds lds;

    const KtSgd a = resolve_sgd(a_in);
    const KtTile tl = tb.tiles[tile0 + blockIdx.x];
    const TileGeom g = tile_geom(tl, tb.b_elems, TILE_ELEMS);
    const int tid = threadIdx.x;
    const void *const *pp = f.peer_ptrs + (int64_t)g.bucket * (K - 1);

    const SolidTile<T> st = solid_tile<T>(tb, tl, g, f, vec_ok);
    if (st.ok) {
        Acc<T> acc[VPT];
        sum_in_chunks<T, DEVW>(acc, [&](int k) { return k == 0 ? st.src : reinterpret_cast<const T *>(pp[k - 1]) + g.start; },
                               wts, K, tid);
        u32x4 red[VPT];
#pragma unroll
        for (int u = 0; u < VPT; ++u) red[u] = acc[u].finish();
        tile_update<T, VPT>(red, lds.red, st.p4, st.v4, st.m2, a);
        return;
    }
    fsgd_other_tile<T, DEVW>(lds.table, tb, tl, g, f, pp, K, wts, a, vec_ok, 0, 1);
}

template <typename T, bool DEVW>
hipError_t launch_fused_sgd_t(const KtDeviceTables &tb, int64_t tile0, int64_t ntiles, const FsgdArgs &f, int K,
                              const KtWeights &w, const KtSgd &a, bool vector_ok, hipStream_t s)
{
    dim3 grid((unsigned)ntiles), block(KT_BLOCK);
    if (!vector_ok || K > 8) {
        kt_fused_sgd_any_kernel<T, DEVW><<<grid, block, 0, s>>>(tb, tile0, f, K, w, a, vector_ok ? 1 : 0);
        return hipGetLastError();
    }
    // SPLIT workgroups per tile; a grid may not hold 2^32 or more lanes: very large plans go in several launches
    constexpr int SPLIT = FsgdShape<T>::SPLIT;
    const int64_t per_launch = (((int64_t)1 << 32) / KT_BLOCK - 1) / SPLIT;
    for (int64_t done = 0; done < ntiles; done += per_launch) {
        const int64_t now = ntiles - done < per_launch ? ntiles - done : per_launch;
        const dim3 g2((unsigned)(now * SPLIT));
        const int64_t t0 = tile0 + done;
        switch (K) {
#define KT_CASE(KK) \
    case KK: kt_fused_sgd_kernel<T, KK, DEVW><<<g2, block, 0, s>>>(tb, t0, f, w, a); break;
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

int kt_launch_fused_sgd(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0, int64_t ntiles,
                        const void *const *d_local_ptrs, const void *const *d_peer_ptrs, int K, const KtWeights &w,
                        void *const *d_param_ptrs, void *const *d_mom_ptrs, void *const *d_model_ptrs,
                        const KtSgd &a, bool vector_ok, void *stream)
{
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const FsgdArgs f{d_local_ptrs, d_peer_ptrs, d_param_ptrs, d_mom_ptrs, d_model_ptrs};
#define KT_FSGD(TT, DD) (int)launch_fused_sgd_t<TT, DD>(tb, tile0, ntiles, f, K, w, a, vector_ok, s)
    if (dt == KT_F32) return w.dev ? KT_FSGD(float, true) : KT_FSGD(float, false);
    return w.dev ? KT_FSGD(uint16_t, true) : KT_FSGD(uint16_t, false);
#undef KT_FSGD
}
