// HIP kernels for gfx950: unpack fused with SGD momentum / weight decay.
#include "kt_sgd_device.h"

namespace {

// Mixed tile: tv.ptr = parameters, tv.ptr2 = momentum of the owning tensor;
// model (MASTER only) = the bf16 model-parameter pointers of the tile's tensors,
// read from the global pointer table (mixed tiles are the rare ones).
template <typename T, bool MASTER, typename V>
__device__ __forceinline__ void sgd_mixed(const V &tv, int nt, const TileGeom &g, int64_t b_n, const T *src,
                                          const KtSgd &a, int vec_ok, int part, int parts, void *const *model)
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
                const uintptr_t pa = tv.ptr[i] + (uintptr_t)r * 4, va = tv.ptr2[i] + (uintptr_t)r * 4;
                const uintptr_t ma = MASTER ? reinterpret_cast<uintptr_t>(model[i]) + (uintptr_t)r * 2 : 0;
                if (((pa | va) & 15u) == 0 && (ma & 7u) == 0) {
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
                        st_vec_copy<sizeof(T) == 2>(reinterpret_cast<u32x4 *>(pa) + h, pr[h]);
                        st_vec_copy<sizeof(T) == 2>(reinterpret_cast<u32x4 *>(va) + h, vr[h]);
                        if (MASTER) st_model_quad<true>(reinterpret_cast<void *>(ma + 8 * h), pr[h]);
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
                if (MASTER) st_elem(reinterpret_cast<uint16_t *>(model[i]) + r, (uint16_t)f32_to_bf16(pv));
            }
        }
    }
}

// A tile of the bucket (16 KiB of gradient) goes with 16 KiB (fp32) or 32 KiB
// (bf16) each of parameters and momentum, read and written in place.  SPLIT
// workgroups share one tile; every workgroup has QB quads of 4 elements per
// lane, all loaded before the first store.  The smaller the share the better
// here, unlike in the read-dominated reduce: with one quad per lane (a
// workgroup reads 4 KiB of p and of v and writes the same 4 KiB back at once)
// the kernel runs at 79 % of 8 TB/s for either gradient type, with 2 quads
// at 75 % (bf16) and 78 % (fp32).  KT_SGD_QB overrides the default for measurement.
#ifndef KT_SGD_QB
#define KT_SGD_QB 1
#endif

template <typename T> struct SgdShape {
    static constexpr int QPT = (int)(KT_TILE_VECS * Elem<T>::VE / 4 / KT_BLOCK);   // quads per lane in a full tile
    static constexpr int QB = QPT < KT_SGD_QB ? QPT : KT_SGD_QB;                    // quads per lane and workgroup
    static constexpr int SPLIT = QPT / QB;                                          // workgroups per tile
    static_assert(QPT % QB == 0, "quads per lane");
};

// A full solid tile's share of one workgroup: QB quads per lane, every load
// issued before the first store.
template <typename T, bool MASTER>
__device__ __forceinline__ void sgd_full_tile(const T *src_tile, u32x4 *p4, u32x4 *v4, u32x2 *m2, int part,
                                              const KtSgd &a)
{
    constexpr int QB = SgdShape<T>::QB;
    const int tid = threadIdx.x;
    const Quad<T> *s4 = reinterpret_cast<const Quad<T> *>(src_tile);
    const int u0 = part * QB;
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
        st_vec_copy<sizeof(T) == 2>(p4 + idx, pr[u]);
        st_vec_copy<sizeof(T) == 2>(v4 + idx, vr[u]);
        if (MASTER) st_model_quad<true>(m2 + idx, pr[u]);
    }
}

// DEVS: the four optimizer scalars come from device memory (uniform scalar loads, issued with
// the tile-table load) instead of the kernel-argument block, so that a recorded launch follows
// a learning-rate schedule.  A separate instantiation: launches with scalars by value run the
// code they always ran.
template <typename T, bool MASTER, bool DEVS>
__global__ __launch_bounds__(KT_BLOCK) void kt_unpack_sgd_kernel(KtDeviceTables tb, int64_t tile0,
                                                                 const void *const *bucket_ptrs,
                                                                 void *const *param_ptrs, void *const *mom_ptrs,
                                                                 void *const *model_ptrs, KtSgd a, int vec_ok)
{
    if (DEVS) {
        const float *d = a.dev;
        a.scale = d[0];
        a.lr = d[1];
        a.mu = d[2];
        a.wd = d[3];
    }
    constexpr int VE = Elem<T>::VE;
    constexpr int64_t TILE_ELEMS = (int64_t)KT_TILE_VECS * VE;
    constexpr int QPT = SgdShape<T>::QPT, SPLIT = SgdShape<T>::SPLIT;
    __shared__ LdsTable lds;

    const int part = SPLIT == 1 ? 0 : (int)(blockIdx.x % SPLIT);
    const KtTile tl = tb.tiles[tile0 + blockIdx.x / SPLIT];
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
        uint16_t *mp = MASTER ? reinterpret_cast<uint16_t *>(model_ptrs[tl.t0]) + rel : nullptr;
        if (((reinterpret_cast<uintptr_t>(pp) | reinterpret_cast<uintptr_t>(vp)) & 15u) == 0 &&
            (reinterpret_cast<uintptr_t>(mp) & 7u) == 0) {
            const Quad<T> *s4 = reinterpret_cast<const Quad<T> *>(src + g.start);
            u32x4 *p4 = reinterpret_cast<u32x4 *>(pp);
            u32x4 *v4 = reinterpret_cast<u32x4 *>(vp);
            u32x2 *m2 = reinterpret_cast<u32x2 *>(mp);
            const int nq = (int)((g.end - g.start) / 4);
            if (nq == QPT * KT_BLOCK) {
                sgd_full_tile<T, MASTER>(src + g.start, p4, v4, m2, part, a);
            } else {
#pragma unroll 1
                for (int idx = part * KT_BLOCK + tid; idx < nq; idx += SPLIT * KT_BLOCK) {
                    const Quad<T> gq = ld_quad(s4 + idx);
                    u32x4 pr = ld_vec(p4 + idx), vr = u32x4{0, 0, 0, 0};
                    if (!a.first) vr = ld_vec(v4 + idx);
                    sgd_quad(gq, pr, vr, a);
                    st_vec_copy<sizeof(T) == 2>(p4 + idx, pr);
                    st_vec_copy<sizeof(T) == 2>(v4 + idx, vr);
                    if (MASTER) st_model_quad<true>(m2 + idx, pr);
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
        sgd_mixed<T, MASTER>(tv, nt, g, b_n, src, a, vec_ok, part, SPLIT, MASTER ? model_ptrs + tl.t0 : nullptr);
    } else {
        const GlobalView tv = global_view(tb, pp, mp, tl.t0);
        sgd_mixed<T, MASTER>(tv, nt, g, b_n, src, a, vec_ok, part, SPLIT, MASTER ? model_ptrs + tl.t0 : nullptr);
    }
}

}  // namespace

int kt_launch_unpack_sgd(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0, int64_t ntiles,
                         const void *const *d_bucket_ptrs, void *const *d_param_ptrs, void *const *d_mom_ptrs,
                         void *const *d_model_ptrs, const KtSgd &a, bool vector_ok, void *stream)
{
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    dim3 block(KT_BLOCK);
    const int split = dt == KT_F32 ? SgdShape<float>::SPLIT : SgdShape<uint16_t>::SPLIT;
    const int v = vector_ok ? 1 : 0;
    // a grid may not hold 2^32 or more lanes: very large plans go in several launches
    const int64_t per_launch = (((int64_t)1 << 32) / KT_BLOCK - 1) / split;
    for (int64_t done = 0; done < ntiles; done += per_launch) {
        const int64_t now = ntiles - done < per_launch ? ntiles - done : per_launch;
        const dim3 grid((unsigned)(now * split));
        const int64_t t0 = tile0 + done;
#define KT_SGD_LAUNCH(TT, MM)                                                                                        \
    do {                                                                                                            \
        if (a.dev)                                                                                                  \
            kt_unpack_sgd_kernel<TT, MM, true><<<grid, block, 0, s>>>(tb, t0, d_bucket_ptrs, d_param_ptrs, d_mom_ptrs, \
                                                                      d_model_ptrs, a, v);                         \
        else                                                                                                        \
            kt_unpack_sgd_kernel<TT, MM, false><<<grid, block, 0, s>>>(tb, t0, d_bucket_ptrs, d_param_ptrs, d_mom_ptrs, \
                                                                       d_model_ptrs, a, v);                        \
    } while (0)
        if (dt == KT_F32) {
            if (d_model_ptrs) KT_SGD_LAUNCH(float, true); else KT_SGD_LAUNCH(float, false);
        } else {
            if (d_model_ptrs) KT_SGD_LAUNCH(uint16_t, true); else KT_SGD_LAUNCH(uint16_t, false);
        }
#undef KT_SGD_LAUNCH
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return (int)e;
    }
    return (int)hipSuccess;
}
