// Device-side helpers of the SGD update shared by the kernels that apply it
// (unpack fused with SGD; the single pass from peer copies to parameters).
#ifndef KT_SGD_DEVICE_H
#define KT_SGD_DEVICE_H

#include "kt_device.h"

namespace {

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

// Mixed precision: the four updated binary32 master values of a quad are also
// written, rounded to nearest-even, as four bf16 model parameters (8 bytes).
// SYS: system-scope store (SGD on unpack: +1-2 points of 8 TB/s), else non-temporal.
template <bool SYS = false> __device__ __forceinline__ void st_model_quad(void *m, u32x4 p)
{
    u32x2 o;
    o[0] = f32_to_bf16(__uint_as_float(p[0])) | (f32_to_bf16(__uint_as_float(p[1])) << 16);
    o[1] = f32_to_bf16(__uint_as_float(p[2])) | (f32_to_bf16(__uint_as_float(p[3])) << 16);
#if KT_WT_STORE && KT_NT_STORE == 1
    if (SYS) {
        *(volatile KT_GLOBAL u32x2 *)m = o;
        return;
    }
#endif
    __builtin_nontemporal_store(o, (KT_GLOBAL u32x2 *)m);
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

}  // namespace

#endif
