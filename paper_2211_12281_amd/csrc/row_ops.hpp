// Row-wise device helpers shared by the preparation kernels and the ranking kernels: element
// access for fp32 / bf16 tables, wave reductions, and the query build of Table 2
// (q = h + r, h o r, h * r (complex), h o e^{ir}, or the TransH projection of h plus r).
#pragma once
#include "prep_kernels.h"

template <bool BF16> struct El;
template <> struct El<true> {
    using T = __bf16;
    static __device__ __forceinline__ float ld(const void *p, int64_t i) { return (float)((const __bf16 *)p)[i]; }
    static __device__ __forceinline__ void st(void *p, int64_t i, float v) { ((__bf16 *)p)[i] = (__bf16)v; }
    static __device__ __forceinline__ float rnd(float v) { return (float)(__bf16)v; }
};
template <> struct El<false> {
    using T = float;
    static __device__ __forceinline__ float ld(const void *p, int64_t i) { return ((const float *)p)[i]; }
    static __device__ __forceinline__ void st(void *p, int64_t i, float v) { ((float *)p)[i] = v; }
    static __device__ __forceinline__ float rnd(float v) { return v; }
};

__device__ __forceinline__ float kge_wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ float kge_wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

constexpr int KGE_MAXJ = 8;   // dim <= 512 -> at most 8 columns per lane

// The query of triple b (fp32, unrounded), spread over a wave: lane holds columns lane + 64*k.
// Returns through references what the callers need besides q.
template <bool BF16>
struct KgeRowCtx {
    float h[KGE_MAXJ], r[KGE_MAXJ], w[KGE_MAXJ], q[KGE_MAXJ];
    float wh;      // w_hat . h     (TransH)
    float wnorm;   // ||w|| clamped (TransH)
};

// Builds q for one triple.  For complex scorers lane column j < d/2 pairs with j + d/2, which is a
// different lane/slot in general, so partner values are fetched from memory again (L1/L2 hits).
// SC >= 0 fixes the scorer at compile time (straight-line code: the loads of a row are issued together).
template <bool BF16, int SC = -1>
__device__ __forceinline__ void kge_build_query(const KgeModelDev &m, int hi, int ri, int lane,
                                                KgeRowCtx<BF16> &cx) {
    const int d = m.dim, c = d >> 1;
    const int64_t hoff = (int64_t)hi * m.ent_ld, roff = (int64_t)ri * m.rel_ld, woff = (int64_t)ri * m.relw_ld;
    float wn2 = 0.f, whp = 0.f;
    // Branch-free: lanes past the row read column 0 instead and are zeroed afterwards, so that all loads of the row
    // are issued together rather than one branch (and one wait) at a time.
#pragma unroll
    for (int k = 0; k < KGE_MAXJ; ++k) {
        const int j = lane + 64 * k;
        const bool ok = j < d;
        const int js = ok ? j : 0;
        const bool lo = js < c;
        const int jp = lo ? js + c : js - c;              // partner component of a complex coordinate
        const float hj = El<BF16>::ld(m.ent, hoff + js);
        float rj = 0.f, wj = 0.f, qj = 0.f;
        switch (SC >= 0 ? SC : m.scorer) {
        case KGE_TRANSE: rj = El<BF16>::ld(m.rel, roff + js); qj = hj + rj; break;
        case KGE_DISTMULT: rj = El<BF16>::ld(m.rel, roff + js); qj = hj * rj; break;
        case KGE_COMPLEX: {
            rj = El<BF16>::ld(m.rel, roff + js);
            const float hp = El<BF16>::ld(m.ent, hoff + jp), rp = El<BF16>::ld(m.rel, roff + jp);
            // q_re = h_re r_re - h_im r_im,  q_im = h_re r_im + h_im r_re
            qj = lo ? hj * rj - hp * rp : hp * rj + hj * rp;
            break;
        }
        case KGE_ROTATE: {
            rj = El<BF16>::ld(m.rel, roff + (lo ? js : js - c));
            const float hp = El<BF16>::ld(m.ent, hoff + jp);
            float sn, cs; sincosf(rj, &sn, &cs);
            qj = lo ? hj * cs - hp * sn : hp * sn + hj * cs;
            break;
        }
        case KGE_TRANSH:
            rj = El<BF16>::ld(m.rel, roff + js); wj = ok ? El<BF16>::ld(m.relw, woff + js) : 0.f;
            wn2 += wj * wj; whp += ok ? wj * hj : 0.f;
            break;
        }
        cx.h[k] = ok ? hj : 0.f; cx.r[k] = ok ? rj : 0.f; cx.w[k] = wj; cx.q[k] = ok ? qj : 0.f;
    }
    cx.wh = 0.f; cx.wnorm = 1.f;
    if ((SC >= 0 ? SC : m.scorer) == KGE_TRANSH) {
        wn2 = kge_wave_sum(wn2); whp = kge_wave_sum(whp);
        const float nrm = fmaxf(sqrtf(wn2), 1e-12f), inv = 1.f / nrm;
        cx.wnorm = nrm; cx.wh = whp * inv;
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) {
            cx.w[k] *= inv;                                           // unit normal
            cx.q[k] = (lane + 64 * k < d) ? cx.h[k] - cx.wh * cx.w[k] + cx.r[k] : 0.f;
        }
    }
}

