// The shared-negative block kernel (gfx950, wave64, MFMA 32x32).
//
// The micro-batch's queries Q [B, d] (built from h and r) meet ONE block of negative tails
// T [N, d] shared by all of them (arXiv 2211.12281, Section 4 "Training", eq. (negsamples)), so the
// B x N scores of Table 2 are a dense contraction Q T^t followed by an elementwise map; the loss of
// Section 3.1 needs row reductions of that block, and its backward pass two more contractions
// (G T and G^t Q).  The block itself never goes to memory: it is recomputed tile by tile.
//
// One template serves all passes.  A workgroup (4 waves) OWNS 128 rows of one operand, held in
// registers as MFMA B-fragments for the whole launch, and STREAMS the other operand through LDS
// in tiles of 32 rows (double buffered).  Per tile and wave:
//   phase 1   acc[32 stream x 32 own] = X_tile . own^t          (contraction over d)
//   epilogue  score / loss statistics / gradient coefficients, element by element
//   phase 2   out[32 own x d] += coef[own x stream] . Xt_tile   (contraction over the stream
//             index; the coefficients go from the accumulator registers straight into the
//             A-operand, the transposed tile Xt supplies matching B-fragments)
// OWN_ROW = true : own = queries  (row statistics, dQ)     stream = negatives
// OWN_ROW = false: own = negatives (score output, dT)      stream = queries
//
// Accumulator layout of v_mfma_f32_32x32x*: lane l holds column (l & 31) and, in register i,
// row 8*(i/4) + 4*(l/32) + (i%4).
#pragma once
#include "kge_internal.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 kge_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float kge_f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float kge_f32x4;

template <bool BF16> struct KgeElem;
template <> struct KgeElem<true>  { using type = __bf16; static constexpr int size = 2; };
template <> struct KgeElem<false> { using type = float;  static constexpr int size = 4; };

// acc += A(16 bytes per lane) . B(16 bytes per lane): one 32x32x16 bf16 MFMA, or four 32x32x2 fp32
template <bool BF16>
__device__ __forceinline__ kge_f32x16 kge_mma16(kge_f32x16 acc, uint4 a, uint4 b) {
    if constexpr (BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(kge_bf16x8, a),
                                                       __builtin_bit_cast(kge_bf16x8, b), acc, 0, 0, 0);
    } else {
        kge_f32x4 fa = __builtin_bit_cast(kge_f32x4, a), fb = __builtin_bit_cast(kge_f32x4, b);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[0], fb[0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[1], fb[1], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[2], fb[2], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[3], fb[3], acc, 0, 0, 0);
        return acc;
    }
}

__device__ __forceinline__ uint32_t kge_pack_bf16x2(float lo, float hi) {
    // round-to-nearest-even of two floats into one dword (lo in bits 0..15)
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf2;
    bf2 v = { (__bf16)lo, (__bf16)hi };
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ float kge_elem_to_float(float x) { return x; }
__device__ __forceinline__ float kge_elem_to_float(__bf16 x) { return (float)x; }

// Squared distance of one (query, tail) pair by direct differences; the fallback for block entries
// whose norm-expansion form cancels.  TransH: u = q - t + (w.t) w.
template <bool BF16, bool TRANSH>
__device__ __noinline__ float kge_direct_d2(const void *qv, const void *tv, const void *wv, int dp) {
    using E = typename KgeElem<BF16>::type;
    const E *q = (const E *)qv, *t = (const E *)tv, *w = (const E *)wv;
    float A = 0.f;
    if constexpr (TRANSH)
        for (int j = 0; j < dp; ++j) A += kge_elem_to_float(w[j]) * kge_elem_to_float(t[j]);
    float acc = 0.f;
    for (int j = 0; j < dp; ++j) {
        float x = kge_elem_to_float(q[j]) - kge_elem_to_float(t[j]);
        if constexpr (TRANSH) x += A * kge_elem_to_float(w[j]);
        acc += x * x;
    }
    return acc;
}

__device__ __forceinline__ float kge_softplus(float y) {
    return fmaxf(y, 0.f) + log1pf(__expf(-fabsf(y)));
}

template <bool BF16, int RB, bool OWN_ROW, int MODE, bool TRANSH, int DSPLIT>
struct KgeBlockCfg {
    static constexpr int ES = KgeElem<BF16>::size;
    static constexpr int DP = RB / ES;                     // padded dim
    static constexpr int KS = RB / 32;                     // 32-byte k-steps of phase 1
    static constexpr int ST = KGE_STREAM_TILE;
    static constexpr int NB = DP / 32;                     // 32-column output blocks of phase 2
    static constexpr int NBH = NB / DSPLIT;                // ... handled by one z-slice
    static constexpr int X_STRIDE = RB + 16;
    static constexpr int X_BYTES = ST * X_STRIDE;
    static constexpr int XT_UNIT = BF16 ? 8 : 16;
    static constexpr int XT_ROWB = ST * ES;
    static constexpr int XT_STRIDE = XT_ROWB + XT_UNIT;
    static constexpr int XT_BYTES = DP * XT_STRIDE;
    static constexpr bool HAS_X2 = TRANSH && !OWN_ROW;     // second streamed operand (normals)
    static constexpr bool HAS_XT = MODE == KGE_MODE_GRAD;
    static constexpr int SIDE_BYTES = ST * 16;
    static constexpr int STAGE_BYTES = X_BYTES * (HAS_X2 ? 2 : 1) + (HAS_XT ? XT_BYTES * (HAS_X2 ? 2 : 1) : 0) + SIDE_BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static constexpr int X_UNITS = ST * RB / 16 / 256;     // 16-byte units per thread
    static constexpr int XT_UNITS = DP * 8 / 256;          // XT_UNIT-byte units per thread
    static_assert(ST * RB / 16 % 256 == 0 && DP * 8 % 256 == 0, "tile copy must divide evenly");
};

template <bool BF16, int RB, bool OWN_ROW, int MODE, bool TRANSH, int DSPLIT>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(1, 1)))
void kge_block_kernel(const KgeBlockArgs a) {
    using C = KgeBlockCfg<BF16, RB, OWN_ROW, MODE, TRANSH, DSPLIT>;
    using XtU = typename std::conditional<BF16, uint2, uint4>::type;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, g = lane >> 5;
    const int own_base = blockIdx.x * KGE_OWN_TILE;
    const int split = blockIdx.y;
    const int dblk0 = blockIdx.z * C::NBH;
    const int oidx = own_base + wave * 32 + lr;
    const int t0 = split * a.tiles_per_split;
    const int t1 = min(a.str_tiles, t0 + a.tiles_per_split);

    // ---- own operand fragments: 16 bytes per lane per 32-byte k-step --------------------------
    uint4 own[C::KS];
    uint4 ownw[(TRANSH && OWN_ROW) ? C::KS : 1];
    {
        const char *p = (const char *)a.own + (size_t)oidx * RB + g * 16;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) own[ks] = *(const uint4 *)(p + ks * 32);
        if constexpr (TRANSH && OWN_ROW) {
            const char *pw = (const char *)a.own2 + (size_t)oidx * RB + g * 16;
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) ownw[ks] = *(const uint4 *)(pw + ks * 32);
        }
    }
    // own-side scalars
    float o_qn = 0.f, o_c = 0.f, o_K = 0.f, o_tn = 0.f;
    if constexpr (OWN_ROW) {
        KgeRowInfo ri = a.rowinfo[oidx];
        o_qn = ri.qn; o_c = ri.c; o_K = ri.K;
    } else {
        o_tn = a.tn[oidx];
    }
    const bool own_valid = OWN_ROW ? (oidx < a.B) : (oidx < a.N);

    // ---- accumulators of the launch ------------------------------------------------------------
    kge_f32x16 acc2[(MODE == KGE_MODE_GRAD) ? C::NBH : 1];
    kge_f32x16 acc2b[(MODE == KGE_MODE_GRAD && TRANSH && OWN_ROW) ? C::NBH : 1];
    if constexpr (MODE == KGE_MODE_GRAD) {
#pragma unroll
        for (int b = 0; b < C::NBH; ++b) {
            for (int i = 0; i < 16; ++i) acc2[b][i] = 0.f;
            if constexpr (TRANSH && OWN_ROW) for (int i = 0; i < 16; ++i) acc2b[b][i] = 0.f;
        }
    }
    float sum1 = 0.f, sum2 = 0.f, sum3 = 0.f;           // GRAD: sums of the coefficients
    float st_m = -INFINITY, st_l = 0.f, st_acc = 0.f;   // STATS: running max / sum / weighted loss

    // ---- global -> register -> LDS staging of one stream tile ----------------------------------
    uint4 px[C::X_UNITS];
    uint4 px2[C::HAS_X2 ? C::X_UNITS : 1];
    XtU pxt[C::HAS_XT ? C::XT_UNITS : 1];
    XtU pxt2[(C::HAS_XT && C::HAS_X2) ? C::XT_UNITS : 1];
    float4 pside = make_float4(0.f, 0.f, 0.f, 0.f);

    auto gload = [&](int tile) {
        const char *src = (const char *)a.str + (size_t)tile * C::ST * RB;
#pragma unroll
        for (int u = 0; u < C::X_UNITS; ++u) px[u] = *(const uint4 *)(src + (size_t)(tid + u * 256) * 16);
        if constexpr (C::HAS_X2) {
            const char *src2 = (const char *)a.str2 + (size_t)tile * C::ST * RB;
#pragma unroll
            for (int u = 0; u < C::X_UNITS; ++u) px2[u] = *(const uint4 *)(src2 + (size_t)(tid + u * 256) * 16);
        }
        if constexpr (C::HAS_XT) {
#pragma unroll
            for (int u = 0; u < C::XT_UNITS; ++u) {
                int unit = tid + u * 256, row = unit >> 3, cu = unit & 7;
                size_t off = ((size_t)row * a.strT_ld + (size_t)tile * C::ST) * C::ES + cu * C::XT_UNIT;
                pxt[u] = *(const XtU *)((const char *)a.strT + off);
                if constexpr (C::HAS_X2) pxt2[u] = *(const XtU *)((const char *)a.strT2 + off);
            }
        }
        if (tid < C::ST) {
            int sidx = tile * C::ST + tid;
            if constexpr (OWN_ROW) {
                pside.x = a.tn[sidx];
            } else {
                KgeRowInfo ri = a.rowinfo[sidx];
                pside = make_float4(ri.qn, ri.c, ri.K, 0.f);
            }
        }
    };
    auto lstore = [&](int stage) {
        char *base = lds + stage * C::STAGE_BYTES;
#pragma unroll
        for (int u = 0; u < C::X_UNITS; ++u) {
            int unit = tid + u * 256, row = unit / (RB / 16), cu = unit % (RB / 16);
            *(uint4 *)(base + row * C::X_STRIDE + cu * 16) = px[u];
            if constexpr (C::HAS_X2) *(uint4 *)(base + C::X_BYTES + row * C::X_STRIDE + cu * 16) = px2[u];
        }
        char *xt = base + C::X_BYTES * (C::HAS_X2 ? 2 : 1);
        if constexpr (C::HAS_XT) {
#pragma unroll
            for (int u = 0; u < C::XT_UNITS; ++u) {
                int unit = tid + u * 256, row = unit >> 3, cu = unit & 7;
                *(XtU *)(xt + row * C::XT_STRIDE + cu * C::XT_UNIT) = pxt[u];
                if constexpr (C::HAS_X2) *(XtU *)(xt + C::XT_BYTES + row * C::XT_STRIDE + cu * C::XT_UNIT) = pxt2[u];
            }
        }
        if (tid < C::ST) {
            char *side = base + C::STAGE_BYTES - C::SIDE_BYTES;
            *(float4 *)(side + tid * 16) = pside;
        }
    };

    if (t0 < t1) {
        gload(t0);
        lstore(0);
    }
    __syncthreads();

    for (int tile = t0; tile < t1; ++tile) {
        const int stage = (tile - t0) & 1;
        const bool more = tile + 1 < t1;
        if (more) gload(tile + 1);

        const char *base = lds + stage * C::STAGE_BYTES;
        const char *side = base + C::STAGE_BYTES - C::SIDE_BYTES;
        // ---- phase 1: acc[stream, own] -------------------------------------------------------
        kge_f32x16 acc, accw;
        for (int i = 0; i < 16; ++i) { acc[i] = 0.f; accw[i] = 0.f; }
        {
            const char *xrow = base + lr * C::X_STRIDE + g * 16;
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) {
                uint4 av = *(const uint4 *)(xrow + ks * 32);
                acc = kge_mma16<BF16>(acc, av, own[ks]);
                if constexpr (TRANSH && OWN_ROW) accw = kge_mma16<BF16>(accw, av, ownw[ks]);
                if constexpr (TRANSH && !OWN_ROW) {
                    uint4 aw = *(const uint4 *)(xrow + C::X_BYTES + ks * 32);
                    accw = kge_mma16<BF16>(accw, aw, own[ks]);
                }
            }
        }
        // ---- epilogue ------------------------------------------------------------------------
        float coef[16], coef2[16];
        float xs[16], sv[16];
        float tile_max = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int sl = 8 * (i >> 2) + 4 * g + (i & 3);
            const int sidx = tile * C::ST + sl;
            float qn, cc, K, tnv;
            int b, n;
            if constexpr (OWN_ROW) {
                qn = o_qn; cc = o_c; K = o_K; tnv = *(const float *)(side + sl * 16);
                b = oidx; n = sidx;
            } else {
                float4 ri = *(const float4 *)(side + sl * 16);
                qn = ri.x; cc = ri.y; K = ri.z; tnv = o_tn;
                b = sidx; n = oidx;
            }
            const bool valid = own_valid && (OWN_ROW ? (sidx < a.N) : (sidx < a.B));
            float s, dist = 0.f, A = 0.f;
            if (a.kind == KGE_KIND_MULT) {
                s = acc[i];
            } else {
                float d2 = qn + tnv - 2.f * acc[i];
                if constexpr (TRANSH) { A = accw[i]; d2 += 2.f * A * cc - A * A; }
                if (valid && d2 < 1e-3f * (qn + tnv)) {
                    const char *qb = (const char *)(OWN_ROW ? a.own : a.str) + (size_t)b * RB;
                    const char *tb = (const char *)(OWN_ROW ? a.str : a.own) + (size_t)n * RB;
                    const char *wb = TRANSH ? (const char *)(OWN_ROW ? a.own2 : a.str2) + (size_t)b * RB : nullptr;
                    d2 = kge_direct_d2<BF16, TRANSH>(qb, tb, wb, C::DP);
                }
                dist = sqrtf(fmaxf(d2, 0.f));
                s = -dist;
            }
            if constexpr (MODE == KGE_MODE_SCORE) {
                if (valid) a.S_out[(size_t)b * a.N + n] = s;
            } else if constexpr (MODE == KGE_MODE_STATS) {
                float x = (a.loss == KGE_LOGSIGMOID) ? a.adv_temp * s : s + a.c_corr;
                x = valid ? x : -INFINITY;
                xs[i] = x; sv[i] = s;
                tile_max = fmaxf(tile_max, x);
            } else {
                float G;
                if (a.loss == KGE_LOGSIGMOID) {
                    float e = __expf(-(a.gamma + s));                 // sigma(gamma + s) = 1 / (1 + e)
                    G = __expf(a.adv_temp * s + K) / (1.f + e);
                } else {
                    G = __expf(s + K);
                }
                float c1 = G;
                if (a.kind == KGE_KIND_DIST) c1 = dist > 0.f ? G / dist : 0.f;
                c1 = valid ? c1 : 0.f;
                coef[i] = c1;
                sum1 += c1;
                if constexpr (TRANSH) {
                    coef2[i] = c1 * A;
                    sum2 += c1 * A;
                    sum3 += c1 * A * A;
                }
            }
        }
        if constexpr (MODE == KGE_MODE_STATS) {
            if (tile_max > -INFINITY) {
                float m_new = fmaxf(st_m, tile_max);
                float r = __expf(st_m - m_new);                       // exp(-inf) = 0 on the first tile
                st_l *= r; st_acc *= r; st_m = m_new;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float e = __expf(xs[i] - m_new);                  // masked entries: exp(-inf) = 0
                    st_l += e;
                    if (a.loss == KGE_LOGSIGMOID && xs[i] > -INFINITY) st_acc += e * kge_softplus(a.gamma + sv[i]);
                }
            }
        }
        // ---- phase 2: out[own, d] += coef[own, stream] . Xt ------------------------------------
        if constexpr (MODE == KGE_MODE_GRAD) {
            const char *xt = base + C::X_BYTES * (C::HAS_X2 ? 2 : 1);
            if constexpr (BF16) {
                uint4 af[2], af2[2];
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    af[s2] = make_uint4(kge_pack_bf16x2(coef[8 * s2 + 0], coef[8 * s2 + 1]),
                                        kge_pack_bf16x2(coef[8 * s2 + 2], coef[8 * s2 + 3]),
                                        kge_pack_bf16x2(coef[8 * s2 + 4], coef[8 * s2 + 5]),
                                        kge_pack_bf16x2(coef[8 * s2 + 6], coef[8 * s2 + 7]));
                    if constexpr (TRANSH)
                        af2[s2] = make_uint4(kge_pack_bf16x2(coef2[8 * s2 + 0], coef2[8 * s2 + 1]),
                                             kge_pack_bf16x2(coef2[8 * s2 + 2], coef2[8 * s2 + 3]),
                                             kge_pack_bf16x2(coef2[8 * s2 + 4], coef2[8 * s2 + 5]),
                                             kge_pack_bf16x2(coef2[8 * s2 + 6], coef2[8 * s2 + 7]));
                }
#pragma unroll
                for (int blk = 0; blk < C::NBH; ++blk) {
                    const char *p = xt + ((dblk0 + blk) * 32 + lr) * C::XT_STRIDE + g * 8;
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        uint2 lo = *(const uint2 *)(p + 32 * s2), hi = *(const uint2 *)(p + 32 * s2 + 16);
                        uint4 bv = make_uint4(lo.x, lo.y, hi.x, hi.y);
                        acc2[blk] = kge_mma16<true>(acc2[blk], af[s2], bv);
                        if constexpr (TRANSH && OWN_ROW) acc2b[blk] = kge_mma16<true>(acc2b[blk], af2[s2], bv);
                        if constexpr (TRANSH && !OWN_ROW) {
                            uint2 lo2 = *(const uint2 *)(p + C::XT_BYTES + 32 * s2);
                            uint2 hi2 = *(const uint2 *)(p + C::XT_BYTES + 32 * s2 + 16);
                            acc2[blk] = kge_mma16<true>(acc2[blk], af2[s2], make_uint4(lo2.x, lo2.y, hi2.x, hi2.y));
                        }
                    }
                }
            } else {
#pragma unroll
                for (int blk = 0; blk < C::NBH; ++blk) {
                    const char *p = xt + ((dblk0 + blk) * 32 + lr) * C::XT_STRIDE + g * 16;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        kge_f32x4 bv = *(const kge_f32x4 *)(p + 32 * j);
                        kge_f32x4 bv2;
                        if constexpr (TRANSH && !OWN_ROW) bv2 = *(const kge_f32x4 *)(p + C::XT_BYTES + 32 * j);
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            acc2[blk] = __builtin_amdgcn_mfma_f32_32x32x2f32(coef[4 * j + r], bv[r], acc2[blk], 0, 0, 0);
                            if constexpr (TRANSH && OWN_ROW)
                                acc2b[blk] = __builtin_amdgcn_mfma_f32_32x32x2f32(coef2[4 * j + r], bv[r], acc2b[blk], 0, 0, 0);
                            if constexpr (TRANSH && !OWN_ROW)
                                acc2[blk] = __builtin_amdgcn_mfma_f32_32x32x2f32(coef2[4 * j + r], bv2[r], acc2[blk], 0, 0, 0);
                        }
                    }
                }
            }
        }
        if (more) lstore(stage ^ 1);
        __syncthreads();
    }

    // ---- write-out ---------------------------------------------------------------------------------
    if constexpr (MODE == KGE_MODE_STATS) {
        // lanes l and l^32 hold the same own row over disjoint stream entries
        float m2 = __shfl_xor(st_m, 32), l2 = __shfl_xor(st_l, 32), a2 = __shfl_xor(st_acc, 32);
        float m = fmaxf(st_m, m2);
        float l = 0.f, ac = 0.f;
        if (m > -INFINITY) {
            float r1 = __expf(st_m - m), r2 = __expf(m2 - m);
            l = st_l * r1 + l2 * r2;
            ac = st_acc * r1 + a2 * r2;
        }
        if (g == 0) a.stat_part[(size_t)split * a.own_pad + oidx] = make_float4(m, l, ac, 0.f);
    }
    if constexpr (MODE == KGE_MODE_GRAD) {
        sum1 += __shfl_xor(sum1, 32); sum2 += __shfl_xor(sum2, 32); sum3 += __shfl_xor(sum3, 32);
        if (g == 0 && blockIdx.z == 0) a.sum_part[(size_t)split * a.own_pad + oidx] = make_float4(sum1, sum2, sum3, 0.f);
#pragma unroll
        for (int blk = 0; blk < C::NBH; ++blk) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                int orow = own_base + wave * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
                size_t o = ((size_t)split * a.own_pad + orow) * C::DP + (dblk0 + blk) * 32 + lr;
                a.acc_part[o] = acc2[blk][i];
                if constexpr (TRANSH && OWN_ROW) a.acc_part2[o] = acc2b[blk][i];
            }
        }
    }
}

template <bool BF16, int RB, bool OWN_ROW, int MODE, bool TRANSH, int DSPLIT>
int kge_block_launch(const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st) {
    using C = KgeBlockCfg<BF16, RB, OWN_ROW, MODE, TRANSH, DSPLIT>;
    auto kern = kge_block_kernel<BF16, RB, OWN_ROW, MODE, TRANSH, DSPLIT>;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES) != hipSuccess)
            return KGE_E_HIP;
        attr_set = true;
    }
    dim3 grid(own_tiles, nsplit, MODE == KGE_MODE_GRAD ? DSPLIT : 1);
    hipLaunchKernelGGL(kern, grid, dim3(256), C::LDS_BYTES, st, a);
    return kge_launch_status();
}
