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
//   epilogue  score / loss weights / gradient coefficients, element by element
//   phase 2   out^t[d x 32 own] += Xt_tile[d x 32 stream] . coef[stream x own]
//             (contraction over the stream index; the coefficients go from the accumulator
//             registers straight into the B-operand, the transposed tile Xt supplies the A-fragments)
// In both phases an own row lives in ONE lane pair (l, l+32), so every per-row quantity (running
// maximum, sums, rescaling factors) is a per-lane scalar.
//
//   MODE_SCORE  own = negatives, stream = queries : writes the scores S[b, n]
//   MODE_FWD    own = queries,   stream = negatives: one pass gives the loss statistics of each row
//               (running max / sum of the softmax weights, weighted loss terms) AND the
//               unnormalised gradient of the queries, rescaled online when the running max moves
//   MODE_GRADT  own = negatives, stream = queries : gradient of the negatives, needs the per-row
//               constants that MODE_FWD's statistics produce
//
// Accumulator layout of v_mfma_f32_32x32x*: lane l holds column (l & 31) and, in register i,
// row 8*(i/4) + 4*(l/32) + (i%4).
#pragma once
#include "kge_internal.h"
#include <type_traits>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 kge_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float kge_f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float kge_f32x4;
typedef uint32_t kge_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t kge_u32x2 __attribute__((ext_vector_type(2)));

constexpr float KGE_LOG2E = 1.4426950408889634f;
constexpr float KGE_LN2 = 0.6931471805599453f;
constexpr float KGE_TAU = 8.f;     // log2 headroom of the softmax weights over their reference exponent

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
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf2;
    bf2 v = { (__bf16)lo, (__bf16)hi };          // round-to-nearest-even, lo in bits 0..15
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ float kge_elem_to_float(float x) { return x; }
__device__ __forceinline__ float kge_elem_to_float(__bf16 x) { return (float)x; }
__device__ __forceinline__ float kge_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float kge_log2(float x) { return __builtin_amdgcn_logf(x); }

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

template <bool BF16, int RB, int MODE, bool TRANSH, int DSPLIT>
struct KgeBlockCfg {
    static constexpr bool OWN_ROW = MODE == KGE_MODE_FWD;
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
    static constexpr bool HAS_XT = MODE != KGE_MODE_SCORE;
    static constexpr int SIDE_BYTES = ST * 16;
    static constexpr int STAGE_BYTES = X_BYTES * (HAS_X2 ? 2 : 1) + (HAS_XT ? XT_BYTES * (HAS_X2 ? 2 : 1) : 0) + SIDE_BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static constexpr int X_UNITS = ST * RB / 16 / 256;     // 16-byte units per thread
    static constexpr int XT_UNITS = DP * 8 / 256;          // XT_UNIT-byte units per thread
    static_assert(ST * RB / 16 % 256 == 0 && DP * 8 % 256 == 0, "tile copy must divide evenly");
};

template <bool BF16, int RB, int MODE, bool TRANSH, int KIND, int LOSS, int DSPLIT>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(1, 1)))
void kge_block_kernel(const KgeBlockArgs a) {
    using C = KgeBlockCfg<BF16, RB, MODE, TRANSH, DSPLIT>;
    using XtU = typename std::conditional<BF16, kge_u32x2, kge_u32x4>::type;
    constexpr bool OWN_ROW = C::OWN_ROW;
    constexpr bool PHASE2 = MODE != KGE_MODE_SCORE;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, g = lane >> 5;
    const int own_base = blockIdx.x * KGE_OWN_TILE;
    const int split = blockIdx.y;
    const int dblk0 = blockIdx.z * C::NBH;
    const int oidx = own_base + wave * 32 + lr;
    const int t0 = split * a.tiles_per_split;
    const int t1 = min(a.str_tiles, t0 + a.tiles_per_split);
    const int str_limit = OWN_ROW ? a.N : a.B;            // valid stream rows

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
    float o_qn = 0.f, o_c = 0.f, o_wn = 1.f, o_tn = 0.f;
    if constexpr (OWN_ROW) {
        KgeRowInfo ri = a.rowinfo[oidx];
        o_qn = ri.qn; o_c = ri.c; o_wn = ri.wn;
    } else {
        o_tn = a.tn[oidx];
    }

    // ---- accumulators of the launch ------------------------------------------------------------
    kge_f32x16 acc2[PHASE2 ? C::NBH : 1];
    kge_f32x16 acc2b[(PHASE2 && TRANSH && OWN_ROW) ? C::NBH : 1];
    if constexpr (PHASE2) {
#pragma unroll
        for (int b = 0; b < C::NBH; ++b) {
            for (int i = 0; i < 16; ++i) acc2[b][i] = 0.f;
            if constexpr (TRANSH && OWN_ROW) for (int i = 0; i < 16; ++i) acc2b[b][i] = 0.f;
        }
    }
    float sum1 = 0.f, sum2 = 0.f, sum3 = 0.f;           // sums of the coefficients over the stream index
    float st_m = -INFINITY, st_l = 0.f, st_acc = 0.f;   // FWD: running max (log2 domain) / sum / weighted loss

    // ---- global -> register -> LDS staging of one stream tile ----------------------------------
    kge_u32x4 px[C::X_UNITS];
    kge_u32x4 px2[C::HAS_X2 ? C::X_UNITS : 1];
    XtU pxt[C::HAS_XT ? C::XT_UNITS : 1];
    XtU pxt2[(C::HAS_XT && C::HAS_X2) ? C::XT_UNITS : 1];
    kge_f32x4 pside = {0.f, 0.f, 0.f, 0.f};

    auto gload = [&](int tile) {
        const char *src = (const char *)a.str + (size_t)tile * C::ST * RB;
#pragma unroll
        for (int u = 0; u < C::X_UNITS; ++u) px[u] = *(const kge_u32x4 *)(src + (size_t)(tid + u * 256) * 16);
        if constexpr (C::HAS_X2) {
            const char *src2 = (const char *)a.str2 + (size_t)tile * C::ST * RB;
#pragma unroll
            for (int u = 0; u < C::X_UNITS; ++u) px2[u] = *(const kge_u32x4 *)(src2 + (size_t)(tid + u * 256) * 16);
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
                pside[0] = a.tn[sidx];
            } else {
                pside = *(const kge_f32x4 *)(a.rowinfo + sidx);
            }
        }
    };
    auto lstore = [&](int stage) {
        char *base = lds + stage * C::STAGE_BYTES;
#pragma unroll
        for (int u = 0; u < C::X_UNITS; ++u) {
            int unit = tid + u * 256, row = unit / (RB / 16), cu = unit % (RB / 16);
            *(kge_u32x4 *)(base + row * C::X_STRIDE + cu * 16) = px[u];
            if constexpr (C::HAS_X2) *(kge_u32x4 *)(base + C::X_BYTES + row * C::X_STRIDE + cu * 16) = px2[u];
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
            *(kge_f32x4 *)(side + tid * 16) = pside;
        }
    };

    if (t0 < t1) {
        gload(t0);
        lstore(0);
    }
    __syncthreads();

    // The FWD pass keeps all weights relative to a per-row reference exponent st_m that is only
    // raised (and the accumulators rescaled) when a tile's maximum exceeds it by more than KGE_TAU:
    // weights stay below 2^KGE_TAU, and the rescaling code sits outside the hot loop.  A tile that
    // trips the check leaves the inner loop before using its weights and is redone after the
    // rescale (its next-tile prefetch is already in flight: have_next).
    int tile = t0;
    bool have_next = false;
    float pend_max = -INFINITY;
    for (;;) {
        if constexpr (MODE == KGE_MODE_FWD) {
            if (tile >= t1) break;
            const float m_new = fmaxf(st_m, pend_max);
            const float r = m_new > st_m ? kge_exp2(st_m - m_new) : 1.f;      // exp2(-inf) = 0 at the start
            st_m = m_new;
            st_l *= r; st_acc *= r; sum1 *= r; sum2 *= r; sum3 *= r;
#pragma unroll
            for (int b = 0; b < C::NBH; ++b) {
                // one block at a time: the accumulators live in AGPRs and pass through VGPRs here
                for (int i = 0; i < 16; ++i) acc2[b][i] *= r;
                asm volatile("" ::: "memory");
                if constexpr (TRANSH) { for (int i = 0; i < 16; ++i) acc2b[b][i] *= r; asm volatile("" ::: "memory"); }
            }
        }
        bool redo = false;
        for (; tile < t1; ++tile) {
        const int stage = (tile - t0) & 1;
        const bool more = tile + 1 < t1;
        if (more && !have_next) gload(tile + 1);
        have_next = more;

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
        const int sbase = tile * C::ST + 4 * g;            // stream index of register i: sbase + 8*(i/4) + (i%4)
        const bool tile_full = tile * C::ST + C::ST <= str_limit;
        float sv[16], dv[16], Av[16];                      // score, 1/distance, w.t
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int sl = 8 * (i >> 2) + 4 * g + (i & 3);
            float s;
            dv[i] = 0.f; Av[i] = 0.f;
            if constexpr (KIND == KGE_KIND_MULT) {
                s = acc[i];
            } else {
                float qn, cc, wn, tnv;
                if constexpr (OWN_ROW) { qn = o_qn; cc = o_c; wn = o_wn; tnv = *(const float *)(side + sl * 16); }
                else { float4 ri = *(const float4 *)(side + sl * 16); qn = ri.x; cc = ri.y; wn = ri.w; tnv = o_tn; }
                float d2 = fmaf(-2.f, acc[i], qn + tnv);
                if constexpr (TRANSH) { const float A = accw[i]; Av[i] = A; d2 += A * (2.f * cc - A * (2.f - wn)); }
                if (d2 < 1e-3f * (qn + tnv)) {             // cancellation: redo this entry by direct differences
                    const int sidx = tile * C::ST + sl;
                    const int b = OWN_ROW ? oidx : sidx, n = OWN_ROW ? sidx : oidx;
                    const char *qb = (const char *)(OWN_ROW ? a.own : a.str) + (size_t)b * RB;
                    const char *tb = (const char *)(OWN_ROW ? a.str : a.own) + (size_t)n * RB;
                    const char *wb = TRANSH ? (const char *)(OWN_ROW ? a.own2 : a.str2) + (size_t)b * RB : nullptr;
                    d2 = kge_direct_d2<BF16, TRANSH>(qb, tb, wb, C::DP);
                }
                d2 = fmaxf(d2, 0.f);
                const float inv = d2 > 0.f ? __builtin_amdgcn_rsqf(d2) : 0.f;
                dv[i] = inv;
                s = -d2 * inv;                              // -sqrt(d2)
            }
            sv[i] = s;
        }
        if constexpr (MODE == KGE_MODE_SCORE) {
            if (oidx < a.N) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int b = sbase + 8 * (i >> 2) + (i & 3);
                    if (b < a.B) a.S_out[(size_t)b * a.N + oidx] = sv[i];
                }
            }
        }
        float coef[16], coef2[16];
        if constexpr (MODE == KGE_MODE_FWD) {
            // softmax weights of this row over the stream index, relative to the reference st_m (log2 domain)
            const float xscale = (LOSS == KGE_LOGSIGMOID ? a.adv_temp : 1.f) * KGE_LOG2E;
            float x2[16], tile_max = -INFINITY;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                x2[i] = sv[i] * xscale;
                if (!tile_full && sbase + 8 * (i >> 2) + (i & 3) >= str_limit) x2[i] = -INFINITY;
                tile_max = fmaxf(tile_max, x2[i]);
            }
            // lanes l and l^32 hold the two halves of the same row and feed ONE contraction in
            // phase 2, so they must share the reference
            tile_max = fmaxf(tile_max, __shfl_xor(tile_max, 32));
            if (__any(tile_max > st_m + KGE_TAU)) { pend_max = tile_max; redo = true; break; }
            const float m_safe = st_m > -INFINITY ? st_m : 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float e = kge_exp2(x2[i] - m_safe);                    // masked entries: exp2(-inf) = 0
                st_l += e;
                float u = e;
                if constexpr (LOSS == KGE_LOGSIGMOID) {
                    // weight * sigma(gamma + s) for the gradient, weight * softplus(gamma + s) for the loss
                    const float y = a.gamma + sv[i];
                    const float t = kge_exp2(-fabsf(y) * KGE_LOG2E);
                    const float rcp = __builtin_amdgcn_rcpf(1.f + t);
                    const float sig = y >= 0.f ? rcp : t * rcp;
                    const float softplus = fmaxf(y, 0.f) + KGE_LN2 * kge_log2(1.f + t);
                    if (e > 0.f) st_acc = fmaf(e, softplus, st_acc);
                    u = e * sig;
                }
                const float c1 = KIND == KGE_KIND_DIST ? u * dv[i] : u;
                coef[i] = c1;
                sum1 += c1;
                if constexpr (TRANSH) { coef2[i] = c1 * Av[i]; sum2 += coef2[i]; sum3 += coef2[i] * Av[i]; }
            }
        }
        if constexpr (MODE == KGE_MODE_GRADT) {
            // gradient coefficient of every (query, negative) pair from the finished row constants
            const float xscale = (LOSS == KGE_LOGSIGMOID ? a.adv_temp : 1.f) * KGE_LOG2E;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int sl = 8 * (i >> 2) + 4 * g + (i & 3);
                const float K2 = *(const float *)(side + sl * 16 + 8);       // -inf for padded queries
                float u = kge_exp2(fmaf(sv[i], xscale, K2));
                if constexpr (LOSS == KGE_LOGSIGMOID) {
                    const float y = a.gamma + sv[i];
                    const float t = kge_exp2(-fabsf(y) * KGE_LOG2E);
                    const float rcp = __builtin_amdgcn_rcpf(1.f + t);
                    u *= y >= 0.f ? rcp : t * rcp;
                }
                const float c1 = KIND == KGE_KIND_DIST ? u * dv[i] : u;
                coef[i] = c1;
                sum1 += c1;
                if constexpr (TRANSH) coef2[i] = c1 * Av[i];
            }
        }
        // ---- phase 2: out^t[d, own] += Xt[d, stream] . coef[stream, own] -----------------------
        if constexpr (PHASE2) {
            const char *xt = base + C::X_BYTES * (C::HAS_X2 ? 2 : 1);
            if constexpr (BF16) {
                uint4 bf[2], bf2[2];
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    bf[s2] = make_uint4(kge_pack_bf16x2(coef[8 * s2 + 0], coef[8 * s2 + 1]),
                                        kge_pack_bf16x2(coef[8 * s2 + 2], coef[8 * s2 + 3]),
                                        kge_pack_bf16x2(coef[8 * s2 + 4], coef[8 * s2 + 5]),
                                        kge_pack_bf16x2(coef[8 * s2 + 6], coef[8 * s2 + 7]));
                    if constexpr (TRANSH)
                        bf2[s2] = make_uint4(kge_pack_bf16x2(coef2[8 * s2 + 0], coef2[8 * s2 + 1]),
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
                        uint4 av = make_uint4(lo.x, lo.y, hi.x, hi.y);
                        acc2[blk] = kge_mma16<true>(acc2[blk], av, bf[s2]);
                        if constexpr (TRANSH && OWN_ROW) acc2b[blk] = kge_mma16<true>(acc2b[blk], av, bf2[s2]);
                        if constexpr (TRANSH && !OWN_ROW) {
                            uint2 lo2 = *(const uint2 *)(p + C::XT_BYTES + 32 * s2);
                            uint2 hi2 = *(const uint2 *)(p + C::XT_BYTES + 32 * s2 + 16);
                            acc2[blk] = kge_mma16<true>(acc2[blk], make_uint4(lo2.x, lo2.y, hi2.x, hi2.y), bf2[s2]);
                        }
                    }
                }
            } else {
#pragma unroll
                for (int blk = 0; blk < C::NBH; ++blk) {
                    const char *p = xt + ((dblk0 + blk) * 32 + lr) * C::XT_STRIDE + g * 16;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        kge_f32x4 av = *(const kge_f32x4 *)(p + 32 * j);
                        kge_f32x4 av2;
                        if constexpr (TRANSH && !OWN_ROW) av2 = *(const kge_f32x4 *)(p + C::XT_BYTES + 32 * j);
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            acc2[blk] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[r], coef[4 * j + r], acc2[blk], 0, 0, 0);
                            if constexpr (TRANSH && OWN_ROW)
                                acc2b[blk] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[r], coef2[4 * j + r], acc2b[blk], 0, 0, 0);
                            if constexpr (TRANSH && !OWN_ROW)
                                acc2[blk] = __builtin_amdgcn_mfma_f32_32x32x2f32(av2[r], coef2[4 * j + r], acc2[blk], 0, 0, 0);
                        }
                    }
                }
            }
        }
        if (more) lstore(stage ^ 1);
        have_next = false;
        __syncthreads();
        }
        if (MODE != KGE_MODE_FWD || !redo) break;
    }

    // ---- write-out ---------------------------------------------------------------------------------
    if constexpr (PHASE2) {
        // lanes l and l^32 hold the same own row over disjoint stream entries (same running max):
        // add their scalars.  The phase-2 accumulators already contain both halves.
        if constexpr (MODE == KGE_MODE_FWD) { st_l += __shfl_xor(st_l, 32); st_acc += __shfl_xor(st_acc, 32); }
        sum1 += __shfl_xor(sum1, 32); sum2 += __shfl_xor(sum2, 32); sum3 += __shfl_xor(sum3, 32);
        if (g == 0 && blockIdx.z == 0) {
            a.sum_part[(size_t)split * a.own_pad + oidx] = make_float4(sum1, sum2, sum3, 0.f);
            if constexpr (MODE == KGE_MODE_FWD) a.stat_part[(size_t)split * a.own_pad + oidx] = make_float4(st_m, st_l, st_acc, 0.f);
        }
#pragma unroll
        for (int blk = 0; blk < C::NBH; ++blk) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int dcol = (dblk0 + blk) * 32 + 8 * q4 + 4 * g;
                const size_t o = ((size_t)split * a.own_pad + oidx) * C::DP + dcol;
                *(float4 *)(a.acc_part + o) = make_float4(acc2[blk][4 * q4], acc2[blk][4 * q4 + 1], acc2[blk][4 * q4 + 2], acc2[blk][4 * q4 + 3]);
                if constexpr (TRANSH && OWN_ROW)
                    *(float4 *)(a.acc_part2 + o) = make_float4(acc2b[blk][4 * q4], acc2b[blk][4 * q4 + 1], acc2b[blk][4 * q4 + 2], acc2b[blk][4 * q4 + 3]);
            }
        }
    }
}

template <bool BF16, int RB, int MODE, bool TRANSH, int KIND, int LOSS, int DSPLIT>
int kge_block_launch(const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st) {
    using C = KgeBlockCfg<BF16, RB, MODE, TRANSH, DSPLIT>;
    auto kern = kge_block_kernel<BF16, RB, MODE, TRANSH, KIND, LOSS, DSPLIT>;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES) != hipSuccess)
            return KGE_E_HIP;
        attr_set = true;
    }
    dim3 grid(own_tiles, nsplit, MODE != KGE_MODE_SCORE ? DSPLIT : 1);
    hipLaunchKernelGGL(kern, grid, dim3(256), C::LDS_BYTES, st, a);
    return kge_launch_status();
}
