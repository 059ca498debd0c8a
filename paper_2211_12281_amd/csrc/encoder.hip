// Feature-projection encoder (arXiv 2211.12281, Section 3.1 "Encoder", eq. (embedding)):
//     e = e_S + M_H e_F  for head entities,   e = e_S + M_T e_F  for tail entities,
// with dropout on the projection and the L3 regularisers of e, e_S and M e_F (Section 3.1
// "Regularisation").  The projection of the 2B + N gathered slots is the second dense contraction of
// the paper's cost model, (B + N) |e_F| d (Section 4.1), and so is its backward pass to M_H, M_T.
//
// Both contractions run through ONE matrix-core kernel, C[M, N] = A[M, K] . B[N, K]^t with both operands
// contiguous along K (so that an MFMA fragment is one 16-byte load per lane and no LDS staging is needed):
//   forward    P[slot, d]  = F[idx[slot], :] . M[d, :]^t          (A rows gathered through the index array)
//   backward   G[d, f]     = dP^t[d, slots] . F^t[f, slots]^t     (transposed copies written by the row kernels;
//                                                                   split over the slots, partials summed in order)
#include "kge_internal.h"
#include "row_ops.hpp"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 enc_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float enc_f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float enc_f32x4;

namespace {

constexpr int ENC_TILE = 128;          // rows and columns of a workgroup's output tile; slot counts are padded to it

template <bool BF16>
__device__ __forceinline__ enc_f32x16 enc_mma16(enc_f32x16 acc, uint4 a, uint4 b) {
    if constexpr (BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(enc_bf16x8, a), __builtin_bit_cast(enc_bf16x8, b),
                                                       acc, 0, 0, 0);
    } else {
        const enc_f32x4 fa = __builtin_bit_cast(enc_f32x4, a), fb = __builtin_bit_cast(enc_f32x4, b);
#pragma unroll
        for (int r = 0; r < 4; ++r) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[r], fb[r], acc, 0, 0, 0);
        return acc;
    }
}

// C[split][M, N] (fp32) = A[M, K] . B[N, K]^t over the k-steps of the split.  A k-step is 32 bytes of a row
// (16 bf16 or 8 fp32); lane l of a fragment reads the 16 bytes at half l / 32 of row l % 32.  Rows at or
// beyond m_valid / n_valid read as zero.  a_idx (optional) maps A's row number to a table row.
// Workgroup = 128 x 128 outputs, wave = 64 x 64 (2 x 2 blocks of 32 x 32).
template <bool BF16>
__global__ __launch_bounds__(256) void enc_gemm_nt_kernel(const char *A, int64_t lda_b, const int32_t *a_idx, int m_valid,
                                                          const char *Bm, int64_t ldb_b, int n_valid, float *C, int64_t ldc,
                                                          int64_t c_split_stride, int ksteps, int ksteps_per_split) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lr = lane & 31, g = lane >> 5;
    const int m0 = blockIdx.x * ENC_TILE + (wave & 1) * 64, n0 = blockIdx.y * ENC_TILE + (wave >> 1) * 64;
    const int k_lo = blockIdx.z * ksteps_per_split, k_hi = min(ksteps, k_lo + ksteps_per_split);
    const char *pa[2], *pb[2];
    bool va[2], vb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = m0 + 32 * i + lr;
        va[i] = row < m_valid;
        const int64_t src = va[i] ? (a_idx ? (int64_t)a_idx[row] : (int64_t)row) : 0;
        pa[i] = A + src * lda_b + g * 16;
        const int col = n0 + 32 * i + lr;
        vb[i] = col < n_valid;
        pb[i] = Bm + (int64_t)(vb[i] ? col : 0) * ldb_b + g * 16;
    }
    enc_f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j)
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    constexpr int U = 4;                                   // k-steps in flight
    for (int ks = k_lo; ks < k_hi; ks += U) {
        uint4 fa[U][2], fb[U][2];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool in = ks + u < k_hi;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[u][i] = (in && va[i]) ? *(const uint4 *)(pa[i] + (int64_t)(ks + u) * 32) : zero;
                fb[u][i] = (in && vb[i]) ? *(const uint4 *)(pb[i] + (int64_t)(ks + u) * 32) : zero;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = enc_mma16<BF16>(acc[i][j], fa[u][i], fb[u][j]);
    }
    // accumulator layout: lane holds column lr of the B side; register e holds A-side row 8 (e/4) + 4 g + e%4
    float *Cs = C + (int64_t)blockIdx.z * c_split_stride;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + 32 * j + lr;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = m0 + 32 * i + 8 * (e >> 2) + 4 * g + (e & 3);
                if (row < m_valid && col < n_valid) Cs[(int64_t)row * ldc + col] = acc[i][j][e];
            }
        }
}

__device__ __forceinline__ void enc_philox_round(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c[0]), lo0 = 0xD2511F53u * c[0];
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c[2]), lo1 = 0xCD9E8D57u * c[2];
    const uint32_t n0 = hi1 ^ c[1] ^ k0, n2 = hi0 ^ c[3] ^ k1;
    c[0] = n0; c[1] = lo1; c[2] = n2; c[3] = lo0;
}
// dropout factor of element (slot, column): counter (slot, column / 4, step, tag), word column % 4; kept when
// the word is >= thr = floor(p 2^32), then scaled by 1 / (1 - p)
__device__ __forceinline__ float enc_dropout(uint32_t seed_lo, uint32_t seed_hi, uint32_t step, uint32_t tag, uint32_t slot,
                                             int col, uint32_t thr, float scale) {
    if (thr == 0u) return 1.f;
    uint32_t c[4] = { slot, (uint32_t)(col >> 2), step, tag };
    uint32_t k0 = seed_lo, k1 = seed_hi;
#pragma unroll
    for (int r = 0; r < 10; ++r) { enc_philox_round(c, k0, k1); k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    return c[col & 3] >= thr ? scale : 0.f;
}

struct EncRowArgs {
    const void *ent_s; int64_t ent_ld; const int32_t *h, *t, *neg; int B, N, d;
    uint32_t seed_lo, seed_hi, step, tag, thr; float scale, reg_t, reg_s, reg_f;
};
__device__ __forceinline__ int enc_slot_entity(const EncRowArgs &a, int i) {
    return i < a.B ? a.h[i] : (i < 2 * a.B ? a.t[i - a.B] : a.neg[i - 2 * a.B]);
}
__device__ __forceinline__ float enc_l3(float c3) { return cbrtf(kge_wave_sum(c3)); }

// forward rows: e = s + D o P, the three norms of the slot; one wave per slot, lane holds columns lane + 64 k
template <bool BF16>
__global__ void enc_finish_kernel(EncRowArgs a, const float *P, void *e_out, float *regv) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (i >= 2 * a.B + a.N) return;
    const int64_t soff = (int64_t)enc_slot_entity(a, i) * a.ent_ld;
    float ct = 0.f, cs = 0.f, cf = 0.f;
    for (int j = lane; j < a.d; j += 64) {
        const float p = P[(int64_t)i * a.d + j], s = El<BF16>::ld(a.ent_s, soff + j);
        const float e = s + enc_dropout(a.seed_lo, a.seed_hi, a.step, a.tag, (uint32_t)i, j, a.thr, a.scale) * p;
        El<BF16>::st(e_out, (int64_t)i * a.d + j, e);
        ct += fabsf(e) * e * e; cs += fabsf(s) * s * s; cf += fabsf(p) * p * p;
    }
    const bool reg = a.reg_t > 0.f || a.reg_s > 0.f || a.reg_f > 0.f;
    if (reg) {
        const float v = a.reg_t * enc_l3(ct) + a.reg_s * enc_l3(cs) + a.reg_f * enc_l3(cf);
        if (lane == 0) regv[i] = v;
    }
}

// reg_out = sum of regv in a fixed order (one workgroup)
__global__ void enc_reg_reduce_kernel(const float *regv, int n, int on, float *reg_out) {
    __shared__ double sh[1024];
    double p[4] = {0, 0, 0, 0};
    if (on)
        for (int i0 = threadIdx.x; i0 < n; i0 += 4 * 1024)
#pragma unroll
            for (int u = 0; u < 4; ++u) { const int i = i0 + u * 1024; p[u] += i < n ? (double)regv[i] : 0.0; }
    sh[threadIdx.x] = (p[0] + p[1]) + (p[2] + p[3]);
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if (threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) *reg_out = (float)sh[0];
}

// Column of slot i in the transposed buffers of the backward pass: heads first, padded to a tile, then the
// tail and negative slots (the two groups contract against different projection matrices).
__device__ __forceinline__ int enc_slot_col(int i, int B, int Bh) { return i < B ? i : Bh + (i - B); }

// backward rows (a workgroup takes 32 slots, a wave 8 of them in turn): de' = de + reg_t grad||e||,
// g_es = de' + reg_s grad||s||, dP = D o de' + reg_f grad||P||; dP leaves through the LDS as dP^t[d][columns]
template <bool BF16>
__global__ __launch_bounds__(256) void enc_bwd_rows_kernel(EncRowArgs a, const float *P, const float *de, float *g_es,
                                                           void *dPt, int Bh, int64_t ncols) {
    extern __shared__ float tile[];                        // [32][d + 1]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = 2 * a.B + a.N;
    const int i0 = blockIdx.x * 32, ldt = a.d + 1;
    for (int r = wave; r < 32; r += 4) {
        const int i = i0 + r;
        if (i >= n) { for (int j = lane; j < a.d; j += 64) tile[r * ldt + j] = 0.f; continue; }
        const int64_t soff = (int64_t)enc_slot_entity(a, i) * a.ent_ld;
        float pv[KGE_MAXJ], sv[KGE_MAXJ], ev[KGE_MAXJ], dv[KGE_MAXJ], Df[KGE_MAXJ];
        float ct = 0.f, cs = 0.f, cf = 0.f;
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) {
            const int j = lane + 64 * k;
            pv[k] = sv[k] = ev[k] = dv[k] = Df[k] = 0.f;
            if (j >= a.d) continue;
            pv[k] = P[(int64_t)i * a.d + j]; sv[k] = El<BF16>::ld(a.ent_s, soff + j); dv[k] = de[(int64_t)i * a.d + j];
            Df[k] = enc_dropout(a.seed_lo, a.seed_hi, a.step, a.tag, (uint32_t)i, j, a.thr, a.scale);
            ev[k] = sv[k] + Df[k] * pv[k];
            ct += fabsf(ev[k]) * ev[k] * ev[k]; cs += fabsf(sv[k]) * sv[k] * sv[k]; cf += fabsf(pv[k]) * pv[k] * pv[k];
        }
        float ft = 0.f, fs = 0.f, ff = 0.f;
        if (a.reg_t > 0.f) { const float nrm = enc_l3(ct); ft = nrm > 0.f ? a.reg_t / (nrm * nrm) : 0.f; }
        if (a.reg_s > 0.f) { const float nrm = enc_l3(cs); fs = nrm > 0.f ? a.reg_s / (nrm * nrm) : 0.f; }
        if (a.reg_f > 0.f) { const float nrm = enc_l3(cf); ff = nrm > 0.f ? a.reg_f / (nrm * nrm) : 0.f; }
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) {
            const int j = lane + 64 * k;
            if (j >= a.d) continue;
            const float dep = dv[k] + ft * fabsf(ev[k]) * ev[k];
            g_es[(int64_t)i * a.d + j] = dep + fs * fabsf(sv[k]) * sv[k];
            tile[r * ldt + j] = Df[k] * dep + ff * fabsf(pv[k]) * pv[k];
        }
    }
    __syncthreads();
    // transposed write-out: row j of dP^t gets the 32 slots of this workgroup (they are contiguous columns unless
    // the group straddles the head / tail boundary, hence the per-slot column)
    for (int idx = threadIdx.x; idx < a.d * 32; idx += 256) {
        const int j = idx >> 5, r = idx & 31, i = i0 + r;
        if (i < n) El<BF16>::st(dPt, (int64_t)j * ncols + enc_slot_col(i, a.B, Bh), tile[r * ldt + j]);
    }
}

// F^t[f][columns] of the gathered slots (a workgroup takes 32 slots)
template <bool BF16>
__global__ __launch_bounds__(256) void enc_gather_t_kernel(EncRowArgs a, const void *feat, int64_t feat_ld, int fd, void *Ft,
                                                           int Bh, int64_t ncols) {
    extern __shared__ float tile[];                        // [32][fd + 1]
    const int n = 2 * a.B + a.N, i0 = blockIdx.x * 32, ldt = fd + 1;
    for (int idx = threadIdx.x; idx < 32 * fd; idx += 256) {
        const int r = idx / fd, k = idx % fd, i = i0 + r;
        tile[r * ldt + k] = i < n ? El<BF16>::ld(feat, (int64_t)enc_slot_entity(a, i) * feat_ld + k) : 0.f;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < fd * 32; idx += 256) {
        const int k = idx >> 5, r = idx & 31, i = i0 + r;
        if (i < n) El<BF16>::st(Ft, (int64_t)k * ncols + enc_slot_col(i, a.B, Bh), tile[r * ldt + k]);
    }
}

__global__ void enc_zero_kernel(uint32_t *p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// out[e] = sum over the splits, in split order
__global__ void enc_split_reduce_kernel(const float *part, int nsplit, int64_t count, float *out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    float s = 0.f;
    for (int k = 0; k < nsplit; ++k) s += part[(int64_t)k * count + i];
    out[i] = s;
}

struct EncPlan { int n, Bh, Th; int64_t ncols; int es; int nsplit_h, nsplit_t, kps; };

EncPlan enc_plan(const kge_encoder_t &e, int64_t B, int64_t N) {
    EncPlan p{};
    p.n = (int)(2 * B + N);
    p.Bh = (int)kge_round_up(B, ENC_TILE); p.Th = (int)kge_round_up(B + N, ENC_TILE);
    p.ncols = (int64_t)p.Bh + p.Th;
    p.es = e.dtype == KGE_BF16 ? 2 : 4;
    // k-steps (32 bytes of a transposed row = 16 or 8 slots) per split: about 1024 slots, so that the
    // 128 x 128 output tiles of all splits fill the chip
    p.kps = 1024 / (32 / p.es);
    const int ksh = p.Bh / (32 / p.es), kst = p.Th / (32 / p.es);
    p.nsplit_h = (ksh + p.kps - 1) / p.kps; p.nsplit_t = (kst + p.kps - 1) / p.kps;
    return p;
}

EncRowArgs enc_row_args(const kge_encoder_t &e, const int32_t *h, const int32_t *t, int64_t B, const int32_t *neg, int64_t N,
                        uint64_t seed, uint64_t step) {
    EncRowArgs a{};
    a.ent_s = e.ent_s; a.ent_ld = e.ent_ld; a.h = h; a.t = t; a.neg = neg; a.B = (int)B; a.N = (int)N; a.d = e.dim;
    a.seed_lo = (uint32_t)seed; a.seed_hi = (uint32_t)(seed >> 32); a.step = (uint32_t)step; a.tag = e.dropout_tag;
    a.thr = e.dropout > 0.f ? (uint32_t)floor((double)e.dropout * 4294967296.0) : 0u;
    a.scale = e.dropout > 0.f ? (float)(1.0 / (1.0 - (double)e.dropout)) : 1.f;
    a.reg_t = e.reg_t; a.reg_s = e.reg_s; a.reg_f = e.reg_f;
    return a;
}

template <bool BF16>
void enc_launch_gemm(const void *A, int64_t lda_b, const int32_t *a_idx, int m_valid, const void *Bm, int64_t ldb_b, int n_valid,
                     float *C, int64_t ldc, int64_t split_stride, int ksteps, int kps, int nsplit, hipStream_t st) {
    dim3 grid((m_valid + ENC_TILE - 1) / ENC_TILE, (n_valid + ENC_TILE - 1) / ENC_TILE, nsplit);
    hipLaunchKernelGGL(enc_gemm_nt_kernel<BF16>, grid, dim3(256), 0, st, (const char *)A, lda_b, a_idx, m_valid, (const char *)Bm,
                       ldb_b, n_valid, C, ldc, split_stride, ksteps, kps);
}

}  // namespace

int kge_validate_encoder(const kge_encoder_t *e) {
    if (!e || (e->dtype != KGE_F32 && e->dtype != KGE_BF16)) return KGE_E_INVALID_ARG;
    const int es = e->dtype == KGE_BF16 ? 2 : 4;
    if (e->dim <= 0 || e->dim > 512 || e->dim % (32 / es) != 0) return KGE_E_INVALID_ARG;
    if (e->feat_dim <= 0 || e->feat_dim > 1024 || e->feat_dim % (32 / es) != 0) return KGE_E_INVALID_ARG;
    if (e->n_ent <= 0 || e->n_ent >= (1ll << 31) || !e->ent_s || !e->feat || !e->m_h || !e->m_t) return KGE_E_INVALID_ARG;
    if (e->ent_ld < e->dim || e->feat_ld < e->feat_dim || e->m_ld < e->feat_dim) return KGE_E_INVALID_ARG;
    // fragments are 16-byte loads: rows of the features and of the projections must start 16-byte aligned
    if ((e->feat_ld * es) % 16 != 0 || (e->m_ld * es) % 16 != 0 || ((uintptr_t)e->feat & 15) || ((uintptr_t)e->m_h & 15) ||
        ((uintptr_t)e->m_t & 15)) return KGE_E_INVALID_ARG;
    if (!(e->dropout >= 0.f && e->dropout < 1.f) || !(e->reg_t >= 0.f) || !(e->reg_s >= 0.f) || !(e->reg_f >= 0.f))
        return KGE_E_INVALID_ARG;
    return KGE_OK;
}

size_t kge_encode_ws(const kge_encoder_t &e, int64_t B, int64_t N, bool bwd) {
    const EncPlan p = enc_plan(e, B, N);
    size_t off = 0;
    auto take = [&](size_t bytes) { off += (bytes + 255) / 256 * 256; };
    take((size_t)(p.n > 0 ? p.n : 1) * 4);                                        // per-slot regulariser terms
    if (bwd) {
        take((size_t)e.dim * p.ncols * p.es);                                     // dP^t
        take((size_t)e.feat_dim * p.ncols * p.es);                                // F^t
        const int ns = p.nsplit_h > p.nsplit_t ? p.nsplit_h : p.nsplit_t;
        take((size_t)(ns > 0 ? ns : 1) * e.dim * e.feat_dim * 4);                 // split partials
    }
    return off + 256;
}

int kge_run_encode(const kge_encoder_t &e, const int32_t *h, const int32_t *t, int64_t B, const int32_t *neg, int64_t N,
                   uint64_t seed, uint64_t step, void *e_out, float *proj_out, float *reg_out, void *ws, hipStream_t st) {
    const EncPlan p = enc_plan(e, B, N);
    const bool bf16 = e.dtype == KGE_BF16;
    float *regv = (float *)ws;
    const int ksteps = e.feat_dim * p.es / 32;
    if (B > 0) {
        if (bf16) enc_launch_gemm<true>(e.feat, e.feat_ld * p.es, h, (int)B, e.m_h, e.m_ld * p.es, e.dim, proj_out, e.dim, 0, ksteps, ksteps, 1, st);
        else      enc_launch_gemm<false>(e.feat, e.feat_ld * p.es, h, (int)B, e.m_h, e.m_ld * p.es, e.dim, proj_out, e.dim, 0, ksteps, ksteps, 1, st);
        float *pt = proj_out + (size_t)B * e.dim;
        if (bf16) enc_launch_gemm<true>(e.feat, e.feat_ld * p.es, t, (int)B, e.m_t, e.m_ld * p.es, e.dim, pt, e.dim, 0, ksteps, ksteps, 1, st);
        else      enc_launch_gemm<false>(e.feat, e.feat_ld * p.es, t, (int)B, e.m_t, e.m_ld * p.es, e.dim, pt, e.dim, 0, ksteps, ksteps, 1, st);
    }
    if (N > 0) {
        float *pn = proj_out + (size_t)2 * B * e.dim;
        if (bf16) enc_launch_gemm<true>(e.feat, e.feat_ld * p.es, neg, (int)N, e.m_t, e.m_ld * p.es, e.dim, pn, e.dim, 0, ksteps, ksteps, 1, st);
        else      enc_launch_gemm<false>(e.feat, e.feat_ld * p.es, neg, (int)N, e.m_t, e.m_ld * p.es, e.dim, pn, e.dim, 0, ksteps, ksteps, 1, st);
    }
    const EncRowArgs a = enc_row_args(e, h, t, B, neg, N, seed, step);
    const bool reg = e.reg_t > 0.f || e.reg_s > 0.f || e.reg_f > 0.f;
    if (p.n > 0) {
        if (bf16) hipLaunchKernelGGL(enc_finish_kernel<true>, dim3((p.n + 3) / 4), dim3(256), 0, st, a, proj_out, e_out, regv);
        else      hipLaunchKernelGGL(enc_finish_kernel<false>, dim3((p.n + 3) / 4), dim3(256), 0, st, a, proj_out, e_out, regv);
    }
    if (reg_out) hipLaunchKernelGGL(enc_reg_reduce_kernel, dim3(1), dim3(1024), 0, st, regv, p.n, reg ? 1 : 0, reg_out);
    return kge_launch_status();
}

int kge_run_encode_bwd(const kge_encoder_t &e, const int32_t *h, const int32_t *t, int64_t B, const int32_t *neg, int64_t N,
                       uint64_t seed, uint64_t step, const float *proj, const float *de, float *g_es, float *g_mh, float *g_mt,
                       void *ws, hipStream_t st) {
    const EncPlan p = enc_plan(e, B, N);
    const bool bf16 = e.dtype == KGE_BF16;
    char *b = (char *)ws; size_t off = 0;
    auto take = [&](size_t bytes) { void *q = b + off; off += (bytes + 255) / 256 * 256; return q; };
    take((size_t)(p.n > 0 ? p.n : 1) * 4);
    void *dPt = take((size_t)e.dim * p.ncols * p.es);
    void *Ft = take((size_t)e.feat_dim * p.ncols * p.es);
    float *part = (float *)take(1);
    const int64_t mcount = (int64_t)e.dim * e.feat_dim;
    // padding columns must read as zero: clear both transposed buffers (a fill kernel, so that the call can be captured)
    const int64_t zwords = (int64_t)(((char *)part - (char *)dPt) / 4);
    hipLaunchKernelGGL(enc_zero_kernel, dim3((unsigned)((zwords + 255) / 256)), dim3(256), 0, st, (uint32_t *)dPt, zwords);
    // the row kernels stage 32 rows in the LDS: more than the default dynamic limit for long rows
    static bool attr_done = false;
    if (!attr_done) {
        const int big = 32 * (1024 + 1) * 4;
        if (hipFuncSetAttribute((const void *)enc_bwd_rows_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, big) != hipSuccess ||
            hipFuncSetAttribute((const void *)enc_bwd_rows_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, big) != hipSuccess ||
            hipFuncSetAttribute((const void *)enc_gather_t_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, big) != hipSuccess ||
            hipFuncSetAttribute((const void *)enc_gather_t_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, big) != hipSuccess)
            return KGE_E_HIP;
        attr_done = true;
    }
    const EncRowArgs a = enc_row_args(e, h, t, B, neg, N, seed, step);
    if (p.n > 0) {
        const int grid = (p.n + 31) / 32;
        if (bf16) {
            hipLaunchKernelGGL(enc_bwd_rows_kernel<true>, dim3(grid), dim3(256), 32 * (e.dim + 1) * 4, st, a, proj, de, g_es, dPt, p.Bh, p.ncols);
            hipLaunchKernelGGL(enc_gather_t_kernel<true>, dim3(grid), dim3(256), 32 * (e.feat_dim + 1) * 4, st, a, e.feat, e.feat_ld, e.feat_dim, Ft, p.Bh, p.ncols);
        } else {
            hipLaunchKernelGGL(enc_bwd_rows_kernel<false>, dim3(grid), dim3(256), 32 * (e.dim + 1) * 4, st, a, proj, de, g_es, dPt, p.Bh, p.ncols);
            hipLaunchKernelGGL(enc_gather_t_kernel<false>, dim3(grid), dim3(256), 32 * (e.feat_dim + 1) * 4, st, a, e.feat, e.feat_ld, e.feat_dim, Ft, p.Bh, p.ncols);
        }
    }
    // G[d, f] = dP^t[d, cols] . F^t[f, cols]^t over the head columns (M_H), then over the tail / negative columns (M_T)
    const int per = 32 / p.es;                             // slots per k-step
    for (int side = 0; side < 2; ++side) {
        const int64_t col0 = side == 0 ? 0 : p.Bh;
        const int ksteps = (side == 0 ? p.Bh : p.Th) / per, nsplit = side == 0 ? p.nsplit_h : p.nsplit_t;
        float *out = side == 0 ? g_mh : g_mt;
        const char *Ap = (const char *)dPt + col0 * p.es, *Bp = (const char *)Ft + col0 * p.es;
        if (nsplit > 0) {
            if (bf16) enc_launch_gemm<true>(Ap, p.ncols * p.es, nullptr, e.dim, Bp, p.ncols * p.es, e.feat_dim, part, e.feat_dim, mcount, ksteps, p.kps, nsplit, st);
            else      enc_launch_gemm<false>(Ap, p.ncols * p.es, nullptr, e.dim, Bp, p.ncols * p.es, e.feat_dim, part, e.feat_dim, mcount, ksteps, p.kps, nsplit, st);
        }
        hipLaunchKernelGGL(enc_split_reduce_kernel, dim3((unsigned)((mcount + 255) / 256)), dim3(256), 0, st, part, nsplit, mcount, out);
    }
    return kge_launch_status();
}
