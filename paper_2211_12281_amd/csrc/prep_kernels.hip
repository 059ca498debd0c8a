// Row-wise kernels around the block kernel: negative ids, gather + query build + positive score,
// gather of the shared negatives, transposes, per-row loss finish, chain rule of the query build.
#include "prep_kernels.h"
#include "row_ops.hpp"
#include "row_finish.hpp"

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void kge_philox_round(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c[0]), lo0 = 0xD2511F53u * c[0];
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c[2]), lo1 = 0xCD9E8D57u * c[2];
    const uint32_t n0 = hi1 ^ c[1] ^ k0, n2 = hi0 ^ c[3] ^ k1;
    c[0] = n0; c[1] = lo1; c[2] = n2; c[3] = lo0;
}

__global__ void kge_step_counter_add_kernel(uint64_t *counter, uint64_t inc) { *counter += inc; }

int kge_run_step_counter_add(uint64_t *counter, uint64_t inc, hipStream_t st) {
    hipLaunchKernelGGL(kge_step_counter_add_kernel, dim3(1), dim3(1), 0, st, counter, inc);
    return kge_launch_status();
}

__global__ void kge_negatives_kernel(uint32_t seed_lo, uint32_t seed_hi, uint32_t step, const uint64_t *step_counter,
                                     uint32_t tag, int64_t lo, uint64_t range, int64_t n, int32_t *out) {
    // one thread per Philox block = two ids
    const int64_t blk = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (2 * blk >= n) return;
    if (step_counter) step += (uint32_t)*step_counter;
    uint32_t c[4] = { (uint32_t)blk, (uint32_t)((uint64_t)blk >> 32), step, tag };
    uint32_t k0 = seed_lo, k1 = seed_hi;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        kge_philox_round(c, k0, k1);
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    const uint64_t x0 = ((uint64_t)c[1] << 32) | c[0], x1 = ((uint64_t)c[3] << 32) | c[2];
    out[2 * blk] = (int32_t)(lo + (int64_t)__umul64hi(x0, range));
    if (2 * blk + 1 < n) out[2 * blk + 1] = (int32_t)(lo + (int64_t)__umul64hi(x1, range));
}

int kge_run_negatives(uint64_t seed, uint64_t step, const uint64_t *step_counter, uint32_t tag, int64_t lo, int64_t hi,
                      int64_t n, int32_t *out, hipStream_t st) {
    const int64_t blocks = (n + 1) / 2;
    const int grid = (int)((blocks + 255) / 256);
    hipLaunchKernelGGL(kge_negatives_kernel, dim3(grid), dim3(256), 0, st, (uint32_t)seed,
                       (uint32_t)(seed >> 32), (uint32_t)step, step_counter, tag, lo, (uint64_t)(hi - lo), n, out);
    return kge_launch_status();
}

// id n of the draw that kge_negatives_kernel makes with these arguments (for the gather that draws its own ids)
__device__ __forceinline__ int32_t kge_negative_id(const KgeNegGen &q, uint32_t step, int64_t n) {
    const int64_t blk = n >> 1;
    uint32_t c[4] = { (uint32_t)blk, (uint32_t)((uint64_t)blk >> 32), step, q.tag };
    uint32_t k0 = q.seed_lo, k1 = q.seed_hi;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        kge_philox_round(c, k0, k1);
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    const uint64_t x = (n & 1) ? (((uint64_t)c[3] << 32) | c[2]) : (((uint64_t)c[1] << 32) | c[0]);
    return (int32_t)(q.lo + (int64_t)__umul64hi(x, q.range));
}

// ---------------------------------------------------------------------------------------------
// gather + query build + positive score (one wave per triple; rows >= B are written as zeros)
// ---------------------------------------------------------------------------------------------
struct KgeQbuildArgs {
    KgeModelDev m; const int32_t *h, *r, *t; int B, Bp, dp; void *Q, *W, *Q2; float *Q32, *W32; KgeRowInfo *rowinfo;
    float *pos_ws, *pos_out;
    _Float16 *planes;                  // optional: the two fp16 pieces of the scaled q, [2][Bp][dp], with W two more for the
                                       // unit normal (scaled by KGE_PLANE_UNIT_SCALE); then rowinfo.K = 1 / scale of the row
};
struct KgeTgatherArgs {
    const int32_t *neg; int N, Np; void *T; float *tn; _Float16 *planes; float *inv_scale; float *bias;
    KgeNegGen gen;                     // gen.out set: the ids are drawn here (and written to gen.out) instead of read from neg
};

// fp32 rows as TWO fp16 planes for the matrix cores: the row is scaled by a power of two s that brings its largest
// magnitude into [2^10, 2^11) (well inside the fp16 range, with the second piece of every element that matters still
// normal), then s x = x1 + x2 with x1 = fp16(s x), x2 = fp16(s x - x1): 22 significand bits, residual < 2^-22 s |x|.
// Plane p of element i at planes[p n + i]; the contraction is multiplied by the two rows' 1 / s afterwards (exact).
__device__ __forceinline__ float kge_plane_scale(float amax, float &inv) {
    if (!(amax > 0.f)) { inv = 1.f; return 1.f; }
    int e;
    (void)frexpf(amax, &e);                                 // amax = f 2^e, f in [0.5, 1)
    e = e < -100 ? -100 : (e > 100 ? 100 : e);
    inv = ldexpf(1.f, e - 11);
    return ldexpf(1.f, 11 - e);
}
__device__ __forceinline__ void kge_store_planes(_Float16 *planes, int64_t n, int64_t i, float xs) {
    const _Float16 x1 = (_Float16)xs;
    planes[i] = x1; planes[n + i] = (_Float16)(xs - (float)x1);
}

template <bool BF16, int SC>
__device__ __forceinline__ void kge_qbuild_body(int blk, const KgeQbuildArgs &a) {
    const KgeModelDev &m = a.m;
    const int32_t *h = a.h, *r = a.r, *t = a.t;
    const int B = a.B, Bp = a.Bp, dp = a.dp;
    void *Q = a.Q, *W = a.W, *Q2 = a.Q2; float *Q32 = a.Q32, *W32 = a.W32;
    KgeRowInfo *rowinfo = a.rowinfo; float *pos_ws = a.pos_ws, *pos_out = a.pos_out;
    const int lane = threadIdx.x & 63;
    const int b = blk * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (b >= Bp) return;
    if (b >= B) {
        for (int j = lane; j < dp; j += 64) {
            El<BF16>::st(Q, (int64_t)b * dp + j, 0.f);
            if (W) El<BF16>::st(W, (int64_t)b * dp + j, 0.f);
            if (Q2) El<BF16>::st(Q2, (int64_t)b * dp + j, 0.f);
            if (Q32) Q32[(int64_t)b * dp + j] = 0.f;
            if (W32) W32[(int64_t)b * dp + j] = 0.f;
            if (a.planes) kge_store_planes(a.planes, (int64_t)Bp * dp, (int64_t)b * dp + j, 0.f);
            if (a.planes && W) kge_store_planes(a.planes + 2 * (int64_t)Bp * dp, (int64_t)Bp * dp, (int64_t)b * dp + j, 0.f);
        }
        if (lane == 0) { rowinfo[b] = KgeRowInfo{0.f, 0.f, a.planes ? 1.f : 0.f, 0.f}; if (pos_ws) pos_ws[b] = 0.f; }
        return;
    }
    KgeRowCtx<BF16> cx;
    kge_build_query<BF16, SC>(m, h[b], r[b], lane, cx);
    const int d = m.dim;
    const int64_t toff = (int64_t)t[b] * m.ent_ld;
    float qn = 0.f, cq = 0.f, wn = 0.f, s_pos = 0.f, wt = 0.f;
    float tv[KGE_MAXJ];
    float q_scale = 1.f, q_inv = 0.f;
    if (a.planes) {
        float amax = 0.f;
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) amax = fmaxf(amax, fabsf(cx.q[k]));
        q_scale = kge_plane_scale(kge_wave_max(amax), q_inv);
    }
#pragma unroll
    for (int k = 0; k < KGE_MAXJ; ++k) {
        const int j = lane + 64 * k;
        const float tj = El<BF16>::ld(m.ent, toff + (j < d ? j : 0));
        tv[k] = j < d ? tj : 0.f;
        const float qr = El<BF16>::rnd(cx.q[k]), wr = El<BF16>::rnd(cx.w[k]);
        qn += qr * qr; cq += wr * qr; wn += wr * wr;          // norms of what the matrix cores will see
        wt += cx.w[k] * tv[k];
        if (j < dp) {
            El<BF16>::st(Q, (int64_t)b * dp + j, cx.q[k]);
            if (W) El<BF16>::st(W, (int64_t)b * dp + j, cx.w[k]);
            if (Q32) Q32[(int64_t)b * dp + j] = cx.q[k];      // unrounded copies for the 1-norm kernels
            if (W32) W32[(int64_t)b * dp + j] = cx.w[k];
            if (a.planes) kge_store_planes(a.planes, (int64_t)Bp * dp, (int64_t)b * dp + j, q_scale * cx.q[k]);
            if (a.planes && W)
                kge_store_planes(a.planes + 2 * (int64_t)Bp * dp, (int64_t)Bp * dp, (int64_t)b * dp + j, KGE_PLANE_UNIT_SCALE * cx.w[k]);
        }
    }
    qn = kge_wave_sum(qn);
    if (SC == KGE_TRANSH) { cq = kge_wave_sum(cq); wn = kge_wave_sum(wn); wt = kge_wave_sum(wt); }
    if (Q2) {   // TransH: q - c * w_hat, the operand of the negatives' gradient contraction
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) {
            const int j = lane + 64 * k;
            if (j < dp) El<BF16>::st(Q2, (int64_t)b * dp + j, El<BF16>::rnd(cx.q[k]) - cq * El<BF16>::rnd(cx.w[k]));
        }
    }
    // positive score by the direct formula (Table 2), fp32
#pragma unroll
    for (int k = 0; k < KGE_MAXJ; ++k) {
        if (SC == KGE_DISTMULT || SC == KGE_COMPLEX) s_pos += cx.q[k] * tv[k];
        else {
            float x = cx.q[k] - tv[k];
            if (SC == KGE_TRANSH) x += wt * cx.w[k];
            s_pos += m.p1 ? fabsf(x) : x * x;
        }
    }
    s_pos = kge_wave_sum(s_pos);
    if (!(SC == KGE_DISTMULT || SC == KGE_COMPLEX)) s_pos = m.p1 ? -s_pos : -sqrtf(s_pos);
    if (lane == 0) {
        rowinfo[b] = KgeRowInfo{qn, cq, q_inv, SC == KGE_TRANSH ? wn : 1.f};     // (K: set by the row finish when training)
        if (pos_ws) pos_ws[b] = s_pos;
        if (pos_out) pos_out[b] = s_pos;
    }
}

// ---------------------------------------------------------------------------------------------
// gather of the shared negatives: T[n] = ent[neg[n]], tn[n] = ||T[n]||^2 (zeros past N)
// ---------------------------------------------------------------------------------------------
// rows of the gathered block that one wave takes: a row of dp elements is covered by dp * ES / 16 lanes with 16 bytes
// each; 64 / (that, rounded up to a power of two) rows share a load instruction, and FOUR such loads are in flight per
// lane (a random row costs a full memory round trip: the bytes in flight bound the rate of the gather)
__host__ __device__ inline int kge_tgather_group_lanes(int dp, int es) {
    const int lpr = dp * es / 16;
    int gl = 1;
    while (gl < lpr) gl <<= 1;
    return gl < 64 ? gl : 64;
}
constexpr int KGE_TG_INFLIGHT = 4;                          // row loads in flight per lane
__host__ __device__ inline int kge_tgather_rows_per_wave(int dp, int es) { return KGE_TG_INFLIGHT * (64 / kge_tgather_group_lanes(dp, es)); }

template <bool BF16>
__device__ __forceinline__ void kge_tgather_body(int blk, const KgeModelDev &m, const int32_t *neg, int N, int Np, int dp, void *T,
                                                 float *tn, _Float16 *planes = nullptr, float *inv_scale = nullptr,
                                                 const KgeNegGen *gen = nullptr) {
    const int lane = threadIdx.x & 63;
    const bool draw = gen && gen->out;
    uint32_t step = 0;
    if (draw) { step = gen->step; if (gen->step_counter) step += (uint32_t)*gen->step_counter; }
    constexpr int ES = BF16 ? 2 : 4;
    const int lpr = dp * ES / 16;                           // lanes that cover a row with 16 bytes each
    const int gl = kge_tgather_group_lanes(dp, ES), rpl = 64 / gl, rpw = KGE_TG_INFLIGHT * rpl;
    const int nbase = (blk * (blockDim.x >> 6) + (threadIdx.x >> 6)) * rpw;
    if (nbase >= Np) return;
    if (m.dim == dp && lpr <= 64 && (m.ent_ld * ES) % 16 == 0 && ((uintptr_t)m.ent & 15) == 0) {
        // unpadded, 16-byte aligned rows: ONE load per lane and row, four rows (groups of rows) requested together
        const int grp = lane / gl, lg = lane % gl;
        uint4 v[KGE_TG_INFLIGHT];
        int64_t off[KGE_TG_INFLIGHT];
        // ids drawn here: lane l draws the id of row nbase + l % rpw (one Philox block per lane instead of one per row and
        // lane), the first rpw lanes write them out, and every lane fetches its rows' ids from the lanes that hold them
        int32_t mine = 0;
        if (draw) {
            const int n = nbase + lane % rpw;
            if (n < N) mine = kge_negative_id(*gen, step, n);
            if (lane < rpw && n < N) gen->out[n] = mine;
        }
#pragma unroll
        for (int u = 0; u < KGE_TG_INFLIGHT; ++u) {
            const int n = nbase + u * rpl + grp;
            int32_t id = 0;
            if (draw) id = __shfl(mine, u * rpl + grp);     // (every lane takes part)
            else if (n < N) id = neg[n];
            off[u] = n < N ? (int64_t)id * m.ent_ld : -1;
        }
#pragma unroll
        for (int u = 0; u < KGE_TG_INFLIGHT; ++u) {
            v[u] = make_uint4(0u, 0u, 0u, 0u);
            if (off[u] >= 0 && lg < lpr) v[u] = *(const uint4 *)((const char *)m.ent + off[u] * ES + lg * 16);
        }
#pragma unroll
        for (int u = 0; u < KGE_TG_INFLIGHT; ++u) {
            const int n = nbase + u * rpl + grp;
            const bool live = n < Np && lg < lpr;
            if (live) *(uint4 *)((char *)T + ((int64_t)n * dp) * ES + lg * 16) = v[u];
            const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
            float s = 0.f, amax = 0.f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if constexpr (BF16) {
                    const float a0 = __uint_as_float(w[k] << 16), a1 = __uint_as_float(w[k] & 0xffff0000u);
                    s += a0 * a0; s += a1 * a1;
                } else { const float a0 = __uint_as_float(w[k]); s += a0 * a0; amax = fmaxf(amax, fabsf(a0)); }
            }
            // sum (and largest magnitude) over the lanes of the row's group (fixed order)
#pragma unroll
            for (int o = 32; o > 0; o >>= 1)
                if (o < gl) { s += __shfl_xor(s, o); amax = fmaxf(amax, __shfl_xor(amax, o)); }
            if (lg == 0 && n < Np) tn[n] = s;
            if constexpr (!BF16) {
                if (planes) {
                    float inv;
                    const float sc = kge_plane_scale(amax, inv);
                    if (live) {                         // the lane's four elements: one 8-byte store per plane
                        typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                        h4 p1, p2;
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const float xs = sc * __uint_as_float(w[k]);
                            p1[k] = (_Float16)xs; p2[k] = (_Float16)(xs - (float)p1[k]);
                        }
                        _Float16 *dst = planes + (int64_t)n * dp + lg * 4;
                        *(h4 *)dst = p1; *(h4 *)(dst + (int64_t)Np * dp) = p2;
                    }
                    if (lg == 0 && n < Np) inv_scale[n] = inv;
                }
            }
        }
        return;
    }
    for (int u = 0; u < rpw; ++u) {
        const int n = nbase + u;
        if (n >= Np) break;                                 // (wave-uniform)
        int64_t off = 0;
        if (n < N) {
            const int32_t id = draw ? kge_negative_id(*gen, step, n) : neg[n];
            if (draw && lane == 0) gen->out[n] = id;
            off = (int64_t)id * m.ent_ld;
        }
        float s = 0.f, amax = 0.f;
        for (int j = lane; j < dp; j += 64) {
            float v = (n < N && j < m.dim) ? El<BF16>::ld(m.ent, off + j) : 0.f;
            El<BF16>::st(T, (int64_t)n * dp + j, v);
            s += v * v; amax = fmaxf(amax, fabsf(v));
        }
        s = kge_wave_sum(s);
        if (lane == 0) tn[n] = s;
        if (!BF16 && planes) {                              // (second walk over the row, now that its scale is known)
            float inv;
            const float sc = kge_plane_scale(kge_wave_max(amax), inv);
            for (int j = lane; j < dp; j += 64) {
                const float v = (n < N && j < m.dim) ? El<BF16>::ld(m.ent, off + j) : 0.f;
                kge_store_planes(planes, (int64_t)Np * dp, (int64_t)n * dp + j, sc * v);
            }
            if (lane == 0) inv_scale[n] = inv;
        }
    }
}
template <bool BF16>
__global__ void kge_tgather_kernel(KgeModelDev m, const int32_t *neg, int N, int Np, int dp, void *T, float *tn, _Float16 *planes,
                                   float *inv_scale) {
    kge_tgather_body<BF16>(blockIdx.x, m, neg, N, Np, dp, T, tn, planes, inv_scale);
}
template <bool BF16, int SC>
__global__ void kge_qbuild_kernel(KgeQbuildArgs a) { kge_qbuild_body<BF16, SC>(blockIdx.x, a); }
// query build and gather of the negatives in ONE launch (the first q_blocks workgroups build queries): the two are
// independent, and a launch of their own each would cost the second one's start-up on the critical path
template <bool BF16, int SC>
__global__ void kge_qbuild_tgather_kernel(int q_blocks, KgeQbuildArgs a, KgeTgatherArgs g) {
    if (g.bias)                                                         // 0 for the negatives, -inf for the padding rows behind them
        for (int n = blockIdx.x * blockDim.x + threadIdx.x; n < g.Np; n += gridDim.x * blockDim.x) g.bias[n] = n < g.N ? 0.f : -INFINITY;
    if ((int)blockIdx.x < q_blocks) kge_qbuild_body<BF16, SC>(blockIdx.x, a);
    else kge_tgather_body<BF16>(blockIdx.x - q_blocks, a.m, g.neg, g.N, g.Np, a.dp, g.T, g.tn, g.planes, g.inv_scale, &g.gen);
}

// gather of the shared negatives AND their transposed copy in one launch: a workgroup takes 32 negatives, every
// wave 8 of them (all of a lane's loads are issued before the first is used), the rows pass through the LDS
// and leave again as the 32-entry segments of the dp rows of Tt (bf16: with the column permutation of
// kge_transpose_kernel).  NJ = dp / 64.
template <bool BF16, int NJ>
__global__ __launch_bounds__(256) void kge_tgather_t_kernel(KgeModelDev m, const int32_t *neg, int N, int Np, void *T, void *Tt,
                                                            float *tn) {
    using E = typename El<BF16>::T;
    constexpr int DP = 64 * NJ, PITCH = DP + (BF16 ? 2 : 1);           // odd stride in 4-byte words
    extern __shared__ __attribute__((aligned(16))) char tg_lds[];
    E *tile = (E *)tg_lds;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n0 = blockIdx.x * 32;
    float v[8][NJ];
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
        const int n = n0 + wave * 8 + rr;
        const int64_t off = n < N ? (int64_t)neg[n] * m.ent_ld : 0;
#pragma unroll
        for (int k = 0; k < NJ; ++k) {
            const int j = lane + 64 * k;
            const float x = El<BF16>::ld(m.ent, off + (j < m.dim ? j : 0));
            v[rr][k] = (n < N && j < m.dim) ? x : 0.f;
        }
    }
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
        const int row = wave * 8 + rr, n = n0 + row;
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < NJ; ++k) {
            const int j = lane + 64 * k;
            El<BF16>::st(T, (int64_t)n * DP + j, v[rr][k]);
            tile[row * PITCH + j] = (E)v[rr][k];
            s += v[rr][k] * v[rr][k];
        }
        s = kge_wave_sum(s);
        if (lane == 0) tn[n] = s;
    }
    __syncthreads();
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int px = BF16 ? ((tx & ~12) | ((tx & 4) << 1) | ((tx & 8) >> 1)) : tx;
    for (int c = ty; c < DP; c += 8) ((E *)Tt)[(int64_t)c * Np + n0 + px] = tile[tx * PITCH + c];
}

// ---------------------------------------------------------------------------------------------
// transpose: src [R][C] -> dst [C][R]   (R, C multiples of 32; elements of 2 or 4 bytes).
// PERM: inside every group of 16 source rows, bits 2 and 3 of the row number are swapped in the
// destination column, which makes the 8 entries that one lane half of the block kernel contracts in
// its second phase contiguous (one 16-byte fragment for 2-byte elements).
// ---------------------------------------------------------------------------------------------
template <typename T, bool PERM>
__global__ void kge_transpose_kernel(const T *src, T *dst, int R, int C) {
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 256 threads: 32 x 8
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    for (int i = ty; i < 32; i += 8) tile[i][tx] = src[(int64_t)(r0 + i) * C + c0 + tx];
    __syncthreads();
    const int px = PERM ? ((tx & ~12) | ((tx & 4) << 1) | ((tx & 8) >> 1)) : tx;
    for (int i = ty; i < 32; i += 8) dst[(int64_t)(c0 + i) * R + r0 + px] = tile[tx][i];
}

__global__ void kge_rowfinish_kernel(const float4 *stat_part, int nsplit, int Bp, int B, int N, int loss,
                                     float gamma, float c_corr, float scale, const float *pos,
                                     KgeRowInfo *rowinfo, float *lossb, float *gpos) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= Bp) return;
    if (b >= B) { lossb[b] = 0.f; gpos[b] = 0.f; rowinfo[b].K = -INFINITY; return; }
    const KgeRowFinish o = kge_rowfinish_row(stat_part, nsplit, Bp, b, N, loss, gamma, c_corr, scale, pos[b]);
    lossb[b] = o.L; gpos[b] = o.gp; rowinfo[b].K = o.K;
}

__global__ void kge_rowfinish_qscale_kernel(KgeRowFinishQArgs a) { kge_rowfinish_qscale_body(blockIdx.x, a); }

// loss_out = scale * sum_b lossb[b], one workgroup, fixed summation tree
__device__ __forceinline__ void kge_loss_reduce_body(const float *lossb, int B, float scale, float *loss_out) {
    __shared__ double sh[256];
    double s = 0.0;
    for (int b = threadIdx.x; b < B; b += 256) s += (double)lossb[b];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss_out = (float)(sh[0] * (double)scale);
}
__global__ void kge_loss_reduce_kernel(const float *lossb, int B, float scale, float *loss_out) {
    kge_loss_reduce_body(lossb, B, scale, loss_out);
}

// ---------------------------------------------------------------------------------------------
// chain rule of the query build + positive triple: one wave per triple
// ---------------------------------------------------------------------------------------------
// (the scorer is a template parameter: with a run-time switch every load of this kernel sat in its own branch
// and was waited for on its own)
struct KgeChainArgs {
    KgeModelDev m; const int32_t *h, *r, *t; int B, Bp, dp; const float *acc_part, *acc_part2; const float4 *sum_part, *stat_part;
    const KgeRowInfo *rowinfo; int nsplit; const float *gpos; float *g_ent, *g_rel, *g_relw; int32_t *g_ent_idx, *g_rel_idx;
    float reg; float *regv;
};
struct KgeTfinishArgs {
    const float *accT_part; const float4 *sumT_part; int nsplit, Np, N, dp, d, dist_kind; const void *T; const int32_t *neg;
    float *g_neg; int32_t *g_neg_idx; const void *ent; int64_t ent_ld; float reg; float *regn;
};

// PB: the partials of the queries' gradient rows are bf16 in the paired-column words that the forward pass of
// block_sym.hip writes (word lane + 64 kk of a row: columns lane + 128 kk and lane + 64 + 128 kk; rows of 256 columns)
template <bool BF16, int SC, bool PB = false>
__device__ __forceinline__ void kge_chain_body(int blk, const KgeChainArgs &a) {
    const KgeModelDev &m = a.m;
    const int32_t *h = a.h, *r = a.r, *t = a.t;
    const int B = a.B, Bp = a.Bp, dp = a.dp, nsplit = a.nsplit;
    const float *acc_part = a.acc_part, *acc_part2 = a.acc_part2, *gpos = a.gpos;
    const float4 *sum_part = a.sum_part, *stat_part = a.stat_part;
    const KgeRowInfo *rowinfo = a.rowinfo;
    float *g_ent = a.g_ent, *g_rel = a.g_rel, *g_relw = a.g_relw, *regv = a.regv;
    int32_t *g_ent_idx = a.g_ent_idx, *g_rel_idx = a.g_rel_idx;
    const float reg = a.reg;
    const int lane = threadIdx.x & 63;
    const int b = blk * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (b >= B) return;
    const int d = m.dim, c = d >> 1;
    KgeRowCtx<BF16> cx;
    kge_build_query<BF16, SC>(m, h[b], r[b], lane, cx);
    const int64_t toff = (int64_t)t[b] * m.ent_ld;
    const float gp = gpos[b];
    // the row pass leaves, per split, sums of UNNORMALISED weights relative to that split's running
    // maximum m_s; exp2(m_s + K) turns them into gradient coefficients
    const float K2 = rowinfo[b].K;
    // (the vector-pipe kernels apply the finished coefficients themselves: their partials are summed as they are)
    auto kappa = [&](int s) {
        if (m.vec) return 1.f;
        const float ms = stat_part[(size_t)s * Bp + b].x;
        return ms > -INFINITY ? exp2f(ms + K2) : 0.f;
    };
    // The partials of four splits are requested together (the wave would otherwise wait for one row of one split
    // at a time) and then added in split order: the sums do not depend on the grouping.
    float s1 = 0.f, s2 = 0.f, s3 = 0.f;
    float a1[KGE_MAXJ], a2[KGE_MAXJ], tv[KGE_MAXJ], dq[KGE_MAXJ], dtp[KGE_MAXJ];
    float wt = 0.f;
#pragma unroll
    for (int k = 0; k < KGE_MAXJ; ++k) {
        const int j = lane + 64 * k;
        a1[k] = a2[k] = 0.f;
        const float tj = El<BF16>::ld(m.ent, toff + (j < d ? j : 0));
        tv[k] = j < d ? tj : 0.f;
        wt += cx.w[k] * tv[k];
    }
    for (int s0 = 0; s0 < nsplit; s0 += 4) {
        float kap[4], v1[4][KGE_MAXJ], v2[4][KGE_MAXJ];
        float4 p[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int s = s0 + u < nsplit ? s0 + u : nsplit - 1;      // past the end: the last split again, weight 0
            kap[u] = s0 + u < nsplit ? kappa(s) : 0.f;
            p[u] = m.vec ? make_float4(0.f, 0.f, 0.f, 0.f) : sum_part[(size_t)s * Bp + b];
#pragma unroll
            for (int k = 0; k < KGE_MAXJ; ++k) {
                v1[u][k] = v2[u][k] = 0.f;
                if constexpr (PB) continue;
                if (64 * k >= dp) continue;                // wave-uniform: the partial rows are dp columns long
                v1[u][k] = acc_part[((size_t)s * Bp + b) * dp + lane + 64 * k];
                if (SC == KGE_TRANSH) v2[u][k] = acc_part2[((size_t)s * Bp + b) * dp + lane + 64 * k];
            }
            if constexpr (PB) {
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const uint32_t w = ((const uint32_t *)acc_part)[((size_t)s * Bp + b) * 128 + lane + 64 * kk];
                    v1[u][2 * kk] = __uint_as_float(w << 16); v1[u][2 * kk + 1] = __uint_as_float(w & 0xFFFF0000u);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            s1 += kap[u] * p[u].x; s2 += kap[u] * p[u].y; s3 += kap[u] * p[u].z;
#pragma unroll
            for (int k = 0; k < KGE_MAXJ; ++k) { a1[k] += kap[u] * v1[u][k]; a2[k] += kap[u] * v2[u][k]; }
        }
    }
    const bool mult = SC == KGE_DISTMULT || SC == KGE_COMPLEX;
    float dwh[KGE_MAXJ];
    if (mult) {
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) { dq[k] = a1[k] + gp * tv[k]; dtp[k] = gp * cx.q[k]; }
    } else {
        if (SC == KGE_TRANSH) wt = kge_wave_sum(wt);
        float u[KGE_MAXJ], d2 = 0.f;
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) {
            u[k] = cx.q[k] - tv[k] + (SC == KGE_TRANSH ? wt * cx.w[k] : 0.f);
            d2 += u[k] * u[k];
        }
        d2 = kge_wave_sum(d2);
        const float dist = sqrtf(d2);
        const float ap = dist > 0.f ? -gp / dist : 0.f;            // gp * df/du = ap * u
        // positive triple: gp * df/du_k, df/du = -u / ||u||_2, or -sign(u) for the 1-norm
        auto pos_term = [&](int k) { return m.p1 ? (u[k] > 0.f ? -gp : (u[k] < 0.f ? gp : 0.f)) : ap * u[k]; };
        float aw = 0.f, cq = 0.f;
        if (SC == KGE_TRANSH) {
#pragma unroll
            for (int k = 0; k < KGE_MAXJ; ++k) { aw += pos_term(k) * cx.w[k]; cq += cx.w[k] * cx.q[k]; }
            aw = kge_wave_sum(aw); cq = kge_wave_sum(cq);
        }
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) {
            const float apu = pos_term(k);
            dq[k] = a1[k] - s1 * cx.q[k] + apu;
            dtp[k] = -apu;
            if (SC == KGE_TRANSH) {
                dq[k] -= s2 * cx.w[k];
                dtp[k] = -(apu - aw * cx.w[k]);
                // gradient with respect to the unit normal: negatives' part + positive's part
                // (vector-pipe kernels: a2 is the finished negatives' part, the sums s1..s3 are zero)
                dwh[k] = (m.vec ? 0.f : -cq * a1[k]) - s2 * cx.q[k] + a2[k] - s3 * cx.w[k] + aw * tv[k] + wt * apu;
            }
        }
    }
    // dq -> dh, dr (and dw)
    float wdq = 0.f;
    if (SC == KGE_TRANSH) {
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) wdq += cx.w[k] * dq[k];
        wdq = kge_wave_sum(wdq);
        float wdw = 0.f;
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) { dwh[k] += -cx.wh * dq[k] - wdq * cx.h[k]; wdw += cx.w[k] * dwh[k]; }
        wdw = kge_wave_sum(wdw);
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) dwh[k] = (dwh[k] - cx.w[k] * wdw) / cx.wnorm;
    }
    float *gh = g_ent + (int64_t)b * d, *gt = g_ent + (int64_t)(B + b) * d;
    const int k_rel = m.rel_dim;
    float *gr = g_rel + (int64_t)b * k_rel;
    // complex scorers need the partner component of dq, held by another lane: exchange through LDS
    if (SC == KGE_COMPLEX || SC == KGE_ROTATE) {
        __shared__ float xch[4][KGE_MAXJ * 64];
        float *tmp = xch[threadIdx.x >> 6];
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) tmp[lane + 64 * k] = dq[k];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) {
            const int j = lane + 64 * k;
            if (j >= d) continue;
            const bool re = j < c;
            const int jp = re ? j + c : j - c;
            const float dq_re = re ? dq[k] : tmp[jp], dq_im = re ? tmp[jp] : dq[k];
            const float h_re = re ? cx.h[k] : El<BF16>::ld(m.ent, (int64_t)h[b] * m.ent_ld + jp);
            const float h_im = re ? El<BF16>::ld(m.ent, (int64_t)h[b] * m.ent_ld + jp) : cx.h[k];
            if (SC == KGE_COMPLEX) {
                const float r_re = re ? cx.r[k] : El<BF16>::ld(m.rel, (int64_t)r[b] * m.rel_ld + jp);
                const float r_im = re ? El<BF16>::ld(m.rel, (int64_t)r[b] * m.rel_ld + jp) : cx.r[k];
                gh[j] = re ? dq_re * r_re + dq_im * r_im : -dq_re * r_im + dq_im * r_re;
                gr[j] = re ? dq_re * h_re + dq_im * h_im : -dq_re * h_im + dq_im * h_re;
            } else {
                float sn, cs; sincosf(cx.r[k], &sn, &cs);
                gh[j] = re ? dq_re * cs + dq_im * sn : -dq_re * sn + dq_im * cs;
                if (re) {
                    const float q_re = cx.q[k], q_im = h_re * sn + h_im * cs;
                    gr[j] = -dq_re * q_im + dq_im * q_re;
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < KGE_MAXJ; ++k) {
        const int j = lane + 64 * k;
        if (j >= d) continue;
        gt[j] = dtp[k];
        if constexpr (SC == KGE_TRANSE) { gh[j] = dq[k]; gr[j] = dq[k]; }
        if constexpr (SC == KGE_DISTMULT) { gh[j] = dq[k] * cx.r[k]; gr[j] = dq[k] * cx.h[k]; }
        if constexpr (SC == KGE_TRANSH) { gh[j] = dq[k] - wdq * cx.w[k]; gr[j] = dq[k]; g_relw[(int64_t)b * d + j] = dwh[k]; }
    }
    if (lane == 0) { g_ent_idx[b] = h[b]; g_ent_idx[B + b] = t[b]; g_rel_idx[b] = r[b]; }
    if (reg > 0.f) {
        // L3 regulariser of the head and tail rows (Section 3.1, Regularisation): reg * ||x||_3 joins the loss,
        // reg * sign(x_j) x_j^2 / ||x||_3^2 the gradient of the slot (every lane re-reads what it wrote above)
        float ch = 0.f, ct = 0.f;
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) { ch += fabsf(cx.h[k]) * cx.h[k] * cx.h[k]; ct += fabsf(tv[k]) * tv[k] * tv[k]; }
        const float nh = cbrtf(kge_wave_sum(ch)), nt = cbrtf(kge_wave_sum(ct));
        const float fh = nh > 0.f ? reg / (nh * nh) : 0.f, ft = nt > 0.f ? reg / (nt * nt) : 0.f;
#pragma unroll
        for (int k = 0; k < KGE_MAXJ; ++k) {
            const int j = lane + 64 * k;
            if (j >= d) continue;
            gh[j] += fh * fabsf(cx.h[k]) * cx.h[k];
            gt[j] += ft * fabsf(tv[k]) * tv[k];
        }
        if (lane == 0) { regv[b] = nh; regv[Bp + b] = nt; }
    }
}

// gradient rows of the shared negatives: sum of the split partials minus colsum * t (distances), plus
// the L3 regulariser of the row (read from the table itself, so it is there without a scored block)
// PB: the split partials are bf16 rows in column order (block_gradp.hip)
template <bool BF16, bool PB = false>
__device__ __forceinline__ void kge_tfinish_body(int blk, const KgeTfinishArgs &a) {
    const float *accT_part = a.accT_part; const float4 *sumT_part = a.sumT_part;
    const int nsplit = a.nsplit, Np = a.Np, N = a.N, dp = a.dp, d = a.d, dist_kind = a.dist_kind;
    const void *T = a.T, *ent = a.ent; const int32_t *neg = a.neg;
    float *g_neg = a.g_neg, *regn = a.regn; int32_t *g_neg_idx = a.g_neg_idx;
    const int64_t ent_ld = a.ent_ld; const float reg = a.reg;
    const int lane = threadIdx.x & 63;
    const int n = blk * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (n >= N) return;
    float cs = 0.f;
    if (dist_kind)
        for (int s = 0; s < nsplit; ++s) cs += sumT_part[(size_t)s * Np + n].x;
    // A lane takes FOUR consecutive columns per step (d is a multiple of 4: a group lies inside the row or past its end),
    // so that a partial row is one 16-byte load per lane.  The row itself is read once (from the gathered copy when
    // there is one, else from the table) and kept in registers.
    constexpr int NG = KGE_MAXJ / 4;                        // column groups per lane
    static_assert(KGE_MAXJ % 4 == 0, "four columns per lane and step");
    float x[NG][4], f = 0.f;
    const bool need_row = reg > 0.f || dist_kind;
    const int64_t rbase = T ? (int64_t)n * dp : (int64_t)neg[n] * ent_ld;
    const void *rsrc = T ? T : ent;
#pragma unroll
    for (int k = 0; k < NG; ++k) {
        const int j = 4 * (lane + 64 * k);
#pragma unroll
        for (int e = 0; e < 4; ++e) x[k][e] = (need_row && j < d) ? El<BF16>::ld(rsrc, rbase + j + e) : 0.f;
    }
    if (reg > 0.f) {
        float c3 = 0.f;
#pragma unroll
        for (int k = 0; k < NG; ++k)
#pragma unroll
            for (int e = 0; e < 4; ++e) c3 += fabsf(x[k][e]) * x[k][e] * x[k][e];
        const float nrm = cbrtf(kge_wave_sum(c3));
        f = nrm > 0.f ? reg / (nrm * nrm) : 0.f;
        if (lane == 0) regn[n] = nrm;
    }
    const bool out16 = ((uintptr_t)g_neg & 15) == 0;        // (d is a multiple of 4: rows of an aligned base are aligned)
#pragma unroll
    for (int k = 0; k < NG; ++k) {
        const int j = 4 * (lane + 64 * k);
        if (j >= d) continue;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        // two splits are requested together, then added in split order
        for (int s0 = 0; s0 < nsplit; s0 += 2) {
            const bool two = s0 + 1 < nsplit;
            float4 p0, p1 = make_float4(0.f, 0.f, 0.f, 0.f);
            if constexpr (PB) {
                const uint16_t *pb = (const uint16_t *)accT_part;
                const uint2 w0 = *(const uint2 *)(pb + ((size_t)s0 * Np + n) * dp + j);
                const uint2 w1 = two ? *(const uint2 *)(pb + ((size_t)(s0 + 1) * Np + n) * dp + j) : make_uint2(0u, 0u);
                p0 = make_float4(__uint_as_float(w0.x << 16), __uint_as_float(w0.x & 0xFFFF0000u), __uint_as_float(w0.y << 16), __uint_as_float(w0.y & 0xFFFF0000u));
                p1 = make_float4(__uint_as_float(w1.x << 16), __uint_as_float(w1.x & 0xFFFF0000u), __uint_as_float(w1.y << 16), __uint_as_float(w1.y & 0xFFFF0000u));
            } else {
                p0 = *(const float4 *)(accT_part + ((size_t)s0 * Np + n) * dp + j);
                if (two) p1 = *(const float4 *)(accT_part + ((size_t)(s0 + 1) * Np + n) * dp + j);
            }
            v[0] += p0.x; v[1] += p0.y; v[2] += p0.z; v[3] += p0.w;
            if (two) { v[0] += p1.x; v[1] += p1.y; v[2] += p1.z; v[3] += p1.w; }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (dist_kind) v[e] -= cs * x[k][e];
            if (reg > 0.f) v[e] += f * fabsf(x[k][e]) * x[k][e];
        }
        float *dst = g_neg + (int64_t)n * d + j;
        if (out16) *(float4 *)dst = make_float4(v[0], v[1], v[2], v[3]);
        else { dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3]; }
    }
    if (lane == 0) g_neg_idx[n] = neg[n];
}
template <bool BF16>
__global__ void kge_tfinish_kernel(KgeTfinishArgs a) { kge_tfinish_body<BF16>(blockIdx.x, a); }
template <bool BF16, int SC>
__global__ __launch_bounds__(256) void kge_chain_kernel(KgeChainArgs a) { kge_chain_body<BF16, SC>(blockIdx.x, a); }
// both finishing kernels in ONE launch (the first chain_blocks workgroups run the chain rule of the queries): they
// read different partials and write different gradient rows
template <bool BF16, int SC, bool PB = false>
__global__ __launch_bounds__(256) void kge_chain_tfinish_kernel(int chain_blocks, KgeChainArgs c, KgeTfinishArgs t, const float *lossb, float scale,
                                         float *loss_out) {
    // (workgroup 0: the loss of the batch from the rows' losses, the reduction that would otherwise be a launch
    // of its own between the two passes)
    if (blockIdx.x == 0) kge_loss_reduce_body(lossb, c.B, scale, loss_out);
    else if ((int)blockIdx.x <= chain_blocks) kge_chain_body<BF16, SC, PB>(blockIdx.x - 1, c);
    else kge_tfinish_body<BF16, PB>(blockIdx.x - 1 - chain_blocks, t);
}

// loss += reg * (sum of the L3 norms of the 2B + N gathered slots): one workgroup of 1024 threads, fixed
// summation order (eight interleaved partial sums per thread keep the loads in flight, then a tree)
__global__ void kge_reg_add_kernel(const float *regv, int B, int Bp, int N, float reg, float *loss_out) {
    __shared__ double sh[1024];
    double p[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    auto add_range = [&](const float *v, int n) {
        for (int i0 = threadIdx.x; i0 < n; i0 += 8 * 1024) {
#pragma unroll
            for (int u = 0; u < 8; ++u) { const int i = i0 + u * 1024; p[u] += i < n ? (double)v[i] : 0.0; }
        }
    };
    add_range(regv, B);
    add_range(regv + Bp, B);
    add_range(regv + 2 * (size_t)Bp, N);
    sh[threadIdx.x] = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if (threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss_out = (float)((double)*loss_out + (double)reg * sh[0]);
}

__global__ void kge_zero_rows_kernel(float *p, int64_t count) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0.f;
}

// ---------------------------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------------------------
#define KGE_SC_SWITCH(BF, LAUNCH)                          \
    switch (m.scorer) {                                   \
    case KGE_TRANSE: LAUNCH(BF, KGE_TRANSE); break;       \
    case KGE_TRANSH: LAUNCH(BF, KGE_TRANSH); break;       \
    case KGE_ROTATE: LAUNCH(BF, KGE_ROTATE); break;       \
    case KGE_DISTMULT: LAUNCH(BF, KGE_DISTMULT); break;   \
    case KGE_COMPLEX: LAUNCH(BF, KGE_COMPLEX); break;     \
    default: return KGE_E_INVALID_ARG;                    \
    }

int kge_run_qbuild(const KgeModelDev &m, const int32_t *h, const int32_t *r, const int32_t *t, int B, int Bp,
                   int dp, void *Q, void *W, void *Q2, float *Q32, float *W32, KgeRowInfo *rowinfo, float *pos_ws,
                   float *pos_out, hipStream_t st, void *planes) {
    const int grid = (Bp + 3) / 4;
    if (grid == 0) return KGE_OK;
    const KgeQbuildArgs a{m, h, r, t, B, Bp, dp, Q, W, Q2, Q32, W32, rowinfo, pos_ws, pos_out, (_Float16 *)planes};
#define KGE_QBUILD(BF, SC) hipLaunchKernelGGL((kge_qbuild_kernel<BF, SC>), dim3(grid), dim3(256), 0, st, a)
    if (m.bf16) { KGE_SC_SWITCH(true, KGE_QBUILD) } else { KGE_SC_SWITCH(false, KGE_QBUILD) }
#undef KGE_QBUILD
    return kge_launch_status();
}

// kge_run_qbuild and kge_run_tgather as one launch (both Bp > 0 and Np > 0)
int kge_run_qbuild_tgather(const KgeModelDev &m, const int32_t *h, const int32_t *r, const int32_t *t, int B, int Bp,
                           int dp, void *Q, void *W, void *Q2, float *Q32, float *W32, KgeRowInfo *rowinfo, float *pos_ws,
                           const int32_t *neg, int N, int Np, void *T, float *tn, hipStream_t st, float *pos_out,
                           void *q_planes, void *t_planes, float *t_inv_scale, float *bias, const KgeNegGen *gen) {
    const int rows_wg = 4 * kge_tgather_rows_per_wave(dp, m.bf16 ? 2 : 4);
    const int qb = (Bp + 3) / 4, tb = (Np + rows_wg - 1) / rows_wg;
    if (qb == 0 || tb == 0 || ((q_planes || t_planes) && m.bf16) || (t_planes && !t_inv_scale)) return KGE_E_INVALID_ARG;
    const KgeQbuildArgs a{m, h, r, t, B, Bp, dp, Q, W, Q2, Q32, W32, rowinfo, pos_ws, pos_out, (_Float16 *)q_planes};
    const KgeTgatherArgs g{neg, N, Np, T, tn, (_Float16 *)t_planes, t_inv_scale, bias, gen ? *gen : KgeNegGen{}};
#define KGE_QT(BF, SC) hipLaunchKernelGGL((kge_qbuild_tgather_kernel<BF, SC>), dim3(qb + tb), dim3(256), 0, st, qb, a, g)
    if (m.bf16) { KGE_SC_SWITCH(true, KGE_QT) } else { KGE_SC_SWITCH(false, KGE_QT) }
#undef KGE_QT
    return kge_launch_status();
}

int kge_run_tgather(const KgeModelDev &m, const int32_t *neg, int N, int Np, int dp, void *T, float *tn, hipStream_t st, void *planes,
                    float *inv_scale) {
    const int rows_wg = 4 * kge_tgather_rows_per_wave(dp, m.bf16 ? 2 : 4);
    const int grid = (Np + rows_wg - 1) / rows_wg;
    if (grid == 0) return KGE_OK;
    if (planes && (m.bf16 || !inv_scale)) return KGE_E_INVALID_ARG;
    if (m.bf16) hipLaunchKernelGGL(kge_tgather_kernel<true>, dim3(grid), dim3(256), 0, st, m, neg, N, Np, dp, T, tn, (_Float16 *)nullptr, (float *)nullptr);
    else        hipLaunchKernelGGL(kge_tgather_kernel<false>, dim3(grid), dim3(256), 0, st, m, neg, N, Np, dp, T, tn, (_Float16 *)planes, inv_scale);
    return kge_launch_status();
}

int kge_run_tgather_t(const KgeModelDev &m, const int32_t *neg, int N, int Np, int dp, void *T, void *Tt, float *tn,
                      hipStream_t st) {
    if (Np == 0) return KGE_OK;
    if (Np % 32 || (dp != 128 && dp != 256 && dp != 512)) return KGE_E_INVALID_ARG;
    const int grid = Np / 32;
#define KGE_TG(BF, NJ) hipLaunchKernelGGL((kge_tgather_t_kernel<BF, NJ>), dim3(grid), dim3(256), 32 * (64 * NJ + (BF ? 2 : 1)) * (BF ? 2 : 4), st, \
                                          m, neg, N, Np, T, Tt, tn)
    if (m.bf16) { if (dp == 128) KGE_TG(true, 2); else if (dp == 256) KGE_TG(true, 4); else KGE_TG(true, 8); }
    else        { if (dp == 128) KGE_TG(false, 2); else if (dp == 256) KGE_TG(false, 4); else return KGE_E_INVALID_ARG; }   // fp32 rows: 512 or 1,024 bytes
#undef KGE_TG
    return kge_launch_status();
}

int kge_run_transpose(const void *src, void *dst, int R, int C, bool bf16, hipStream_t st) {
    if (R == 0 || C == 0) return KGE_OK;
    dim3 grid(C / 32, R / 32);
    if (bf16) hipLaunchKernelGGL((kge_transpose_kernel<uint16_t, true>), grid, dim3(256), 0, st, (const uint16_t *)src, (uint16_t *)dst, R, C);
    else      hipLaunchKernelGGL((kge_transpose_kernel<uint32_t, false>), grid, dim3(256), 0, st, (const uint32_t *)src, (uint32_t *)dst, R, C);
    return kge_launch_status();
}

int kge_run_rowfinish(const float4 *stat_part, int nsplit, int Bp, int B, int N, int loss, float gamma,
                      float c_corr, float scale, const float *pos, KgeRowInfo *rowinfo, float *lossb,
                      float *gpos, float *loss_out, hipStream_t st) {
    if (Bp > 0)
        hipLaunchKernelGGL(kge_rowfinish_kernel, dim3((Bp + 255) / 256), dim3(256), 0, st, stat_part, nsplit, Bp, B, N,
                           loss, gamma, c_corr, scale, pos, rowinfo, lossb, gpos);
    if (loss_out) hipLaunchKernelGGL(kge_loss_reduce_kernel, dim3(1), dim3(256), 0, st, lossb, B, scale, loss_out);
    return kge_launch_status();
}

int kge_run_rowfinish_qscale(const float4 *stat_part, int nsplit, int Bp, int B, int N, int loss, float gamma, float c_corr,
                              float scale, const float *pos, KgeRowInfo *rowinfo, float *lossb, float *gpos, const void *Q,
                              void *Qs, hipStream_t st) {
    if (Bp > 0) {
        const KgeRowFinishQArgs a{stat_part, nsplit, Bp, B, N, loss, gamma, c_corr, scale, pos, rowinfo, lossb, gpos,
                                  (const uint16_t *)Q, (uint16_t *)Qs};
        hipLaunchKernelGGL(kge_rowfinish_qscale_kernel, dim3((Bp + 3) / 4), dim3(256), 0, st, a);
    }
    return kge_launch_status();
}

int kge_run_chain(const KgeModelDev &m, const int32_t *h, const int32_t *r, const int32_t *t, int B, int Bp, int dp,
                  const float *acc_part, const float *acc_part2, const float4 *sum_part, const float4 *stat_part,
                  const KgeRowInfo *rowinfo, int nsplit, const float *gpos, float *g_ent, float *g_rel,
                  float *g_relw, int32_t *g_ent_idx, int32_t *g_rel_idx, float reg, float *regv, hipStream_t st) {
    if (B == 0) return KGE_OK;
    const int grid = (B + 3) / 4;
    const KgeChainArgs a{m, h, r, t, B, Bp, dp, acc_part, acc_part2, sum_part, stat_part, rowinfo, nsplit, gpos,
                         g_ent, g_rel, g_relw, g_ent_idx, g_rel_idx, reg, regv};
#define KGE_CHAIN(BF, SC) hipLaunchKernelGGL((kge_chain_kernel<BF, SC>), dim3(grid), dim3(256), 0, st, a)
    if (m.bf16) { KGE_SC_SWITCH(true, KGE_CHAIN) } else { KGE_SC_SWITCH(false, KGE_CHAIN) }
#undef KGE_CHAIN
    return kge_launch_status();
}

int kge_run_tfinish(const float *accT_part, const float4 *sumT_part, int nsplit, int Np, int N, int dp, int d,
                    int dist_kind, const void *T, bool bf16, const int32_t *neg, float *g_neg, int32_t *g_neg_idx,
                    const void *ent, int64_t ent_ld, float reg, float *regn, hipStream_t st) {
    if (N == 0) return KGE_OK;
    const int grid = (N + 3) / 4;
    const KgeTfinishArgs a{accT_part, sumT_part, nsplit, Np, N, dp, d, dist_kind, T, neg, g_neg, g_neg_idx, ent, ent_ld, reg, regn};
    if (bf16) hipLaunchKernelGGL(kge_tfinish_kernel<true>, dim3(grid), dim3(256), 0, st, a);
    else      hipLaunchKernelGGL(kge_tfinish_kernel<false>, dim3(grid), dim3(256), 0, st, a);
    return kge_launch_status();
}

// kge_run_chain and kge_run_tfinish as one launch (B > 0 and N > 0)
int kge_run_chain_tfinish(const KgeModelDev &m, const int32_t *h, const int32_t *r, const int32_t *t, int B, int Bp, int dp,
                          const float *acc_part, const float *acc_part2, const float4 *sum_part, const float4 *stat_part,
                          const KgeRowInfo *rowinfo, int nsplit, const float *gpos, float *g_ent, float *g_rel,
                          float *g_relw, int32_t *g_ent_idx, int32_t *g_rel_idx, float reg, float *regv,
                          const float *accT_part, const float4 *sumT_part, int nsplit_t, int Np, int N, int d, int dist_kind,
                          const void *T, const int32_t *neg, float *g_neg, int32_t *g_neg_idx, float *regn,
                          const float *lossb, float scale, float *loss_out, hipStream_t st, bool part_bf16) {
    if (B == 0 || N == 0) return KGE_E_INVALID_ARG;
    const int cb = (B + 3) / 4, tb = (N + 3) / 4;
    const KgeChainArgs a{m, h, r, t, B, Bp, dp, acc_part, acc_part2, sum_part, stat_part, rowinfo, nsplit, gpos,
                         g_ent, g_rel, g_relw, g_ent_idx, g_rel_idx, reg, regv};
    const KgeTfinishArgs f{accT_part, sumT_part, nsplit_t, Np, N, dp, d, dist_kind, T, neg, g_neg, g_neg_idx, m.ent, m.ent_ld, reg, regn};
    if (part_bf16) {
        // (written by the bilinear kernels on bf16 rows of 512 bytes only)
        if (!m.bf16 || dp != 256 || m.vec || (m.scorer != KGE_DISTMULT && m.scorer != KGE_COMPLEX)) return KGE_E_INVALID_ARG;
        if (m.scorer == KGE_DISTMULT)
            hipLaunchKernelGGL((kge_chain_tfinish_kernel<true, KGE_DISTMULT, true>), dim3(1 + cb + tb), dim3(256), 0, st, cb, a, f, lossb, scale, loss_out);
        else
            hipLaunchKernelGGL((kge_chain_tfinish_kernel<true, KGE_COMPLEX, true>), dim3(1 + cb + tb), dim3(256), 0, st, cb, a, f, lossb, scale, loss_out);
        return kge_launch_status();
    }
#define KGE_CT(BF, SC) hipLaunchKernelGGL((kge_chain_tfinish_kernel<BF, SC>), dim3(1 + cb + tb), dim3(256), 0, st, cb, a, f, lossb, scale, loss_out)
    if (m.bf16) { KGE_SC_SWITCH(true, KGE_CT) } else { KGE_SC_SWITCH(false, KGE_CT) }
#undef KGE_CT
    return kge_launch_status();
}
#undef KGE_SC_SWITCH

int kge_run_reg_add(const float *regv, int B, int Bp, int N, float reg, float *loss_out, hipStream_t st) {
    hipLaunchKernelGGL(kge_reg_add_kernel, dim3(1), dim3(1024), 0, st, regv, B, Bp, N, reg, loss_out);
    return kge_launch_status();
}
