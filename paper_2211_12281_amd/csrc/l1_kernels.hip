// The distance scorers with the 1-norm (Table 2, p = 1): f = -sum_j |q_j - t_j| over the query q = h + r (TransE)
// or h o e^{ir} taken in R^d (RotatE).  There is no contraction form: every (query, negative, dimension) triple
// costs vector instructions, so the score block IS written to memory here (4 bytes per pair against 2 d vector
// operations) and the backward pass reads it back instead of recomputing it:
//   scores      S[b, n] = -sum_j |q_bj - t_nj|
//   row pass    per query the maximum and the sums of the loss weights over its row of S
//   gradients   dq[b, j] = -sum_n w(b, n) sign(q_bj - t_nj),   dt[n, j] = +sum_b w(b, n) sign(q_bj - t_nj)
// with w(b, n) = dL/dS[b, n] from S and the finished row constants; sign(0) = 0 (sub-gradient at the kink).
// The queries are read from an unrounded fp32 copy also when the tables are bf16 (a sign flips when rounding moves a
// difference across zero; the table rows themselves are exact).  All three block kernels stage 64 x 64 fp32 tiles in the LDS (row pitch 68 floats: the 16 lanes that read 16
// different rows at one column offset hit 16 different 16-byte bank groups) and keep a 4 x 4 register tile per
// thread; they are bound by the vector pipe.
#include "row_ops.hpp"

namespace {

constexpr int L1_TILE = 64;            // rows and columns of a staged tile
constexpr int L1_PITCH = 68;           // floats per LDS row
constexpr float L1_LOG2E = 1.4426950408889634f, L1_LN2 = 0.6931471805599453f;
constexpr float L1_BIG = 0x1p100f;     // scale of the operands of the sign computation

typedef float l1_f32x4 __attribute__((ext_vector_type(4)));

// rows [r0, r0 + 64) x columns [c0, c0 + 64) of a row-major [rows][ld] array of the table type -> fp32 LDS tile
// (times scale, a power of two)
template <bool BF16>
__device__ __forceinline__ void l1_stage(const void *src, int64_t ld, int r0, int c0, float *tile, float scale = 1.f) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = threadIdx.x + 256 * k, row = e >> 4, cq = e & 15;
        const int64_t off = (int64_t)(r0 + row) * ld + c0 + 4 * cq;
        l1_f32x4 v;
        if constexpr (BF16) {
            const uint2 raw = *(const uint2 *)((const __bf16 *)src + off);
            v = l1_f32x4{__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u),
                         __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xffff0000u)};
        } else {
            v = *(const l1_f32x4 *)((const float *)src + off);
        }
        *(l1_f32x4 *)(tile + row * L1_PITCH + 4 * cq) = v * scale;
    }
}

// S[b, n] = -sum_j |q_bj - t_nj|; workgroup = 64 queries x 64 negatives, thread = queries 4 ty + i, negatives tx + 16 k
template <bool BF16>
__global__ __launch_bounds__(256) void l1_score_kernel(const float *Q, const void *T, int B, int N, int dp, float *S, int64_t ldS) {
    __shared__ __attribute__((aligned(16))) float qs[L1_TILE * L1_PITCH], ts[L1_TILE * L1_PITCH];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int n0 = blockIdx.x * L1_TILE, b0 = blockIdx.y * L1_TILE;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        for (int k = 0; k < 4; ++k) acc[i][k] = 0.f;
    for (int j0 = 0; j0 < dp; j0 += L1_TILE) {
        __syncthreads();
        l1_stage<false>(Q, dp, b0, j0, qs);
        l1_stage<BF16>(T, dp, n0, j0, ts);
        __syncthreads();
#pragma unroll 4
        for (int jq = 0; jq < 16; ++jq) {
            l1_f32x4 q4[4], t4[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                q4[i] = *(const l1_f32x4 *)(qs + (4 * ty + i) * L1_PITCH + 4 * jq);
                t4[i] = *(const l1_f32x4 *)(ts + (tx + 16 * i) * L1_PITCH + 4 * jq);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[i][k] += fabsf(q4[i][c] - t4[k][c]);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int b = b0 + 4 * ty + i;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int n = n0 + tx + 16 * k;
            if (b < B && n < N) S[(int64_t)b * ldS + n] = -acc[i][k];
        }
    }
}

__device__ __forceinline__ float l1_wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float l1_sigmoid(float y) {
    const float t = __builtin_amdgcn_exp2f(-fabsf(y) * L1_LOG2E), rcp = 1.f / (1.f + t);
    return y >= 0.f ? rcp : t * rcp;
}

// Row statistics of the loss (Section 3.1 "Loss Functions"), one wave per query: with x = a s (log-sigmoid
// loss, a the self-adversarial temperature) or x = s (sampled softmax), both times log2(e):
// {m = max_n x_n, sum_n 2^(x_n - m), sum_n 2^(x_n - m) softplus(gamma + s_n), 0}
__global__ __launch_bounds__(256) void l1_rowstat_kernel(const float *S, int64_t ldS, int B, int N, int Bp, int loss, float gamma,
                                                         float adv_temp, float4 *stat) {
    const int lane = threadIdx.x & 63;
    const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (b >= Bp) return;
    if (b >= B) { if (lane == 0) stat[b] = make_float4(-INFINITY, 0.f, 0.f, 0.f); return; }
    const float xscale = (loss == KGE_LOGSIGMOID ? adv_temp : 1.f) * L1_LOG2E;
    const float *row = S + (int64_t)b * ldS;
    float m = -INFINITY;
    for (int n = lane; n < N; n += 64) m = fmaxf(m, row[n] * xscale);
    m = l1_wave_max(m);
    float l = 0.f, ac = 0.f;
    for (int n = lane; n < N; n += 64) {
        const float s = row[n], e = __builtin_amdgcn_exp2f(fmaf(s, xscale, -m));
        l += e;
        if (loss == KGE_LOGSIGMOID) {
            const float y = gamma + s;
            const float t = __builtin_amdgcn_exp2f(-fabsf(y) * L1_LOG2E);
            ac = fmaf(e, fmaxf(y, 0.f) + L1_LN2 * __builtin_amdgcn_logf(1.f + t), ac);
        }
    }
    l = kge_wave_sum(l); ac = kge_wave_sum(ac);
    if (lane == 0) stat[b] = make_float4(m, l, ac, 0.f);
}

// out[split][o, j] = -sum_s w(o, s) sign(own_oj - str_sj) over the split's rows of the streamed operand: with
// own = queries this is dq (s runs over the negatives), with own = negatives it is dt (s runs over the queries;
// the sign flips twice).  Workgroup = 128 own rows x 64 dimensions; thread = own rows 4 ty + i + 64 i',
// dimensions 4 tx + c (an 8 x 4 register tile: three 16-byte LDS reads feed 32 sign terms; about 120 registers,
// four waves per SIMD).  The queries
// are fp32, the negatives of the table type.  Both operands are scaled by 2^100 when they are loaded (exact), so that
// sign(own - str) = median(-1, (own - str) 2^100, 1) is one subtraction and one median: a non-zero difference of
// two floats whose magnitudes exceed 2^-76 is at least 2^-100, its scaled value at least 1; a zero difference
// stays zero (sub-gradient 0).  Three vector operations per (own row, streamed row, dimension).  Per chunk of 32
// streamed rows the weights w = 2^(x log2e + K_b) (times sigma(gamma + s) for the log-sigmoid loss) are computed
// once from S and the finished row constants into the LDS.
constexpr int L1_GO = 128, L1_GD = 64, L1_GS = 32;   // own rows, dimensions, streamed rows per chunk of a gradient workgroup
constexpr int L1_WP = 132;                            // floats per LDS row of the weights (16 lanes x 16 bytes stay conflict-free)

template <bool BF16, bool OWN_Q>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void l1_grad_kernel(
        const void *own, const void *str, const float *S, int64_t ldS, const KgeRowInfo *rowinfo, int B, int N, int own_pad,
        int dp, int chunks, int cps, int loss, float gamma, float adv_temp, float *acc_part) {
    __shared__ __attribute__((aligned(16))) float ss[L1_GS * L1_PITCH], ws[L1_GS * L1_WP];
    constexpr bool SBF = BF16 && OWN_Q, OBF = BF16 && !OWN_Q;   // table type of the streamed / own operand
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int o0 = blockIdx.x * L1_GO, j0 = blockIdx.y * L1_GD, split = blockIdx.z;
    const float xscale = (loss == KGE_LOGSIGMOID ? adv_temp : 1.f) * L1_LOG2E;
    float ov[8][4], acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int o = o0 + 4 * ty + (i & 3) + 64 * (i >> 2);
            ov[i][c] = El<OBF>::ld(own, (int64_t)o * dp + j0 + 4 * tx + c) * L1_BIG;
            acc[i][c] = 0.f;
        }
    const int c_lo = split * cps, c_hi = min(chunks, (split + 1) * cps);
    for (int ch = c_lo; ch < c_hi; ++ch) {
        const int s0 = ch * L1_GS;
        __syncthreads();                                    // everyone is done with the previous chunk
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int e = threadIdx.x + 256 * k, row = e >> 4, cq = e & 15;
            const int64_t off = (int64_t)(s0 + row) * dp + j0 + 4 * cq;
            l1_f32x4 v;
            if constexpr (SBF) {
                const uint2 raw = *(const uint2 *)((const __bf16 *)str + off);
                v = l1_f32x4{__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u),
                             __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xffff0000u)};
            } else {
                v = *(const l1_f32x4 *)((const float *)str + off);
            }
            *(l1_f32x4 *)(ss + row * L1_PITCH + 4 * cq) = v * L1_BIG;
        }
#pragma unroll 4
        for (int k = 0; k < 16; ++k) {
            const int e = threadIdx.x + 256 * k;
            // consecutive threads take consecutive negatives: the reads of S are coalesced either way
            const int ol = OWN_Q ? e >> 5 : e & 127, sl = OWN_Q ? e & 31 : e >> 7;
            const int b = OWN_Q ? o0 + ol : s0 + sl, n = OWN_Q ? s0 + sl : o0 + ol;
            float w = 0.f;
            if (b < B && n < N) {
                const float sc = S[(int64_t)b * ldS + n];
                w = __builtin_amdgcn_exp2f(fmaf(sc, xscale, rowinfo[b].K));
                if (loss == KGE_LOGSIGMOID) w *= l1_sigmoid(gamma + sc);
            }
            ws[sl * L1_WP + ol] = w;
        }
        __syncthreads();
#pragma unroll 4
        for (int sl = 0; sl < L1_GS; ++sl) {
            const l1_f32x4 w4[2] = { *(const l1_f32x4 *)(ws + sl * L1_WP + 4 * ty), *(const l1_f32x4 *)(ws + sl * L1_WP + 4 * ty + 64) };
            const l1_f32x4 t4 = *(const l1_f32x4 *)(ss + sl * L1_PITCH + 4 * tx);
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    acc[i][c] = fmaf(-w4[i >> 2][i & 3], __builtin_amdgcn_fmed3f(ov[i][c] - t4[c], -1.f, 1.f), acc[i][c]);
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
        *(l1_f32x4 *)(acc_part + ((int64_t)split * own_pad + o0 + 4 * ty + (i & 3) + 64 * (i >> 2)) * dp + j0 + 4 * tx) =
            l1_f32x4{acc[i][0], acc[i][1], acc[i][2], acc[i][3]};
}

// ---------------------------------------------------------------------------------------------
// TransH under the 1-norm (Table 2, p = 1): x_j = q'_j - t_j + A w^_j with q' = h_perp + r, A = w^ . t, and
//   f = -sum_j |x_j|,  u_j = sign(x_j),  P = u . w^
//   df/dq'_j = -u_j,   df/dt_j = u_j - P w^_j,   df/dw^_j = -(P t_j + A u_j)
// The hyperplane term sits inside the absolute values, so the score kernel walks the dimensions twice (first A,
// then the distance and P) and leaves A and P beside S for the two gradient kernels.  Queries and unit normals are
// unrounded fp32 rows.  Same tiling as above with 64 own rows per gradient workgroup (a 4 x 4 register tile; the
// pass over the queries carries two accumulators, dq' and dw^).
// ---------------------------------------------------------------------------------------------
// PN = 2 runs the same three kernels for the 2-norm (rows too wide for the matrix-core TransH kernels): the distance sums
// x_j^2, u = x / ||x|| (0 at distance 0), P = (x . w^) / ||x||; the gradient kernels fold 1 / ||x|| = -1 / S into the
// weight of the pair and use x itself where the 1-norm has sign(x).
template <bool BF16, int PN>
__global__ __launch_bounds__(256) void l1h_score_kernel(const float *Q, const float *W, const void *T, int B, int N, int dp,
                                                        float *S, float *A, float *P, int64_t ldS) {
    __shared__ __attribute__((aligned(16))) float qs[L1_TILE * L1_PITCH], ws[L1_TILE * L1_PITCH], ts[L1_TILE * L1_PITCH];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int n0 = blockIdx.x * L1_TILE, b0 = blockIdx.y * L1_TILE;
    float a[4][4], acc[4][4], pp[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        for (int k = 0; k < 4; ++k) a[i][k] = acc[i][k] = pp[i][k] = 0.f;
    for (int j0 = 0; j0 < dp; j0 += L1_TILE) {
        __syncthreads();
        l1_stage<false>(W, dp, b0, j0, ws);
        l1_stage<BF16>(T, dp, n0, j0, ts);
        __syncthreads();
#pragma unroll 4
        for (int jq = 0; jq < 16; ++jq) {
            l1_f32x4 w4[4], t4[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                w4[i] = *(const l1_f32x4 *)(ws + (4 * ty + i) * L1_PITCH + 4 * jq);
                t4[i] = *(const l1_f32x4 *)(ts + (tx + 16 * i) * L1_PITCH + 4 * jq);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int c = 0; c < 4; ++c) a[i][k] = fmaf(w4[i][c], t4[k][c], a[i][k]);
        }
    }
    for (int j0 = 0; j0 < dp; j0 += L1_TILE) {
        __syncthreads();
        l1_stage<false>(Q, dp, b0, j0, qs);
        l1_stage<false>(W, dp, b0, j0, ws);
        l1_stage<BF16>(T, dp, n0, j0, ts);
        __syncthreads();
#pragma unroll 2
        for (int jq = 0; jq < 16; ++jq) {
            l1_f32x4 q4[4], w4[4], t4[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                q4[i] = *(const l1_f32x4 *)(qs + (4 * ty + i) * L1_PITCH + 4 * jq);
                w4[i] = *(const l1_f32x4 *)(ws + (4 * ty + i) * L1_PITCH + 4 * jq);
                t4[i] = *(const l1_f32x4 *)(ts + (tx + 16 * i) * L1_PITCH + 4 * jq);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float x = fmaf(a[i][k], w4[i][c], q4[i][c] - t4[k][c]);
                        if constexpr (PN == 1) {
                            acc[i][k] += fabsf(x);
                            pp[i][k] = fmaf(__builtin_amdgcn_fmed3f(x * L1_BIG, -1.f, 1.f), w4[i][c], pp[i][k]);
                        } else {
                            acc[i][k] = fmaf(x, x, acc[i][k]);
                            pp[i][k] = fmaf(x, w4[i][c], pp[i][k]);
                        }
                    }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int b = b0 + 4 * ty + i;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int n = n0 + tx + 16 * k;
            if (b < B && n < N) {
                const float dist = PN == 1 ? acc[i][k] : sqrtf(acc[i][k]);
                S[(int64_t)b * ldS + n] = -dist;
                if (A) { A[(int64_t)b * ldS + n] = a[i][k]; P[(int64_t)b * ldS + n] = PN == 1 ? pp[i][k] : (dist > 0.f ? pp[i][k] / dist : 0.f); }
            }
        }
    }
}

constexpr int L1H_GO = 64;             // own rows of a TransH gradient workgroup

// OWN_Q: own = 64 queries (q' and w^), streamed = negatives: acc_part = dq' = -sum_n w u,
//        acc_part2 = dw^ = -sum_n (w P) t_n + (w A) u.
// else:  own = 64 negatives, streamed = queries: acc_part = dt = sum_b w u - (w P) w^_b.
// u = sign(x) = median(-1, x 2^100, 1) (a non-zero x of magnitude at least 2^-100 scales to at least 1).
template <bool BF16, bool OWN_Q, int PN>
__global__ __launch_bounds__(256) void l1h_grad_kernel(const float *Q, const float *W, const void *T, const float *S,
                                                       const float *A, const float *P, int64_t ldS, const KgeRowInfo *rowinfo,
                                                       int B, int N, int own_pad, int dp, int chunks, int cps, int loss,
                                                       float gamma, float adv_temp, float *acc_part, float *acc_part2) {
    __shared__ __attribute__((aligned(16))) float s1[L1_GS * L1_PITCH], s2[L1_GS * L1_PITCH];
    __shared__ __attribute__((aligned(16))) float cw[L1_GS * L1_PITCH], ca[L1_GS * L1_PITCH], cp[L1_GS * L1_PITCH];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int o0 = blockIdx.x * L1H_GO, j0 = blockIdx.y * L1_GD, split = blockIdx.z;
    const float xscale = (loss == KGE_LOGSIGMOID ? adv_temp : 1.f) * L1_LOG2E;
    float o1[4][4], o2[4][4], acc1[4][4], acc2[4][4];      // own rows: (q', w^) or (t, -)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int64_t off = (int64_t)(o0 + 4 * ty + i) * dp + j0 + 4 * tx + c;
            o1[i][c] = OWN_Q ? Q[off] : El<BF16>::ld(T, off);
            o2[i][c] = OWN_Q ? W[off] : 0.f;
            acc1[i][c] = acc2[i][c] = 0.f;
        }
    const int c_lo = split * cps, c_hi = min(chunks, (split + 1) * cps);
    for (int ch = c_lo; ch < c_hi; ++ch) {
        const int s0 = ch * L1_GS;
        __syncthreads();                                    // everyone is done with the previous chunk
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int e = threadIdx.x + 256 * k, row = e >> 4, cq = e & 15;
            const int64_t off = (int64_t)(s0 + row) * dp + j0 + 4 * cq;
            if constexpr (OWN_Q) {
                l1_f32x4 v;
                if constexpr (BF16) {
                    const uint2 raw = *(const uint2 *)((const __bf16 *)T + off);
                    v = l1_f32x4{__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u),
                                 __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xffff0000u)};
                } else {
                    v = *(const l1_f32x4 *)((const float *)T + off);
                }
                *(l1_f32x4 *)(s1 + row * L1_PITCH + 4 * cq) = v;
            } else {
                *(l1_f32x4 *)(s1 + row * L1_PITCH + 4 * cq) = *(const l1_f32x4 *)(Q + off);
                *(l1_f32x4 *)(s2 + row * L1_PITCH + 4 * cq) = *(const l1_f32x4 *)(W + off);
            }
        }
#pragma unroll 4
        for (int k = 0; k < 8; ++k) {
            const int e = threadIdx.x + 256 * k;
            // consecutive threads take consecutive negatives: the reads of S, A and P are coalesced either way
            const int ol = OWN_Q ? e >> 5 : e & 63, sl = OWN_Q ? e & 31 : e >> 6;
            const int b = OWN_Q ? o0 + ol : s0 + sl, n = OWN_Q ? s0 + sl : o0 + ol;
            float w = 0.f, av = 0.f, pv = 0.f;
            if (b < B && n < N) {
                const float sc = S[(int64_t)b * ldS + n];
                w = __builtin_amdgcn_exp2f(fmaf(sc, xscale, rowinfo[b].K));
                if (loss == KGE_LOGSIGMOID) w *= l1_sigmoid(gamma + sc);
                av = A[(int64_t)b * ldS + n];
                pv = w * P[(int64_t)b * ldS + n];
                if constexpr (PN == 2) w = sc < 0.f ? -w / sc : 0.f;    // u = x / ||x||: the pair's 1 / ||x|| rides on its weight
            }
            cw[sl * L1_PITCH + ol] = w; ca[sl * L1_PITCH + ol] = av; cp[sl * L1_PITCH + ol] = pv;
        }
        __syncthreads();
#pragma unroll 2
        for (int sl = 0; sl < L1_GS; ++sl) {
            const l1_f32x4 w4 = *(const l1_f32x4 *)(cw + sl * L1_PITCH + 4 * ty);
            const l1_f32x4 a4 = *(const l1_f32x4 *)(ca + sl * L1_PITCH + 4 * ty);
            const l1_f32x4 p4 = *(const l1_f32x4 *)(cp + sl * L1_PITCH + 4 * ty);
            const l1_f32x4 r1 = *(const l1_f32x4 *)(s1 + sl * L1_PITCH + 4 * tx);
            if constexpr (OWN_Q) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float wa = w4[i] * a4[i];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float x = fmaf(a4[i], o2[i][c], o1[i][c] - r1[c]);
                        const float u = PN == 1 ? __builtin_amdgcn_fmed3f(x * L1_BIG, -1.f, 1.f) : x;
                        acc1[i][c] = fmaf(-w4[i], u, acc1[i][c]);
                        acc2[i][c] = fmaf(-p4[i], r1[c], fmaf(-wa, u, acc2[i][c]));
                    }
                }
            } else {
                const l1_f32x4 r2 = *(const l1_f32x4 *)(s2 + sl * L1_PITCH + 4 * tx);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float x = fmaf(a4[i], r2[c], r1[c] - o1[i][c]);
                        const float u = PN == 1 ? __builtin_amdgcn_fmed3f(x * L1_BIG, -1.f, 1.f) : x;
                        acc1[i][c] = fmaf(w4[i], u, fmaf(-p4[i], r2[c], acc1[i][c]));
                    }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t off = ((int64_t)split * own_pad + o0 + 4 * ty + i) * dp + j0 + 4 * tx;
        *(l1_f32x4 *)(acc_part + off) = l1_f32x4{acc1[i][0], acc1[i][1], acc1[i][2], acc1[i][3]};
        if constexpr (OWN_Q) *(l1_f32x4 *)(acc_part2 + off) = l1_f32x4{acc2[i][0], acc2[i][1], acc2[i][2], acc2[i][3]};
    }
}

}  // namespace

int kge_run_l1_score(bool bf16, const float *Q, const void *T, int B, int N, int Bp, int Np, int dp, float *S, int64_t ldS,
                     hipStream_t st) {
    if (Bp % L1_TILE || Np % L1_TILE || dp % L1_TILE) return KGE_E_INVALID_ARG;
    if (Bp == 0 || Np == 0) return KGE_OK;
    if (Bp / L1_TILE > 65535) return KGE_E_UNSUPPORTED;   // grid limit of the second dimension
    KgeProfScope prof(KGE_PROF_BLOCK_SCORE, st);
    const dim3 grid(Np / L1_TILE, Bp / L1_TILE);
    if (bf16) hipLaunchKernelGGL(l1_score_kernel<true>, grid, dim3(256), 0, st, Q, T, B, N, dp, S, ldS);
    else      hipLaunchKernelGGL(l1_score_kernel<false>, grid, dim3(256), 0, st, Q, T, B, N, dp, S, ldS);
    return kge_launch_status();
}

int kge_run_l1_rowstat(const float *S, int64_t ldS, int B, int N, int Bp, int loss, float gamma, float adv_temp,
                       float4 *stat, hipStream_t st) {
    if (Bp == 0) return KGE_OK;
    hipLaunchKernelGGL(l1_rowstat_kernel, dim3((Bp + 3) / 4), dim3(256), 0, st, S, ldS, B, N, Bp, loss, gamma, adv_temp, stat);
    return kge_launch_status();
}

// splits over the streamed rows: enough workgroups for about four per compute unit
int kge_l1_nsplit(int own_pad, int str_pad, int dp, bool transh) {
    const int base = (own_pad / (transh ? L1H_GO : L1_GO)) * (dp / L1_GD), chunks = str_pad / L1_GS;
    if (base == 0 || chunks == 0) return 0;
    int want = (1024 + base - 1) / base;
    if (want > chunks) want = chunks;
    const int cps = (chunks + want - 1) / want;
    return (chunks + cps - 1) / cps;
}

int kge_run_l1_grad(bool bf16, bool own_is_query, const void *own, const void *str, const float *S, int64_t ldS,
                    const KgeRowInfo *rowinfo, int B, int N, int own_pad, int str_pad, int dp, int loss, float gamma,
                    float adv_temp, int nsplit, float *acc_part, hipStream_t st) {
    if (own_pad % L1_GO || str_pad % L1_GS || dp % L1_GD) return KGE_E_INVALID_ARG;
    if (nsplit <= 0 || nsplit != kge_l1_nsplit(own_pad, str_pad, dp, false)) return KGE_E_INVALID_ARG;
    KgeProfScope prof(own_is_query ? KGE_PROF_BLOCK_FWD : KGE_PROF_BLOCK_GRADT, st);
    const int chunks = str_pad / L1_GS, cps = (chunks + nsplit - 1) / nsplit;
    const dim3 grid(own_pad / L1_GO, dp / L1_GD, nsplit);
#define L1_GRAD(BF, OQ) hipLaunchKernelGGL((l1_grad_kernel<BF, OQ>), grid, dim3(256), 0, st, own, str, S, ldS, rowinfo, B, N, \
                                           own_pad, dp, chunks, cps, loss, gamma, adv_temp, acc_part)
    if (bf16) { if (own_is_query) L1_GRAD(true, true); else L1_GRAD(true, false); }
    else      { if (own_is_query) L1_GRAD(false, true); else L1_GRAD(false, false); }
#undef L1_GRAD
    return kge_launch_status();
}

// TransH: scores (and, with A and P given, the two per-pair scalars that the gradient kernels need)
int kge_run_l1h_score(bool bf16, const float *Q, const float *W, const void *T, int B, int N, int Bp, int Np, int dp, float *S,
                      float *A, float *P, int64_t ldS, hipStream_t st, int pn) {
    if (Bp % L1_TILE || Np % L1_TILE || dp % L1_TILE || (A == nullptr) != (P == nullptr)) return KGE_E_INVALID_ARG;
    if (Bp == 0 || Np == 0) return KGE_OK;
    if (Bp / L1_TILE > 65535) return KGE_E_UNSUPPORTED;
    KgeProfScope prof(KGE_PROF_BLOCK_SCORE, st);
    const dim3 grid(Np / L1_TILE, Bp / L1_TILE);
#define L1H_SCORE(BF, PN) hipLaunchKernelGGL((l1h_score_kernel<BF, PN>), grid, dim3(256), 0, st, Q, W, T, B, N, dp, S, A, P, ldS)
    if (bf16) { if (pn == 1) L1H_SCORE(true, 1); else L1H_SCORE(true, 2); }
    else      { if (pn == 1) L1H_SCORE(false, 1); else L1H_SCORE(false, 2); }
#undef L1H_SCORE
    return kge_launch_status();
}

int kge_run_l1h_grad(bool bf16, bool own_is_query, const float *Q, const float *W, const void *T, const float *S, const float *A,
                     const float *P, int64_t ldS, const KgeRowInfo *rowinfo, int B, int N, int own_pad, int str_pad, int dp,
                     int loss, float gamma, float adv_temp, int nsplit, float *acc_part, float *acc_part2, hipStream_t st, int pn) {
    if (own_pad % L1H_GO || str_pad % L1_GS || dp % L1_GD) return KGE_E_INVALID_ARG;
    if (nsplit <= 0 || nsplit != kge_l1_nsplit(own_pad, str_pad, dp, true)) return KGE_E_INVALID_ARG;
    KgeProfScope prof(own_is_query ? KGE_PROF_BLOCK_FWD : KGE_PROF_BLOCK_GRADT, st);
    const int chunks = str_pad / L1_GS, cps = (chunks + nsplit - 1) / nsplit;
    const dim3 grid(own_pad / L1H_GO, dp / L1_GD, nsplit);
    if (grid.z > 65535 || grid.y > 65535) return KGE_E_UNSUPPORTED;
#define L1H_GRAD(BF, OQ) do { if (pn == 1) hipLaunchKernelGGL((l1h_grad_kernel<BF, OQ, 1>), grid, dim3(256), 0, st, Q, W, T, S, A, P, ldS, rowinfo, B, N, \
                                                                  own_pad, dp, chunks, cps, loss, gamma, adv_temp, acc_part, acc_part2); \
                              else hipLaunchKernelGGL((l1h_grad_kernel<BF, OQ, 2>), grid, dim3(256), 0, st, Q, W, T, S, A, P, ldS, rowinfo, B, N, \
                                                      own_pad, dp, chunks, cps, loss, gamma, adv_temp, acc_part, acc_part2); } while (0)
    if (bf16) { if (own_is_query) L1H_GRAD(true, true); else L1H_GRAD(true, false); }
    else      { if (own_is_query) L1H_GRAD(false, true); else L1H_GRAD(false, false); }
#undef L1H_GRAD
    return kge_launch_status();
}
