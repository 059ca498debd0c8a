// Per-row finish of the loss, shared by the launch of its own (prep_kernels.hip) and the launch that it shares with the
// sorts of the step's row ids (sparse_adam.hip).
#pragma once
#include "kge_internal.h"

// ---------------------------------------------------------------------------------------------
// per-row finish of the loss (Section 3.1): combines the split statistics with the positive score
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float kge_softplus_f(float y) { return fmaxf(y, 0.f) + log1pf(expf(-fabsf(y))); }

struct KgeRowFinish { float L, gp, K; };
__device__ __forceinline__ KgeRowFinish kge_rowfinish_row(const float4 *stat_part, int nsplit, int Bp, int b, int N, int loss,
                                                          float gamma, float c_corr, float scale, float fp) {
    const float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;
    // merge the splits: m is the running maximum of x * log2(e) (x = a*s or s), l the sum of
    // exp(x - max), ac the sum of exp(x - max) * softplus(gamma + s)
    float m = -INFINITY, l = 0.f, ac = 0.f;
    for (int s0 = 0; s0 < nsplit; s0 += 8) {                // fixed order; eight loads in flight
        float4 pv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) pv[u] = stat_part[(size_t)(s0 + u < nsplit ? s0 + u : nsplit - 1) * Bp + b];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float4 p = pv[u];
            if (s0 + u >= nsplit || p.x == -INFINITY) continue;
            const float mn = fmaxf(m, p.x);
            const float r0 = exp2f(m - mn), r1 = exp2f(p.x - mn);
            l = l * r0 + p.y * r1; ac = ac * r0 + p.z * r1; m = mn;
        }
    }
    KgeRowFinish o;
    if (loss == KGE_LOGSIGMOID) {
        o.L = kge_softplus_f(-(gamma + fp));
        const float e = expf(-fabsf(gamma + fp));           // sigma(-(gamma+fp)), stable
        o.gp = -((gamma + fp) >= 0.f ? e / (1.f + e) : 1.f / (1.f + e)) * scale;
        if (N > 0 && l > 0.f) { o.L += ac / l; o.K = -m - log2f(l) + log2f(scale); } else o.K = -INFINITY;
    } else {
        if (N > 0 && l > 0.f) {
            const float A = c_corr + logf(l) + m * LN2;     // log of the negatives' share of the partition sum
            const float M = fmaxf(A, fp);
            const float lse = M + logf(expf(A - M) + expf(fp - M));
            o.L = lse - fp;
            o.gp = (expf(fp - lse) - 1.f) * scale;
            o.K = (c_corr - lse + logf(scale)) * LOG2E;
        } else { o.L = 0.f; o.gp = 0.f; o.K = -INFINITY; }
    }
    return o;
}

// The same finish, one wave per row, which also leaves the bf16 query row (256 elements) scaled for every forward split s:
// qs[s][b] = bf16(exp2(ref_s[b] + K[b]) q[b]), ref_s the reference exponent that split s weighted the row's scores
// against (stat_part[s][b].x) - the factor that turns a stored weight of the forward pass into the pair's gradient
// coefficient (block_gradp.hip).  Rows b >= B and splits that saw no negative get zeros.
__device__ __forceinline__ void kge_rowfinish_qscale_body(int blk, const KgeRowFinishQArgs &a) {
    const float4 *stat_part = a.stat_part;
    const int nsplit = a.nsplit, Bp = a.Bp, B = a.B;
    const int lane = threadIdx.x & 63;
    const int b = blk * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (b >= Bp) return;
    float K = -INFINITY;
    if (b < B) {
        const KgeRowFinish o = kge_rowfinish_row(stat_part, nsplit, Bp, b, a.N, a.loss, a.gamma, a.c_corr, a.scale, a.pos[b]);
        K = o.K;
        if (lane == 0) { a.lossb[b] = o.L; a.gpos[b] = o.gp; a.rowinfo[b].K = o.K; }
    } else if (lane == 0) { a.lossb[b] = 0.f; a.gpos[b] = 0.f; a.rowinfo[b].K = -INFINITY; }
    const uint2 raw = *(const uint2 *)(a.Q + (size_t)b * 256 + 4 * lane);
    const float q[4] = { __uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u),
                         __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xffff0000u) };
    for (int s0 = 0; s0 < nsplit; s0 += 8) {
      float refs[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) refs[u] = s0 + u < nsplit ? stat_part[(size_t)(s0 + u) * Bp + b].x : -INFINITY;   // eight loads in flight
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int s = s0 + u;
        if (s >= nsplit) break;
        const float ref = refs[u];
        const float f = (b < B && ref > -INFINITY && K > -INFINITY) ? exp2f(ref + K) : 0.f;
        uint16_t o[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) o[c] = __builtin_bit_cast(uint16_t, (__bf16)(f * q[c]));
        *(uint2 *)(a.Qs + ((size_t)s * Bp + b) * 256 + 4 * lane) =
            make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16));
      }
    }
}
