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
typedef uint32_t enc_u32x4 __attribute__((ext_vector_type(4)));   // (arrays of HIP's uint4 struct end up in scratch memory)

namespace {

constexpr int ENC_TILE = 128;          // rows and columns of a workgroup's output tile; slot counts are padded to it

template <bool BF16>
__device__ __forceinline__ enc_f32x16 enc_mma16(enc_f32x16 acc, enc_u32x4 a, enc_u32x4 b) {
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

// One contraction C[split][M, N] (fp32) = A[M, K] . B[N, K]^t, K counted in k-steps of 32 bytes of a row (16 bf16
// or 8 fp32).  Rows at or beyond m_valid / n_valid read as zero.  A's row r is table row idx0[r] for r < n_idx0,
// idx1[r - n_idx0] beyond (gather == 0: row r itself): the gather of the feature rows is part of the load.
struct EncGemm {
    const char *A; int64_t lda_b; const int32_t *idx0, *idx1; int n_idx0; int gather; int m_valid;
    const char *B; int64_t ldb_b; int n_valid;
    float *C; int64_t ldc, split_stride;
    int ksteps, kps, nsplit, tiles_m, tiles_n;
};
// A launch runs two contractions (heads against M_H, tails and negatives against M_T) so that the chip is filled
// once; work items enumerate (contraction, split, row tile, column tile), column tile fastest.
struct EncGemmPair { EncGemm g[2]; int wgs0, total; };

constexpr int ENC_NSTAGE = 4;                                // chunks resident in the LDS ring
constexpr int ENC_ROW_BYTES = 64;                            // a chunk is two k-steps: 64 bytes of every row
constexpr int ENC_HALF_BYTES = ENC_TILE * ENC_ROW_BYTES;     // one operand's rows of one chunk
constexpr int ENC_STAGE_BYTES = 2 * ENC_HALF_BYTES;
constexpr int ENC_LDS_BYTES = ENC_NSTAGE * ENC_STAGE_BYTES;  // 64 KB: two workgroups per compute unit
constexpr int ENC_LPW = 4;                                   // asynchronous copies per wave and chunk

__device__ __forceinline__ void enc_async_copy16(const void *g, uint32_t lds_addr) {
    // lane l of the wave writes its 16 bytes to LDS byte address lds_addr + 16 l; completion is tracked by vmcnt and
    // the compiler does not see the load, so the waits below are explicit
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(g) : "memory");
}
template <int N> __device__ __forceinline__ void enc_wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Workgroup = 128 x 128 outputs, wave = 64 x 64 (2 x 2 blocks of 32 x 32).  Both operands pass through the LDS
// in chunks of two k-steps (64 bytes of every row).  The chunks are copied global -> LDS asynchronously into a
// ring of ENC_NSTAGE stages, so that the rows of ENC_NSTAGE - 1 chunks (random table rows in the forward pass:
// pure latency) are in flight while one chunk is multiplied; no registers are tied up by the copies.  The ring
// takes 64 KB and the kernel at most 128 registers per lane, so two workgroups share a compute unit: one's
// prologue, barriers and write-out overlap the other's products.  A 64-byte LDS row keeps its four 16-byte pieces
// XOR-swizzled by (row / 2) % 4, so that the fragment reads of 8 consecutive rows fall into 8 different bank
// groups; a copy instruction fills 16 rows, lane l fetching piece (l % 4) ^ ((l / 8) % 4) of row l / 4 into slot
// l % 4.  Fragment of (row block, k-step): lane l reads piece 2 ks + l / 32 of row l % 32.  Rows beyond m_valid /
// n_valid are read from row 0 instead (valid memory); their outputs are never stored.  An odd last k-step goes
// through registers with zeros selected for the missing pieces.
// Workgroup ids are dealt round-robin to the 8 dies: id -> work item (id % 8) * ceil(total / 8) + id / 8, so that
// the tiles that share operand rows run on the same die and meet in its L2.
template <bool BF16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void enc_gemm_nt_kernel(const EncGemmPair pr) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, g = lane >> 5;
    const int per = (pr.total + 7) >> 3;
    int w = ((int)blockIdx.x & 7) * per + ((int)blockIdx.x >> 3);
    if (w >= pr.total) return;
    const bool second = w >= pr.wgs0;
    const EncGemm &q = pr.g[second ? 1 : 0];
    w -= second ? pr.wgs0 : 0;
    const int tn = w % q.tiles_n; w /= q.tiles_n;
    const int tm = w % q.tiles_m, split = w / q.tiles_m;
    const int m0 = tm * ENC_TILE, n0 = tn * ENC_TILE;
    const int k_lo = split * q.kps, k_hi = min(q.ksteps, k_lo + q.kps);
    const int nfull = (k_hi - k_lo) >> 1, rem = (k_hi - k_lo) & 1;
    // staging: copy j (j < 2) of wave v fills rows 32 v + 16 j .. + 15 of a tile; this lane's row and piece
    const int srow = lane >> 2, piece = (lane & 3) ^ ((srow >> 1) & 3);
    const char *ga[2], *gb[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int ra = m0 + 32 * wave + 16 * j + srow, rb = n0 + 32 * wave + 16 * j + srow;
        int64_t src = 0;
        if (ra < q.m_valid) src = q.gather ? (ra < q.n_idx0 ? (int64_t)q.idx0[ra] : (int64_t)q.idx1[ra - q.n_idx0]) : (int64_t)ra;
        ga[j] = q.A + src * q.lda_b + piece * 16 + (int64_t)k_lo * 32;
        gb[j] = q.B + (int64_t)(rb < q.n_valid ? rb : 0) * q.ldb_b + piece * 16 + (int64_t)k_lo * 32;
    }
    // the row indices must have arrived before the loop: a compiler-inserted wait inside it would drain the ring
#pragma unroll
    for (int j = 0; j < 2; ++j) asm volatile("" : "+v"(ga[j]), "+v"(gb[j]));
    auto issue = [&](int c) {                             // chunk min(c, nfull - 1) -> stage c % ENC_NSTAGE
        const int64_t off = (int64_t)min(c, nfull - 1) * ENC_ROW_BYTES;
        const uint32_t sb = lds0 + (uint32_t)(c & (ENC_NSTAGE - 1)) * ENC_STAGE_BYTES + (uint32_t)wave * (32 * ENC_ROW_BYTES);
#pragma unroll
        for (int j = 0; j < 2; ++j) enc_async_copy16(ga[j] + off, __builtin_amdgcn_readfirstlane(sb + j * 1024));
#pragma unroll
        for (int j = 0; j < 2; ++j) enc_async_copy16(gb[j] + off, __builtin_amdgcn_readfirstlane(sb + ENC_HALF_BYTES + j * 1024));
    };
    enc_f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j)
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    const int wm = (wave & 1) * 64, wn = (wave >> 1) * 64;
    auto compute = [&](int stage) {
        const char *sa = lds + stage * ENC_STAGE_BYTES, *sb = sa + ENC_HALF_BYTES;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            enc_u32x4 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int rowa = wm + 32 * i + lr, rowb = wn + 32 * i + lr;
                fa[i] = *(const enc_u32x4 *)(sa + rowa * ENC_ROW_BYTES + (((2 * ks + g) ^ ((rowa >> 1) & 3)) * 16));
                fb[i] = *(const enc_u32x4 *)(sb + rowb * ENC_ROW_BYTES + (((2 * ks + g) ^ ((rowb >> 1) & 3)) * 16));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = enc_mma16<BF16>(acc[i][j], fa[i], fb[j]);
        }
    };
    static_assert((ENC_NSTAGE & (ENC_NSTAGE - 1)) == 0 && (ENC_NSTAGE - 2) * ENC_LPW < 64, "ring size");
    if (nfull > 0) {
        for (int c = 0; c < ENC_NSTAGE - 1; ++c) issue(c);
        for (int c = 0; c < nfull; ++c) {
            // chunks up to c + ENC_NSTAGE - 2 are issued; all but the last ENC_NSTAGE - 2 of them must have landed
            enc_wait_vmcnt<(ENC_NSTAGE - 2) * ENC_LPW>();
            __syncthreads();                                // chunk c is complete; everyone is done with chunk c - 1
            issue(c + ENC_NSTAGE - 1);                      // ... whose stage is refilled (past the end: a harmless repeat)
            compute(c & (ENC_NSTAGE - 1));
        }
        enc_wait_vmcnt<0>();                                // no copy may be in flight when the LDS is reused or released
    }
    if (rem > 0) {
        __syncthreads();
        const enc_u32x4 zero = {0u, 0u, 0u, 0u};
        const bool in = (piece >> 1) < rem;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const enc_u32x4 xa = in ? *(const enc_u32x4 *)(ga[j] + (int64_t)nfull * ENC_ROW_BYTES) : zero;
            const enc_u32x4 xb = in ? *(const enc_u32x4 *)(gb[j] + (int64_t)nfull * ENC_ROW_BYTES) : zero;
            char *dst = lds + (32 * wave + 16 * j) * ENC_ROW_BYTES + lane * 16;
            *(enc_u32x4 *)dst = xa;
            *(enc_u32x4 *)(dst + ENC_HALF_BYTES) = xb;
        }
        __syncthreads();
        compute(0);
    }
    // accumulator layout: lane holds column lr of the B side; register e holds A-side row 8 (e/4) + 4 g + e%4
    float *Cs = q.C + (int64_t)split * q.split_stride;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn + 32 * j + lr;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = m0 + wm + 32 * i + 8 * (e >> 2) + 4 * g + (e & 3);
                if (row < q.m_valid && col < q.n_valid) Cs[(int64_t)row * q.ldc + col] = acc[i][j][e];
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

// Transposed buffers of the backward pass: columns [0, Bh) hold the head slots (Bh = B padded to a tile), columns
// [Bh, Bh + B + N) the tail and negative slots - the two groups contract against different projection matrices.
// The row kernels below work on groups of 32 slots that never straddle the two sections: workgroup w takes head
// slots 32 w .. if w < ceil(B / 32), else tail-section slots 32 (w - ceil(B / 32)) ..
struct EncGroup { int slot0, count, col0; };      // first slot, valid slots (<= 32), first column
__device__ __forceinline__ EncGroup enc_group(int w, int B, int N, int Bh) {
    const int hg = (B + 31) / 32;
    EncGroup gr;
    if (w < hg) { gr.slot0 = 32 * w; gr.count = min(32, B - gr.slot0); gr.col0 = gr.slot0; }
    else { const int o = 32 * (w - hg); gr.slot0 = B + o; gr.count = min(32, B + N - o); gr.col0 = Bh + o; }
    return gr;
}

// 32 x len tile (fp32 in the LDS, row stride len + 1) -> rows of the transposed buffer, 8 columns per store
template <bool BF16>
__device__ __forceinline__ void enc_write_transposed(const float *tile, int ldt, int len, void *dst, int64_t ncols,
                                                      const EncGroup &gr) {
    // element (j, 8 q .. 8 q + 7): one 16-byte (bf16) or two 16-byte (fp32) stores; columns past the group's count
    // are padding or belong to nobody (they stay zero / are written as zero)
    for (int idx = threadIdx.x; idx < len * 4; idx += 256) {
        const int j = idx >> 2, q = idx & 3;
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = (8 * q + u < gr.count) ? tile[(8 * q + u) * ldt + j] : 0.f;
        if (8 * q >= gr.count) continue;
        char *p = (char *)dst + ((int64_t)j * ncols + gr.col0 + 8 * q) * (BF16 ? 2 : 4);
        if constexpr (BF16) {
            typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf2;
            enc_u32x4 o;
#pragma unroll
            for (int u = 0; u < 4; ++u) { bf2 t = { (__bf16)v[2 * u], (__bf16)v[2 * u + 1] }; o[u] = __builtin_bit_cast(uint32_t, t); }
            *(enc_u32x4 *)p = o;
        } else {
            *(enc_f32x4 *)p = enc_f32x4{v[0], v[1], v[2], v[3]};
            *(enc_f32x4 *)(p + 16) = enc_f32x4{v[4], v[5], v[6], v[7]};
        }
    }
}

// backward rows (a workgroup takes a group of 32 slots, a wave 8 of them in turn): de' = de + reg_t grad||e||,
// g_es = de' + reg_s grad||s||, dP = D o de' + reg_f grad||P||; dP leaves through the LDS as dP^t[d][columns]
template <bool BF16>
__global__ __launch_bounds__(256) void enc_bwd_rows_kernel(EncRowArgs a, const float *P, const float *de, float *g_es,
                                                           void *dPt, int Bh, int64_t ncols) {
    extern __shared__ float tile[];                        // [32][d + 1]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const EncGroup gr = enc_group(blockIdx.x, a.B, a.N, Bh);
    const int ldt = a.d + 1;
    for (int r = wave; r < gr.count; r += 4) {
        const int i = gr.slot0 + r;
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
    enc_write_transposed<BF16>(tile, ldt, a.d, dPt, ncols, gr);
}

// F^t[f][columns] of the gathered slots (a workgroup takes a group of 32 slots); rows are read with 16-byte loads
template <bool BF16>
__global__ __launch_bounds__(256) void enc_gather_t_kernel(EncRowArgs a, const void *feat, int64_t feat_ld, int fd, void *Ft,
                                                           int Bh, int64_t ncols) {
    extern __shared__ float tile[];                        // [32][fd + 1]
    const EncGroup gr = enc_group(blockIdx.x, a.B, a.N, Bh);
    const int ldt = fd + 1;
    constexpr int EPV = BF16 ? 8 : 4;                      // elements per 16 bytes
    const int ppr = fd / EPV;                              // 16-byte pieces per row
    // six pieces per thread are requested before the first is used (random rows: the bytes in flight bound the rate)
    constexpr int U = 6;
    const int total = gr.count * ppr;
    for (int base = threadIdx.x; base < total; base += 256 * U) {
        enc_u32x4 v[U];
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const int idx = base + q * 256;
            if (idx < total) {
                const int r = idx / ppr, pc = idx % ppr;
                v[q] = *(const enc_u32x4 *)((const char *)feat +
                                            ((int64_t)enc_slot_entity(a, gr.slot0 + r) * feat_ld + pc * EPV) * (BF16 ? 2 : 4));
            }
        }
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const int idx = base + q * 256;
            if (idx >= total) continue;
            const int r = idx / ppr, pc = idx % ppr;
            float *dst = tile + r * ldt + pc * EPV;
            if constexpr (BF16) {
#pragma unroll
                for (int u = 0; u < 4; ++u) { dst[2 * u] = __uint_as_float(v[q][u] << 16); dst[2 * u + 1] = __uint_as_float(v[q][u] & 0xffff0000u); }
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) dst[u] = __uint_as_float(v[q][u]);
            }
        }
    }
    __syncthreads();
    enc_write_transposed<BF16>(tile, ldt, fd, Ft, ncols, gr);
}

// the padding columns [B, Bh) and [Bh + B + N, ncols) of the transposed buffers must read as zero
template <bool BF16>
__global__ void enc_zero_pad_kernel(void *buf, int rows, int64_t ncols, int B, int Bh, int tail_end) {
    const int row = blockIdx.x;
    if (row >= rows) return;
    const int pad1 = Bh - B, pad2 = (int)(ncols - tail_end);
    for (int c = threadIdx.x; c < pad1 + pad2; c += blockDim.x) {
        const int64_t col = c < pad1 ? B + c : tail_end + (c - pad1);
        El<BF16>::st(buf, (int64_t)row * ncols + col, 0.f);
    }
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

EncGemm enc_gemm_desc(const void *A, int64_t lda_b, bool gather, const int32_t *idx0, int n_idx0, const int32_t *idx1, int m_valid,
                      const void *Bm, int64_t ldb_b, int n_valid, float *C, int64_t ldc, int64_t split_stride, int ksteps,
                      int kps, int nsplit) {
    EncGemm q{};
    q.A = (const char *)A; q.lda_b = lda_b; q.idx0 = idx0; q.idx1 = idx1; q.n_idx0 = n_idx0; q.gather = gather ? 1 : 0; q.m_valid = m_valid;
    q.B = (const char *)Bm; q.ldb_b = ldb_b; q.n_valid = n_valid; q.C = C; q.ldc = ldc; q.split_stride = split_stride;
    q.ksteps = ksteps; q.kps = kps; q.nsplit = m_valid > 0 && ksteps > 0 ? nsplit : 0;
    q.tiles_m = (m_valid + ENC_TILE - 1) / ENC_TILE; q.tiles_n = (n_valid + ENC_TILE - 1) / ENC_TILE;
    return q;
}

int enc_launch_pair(bool bf16, const EncGemm &g0, const EncGemm &g1, hipStream_t st) {
    // the ring of stages is larger than the default dynamic limit
    static KgeLdsLimit lim_bf16, lim_f32;
    if (lim_bf16.set((const void *)enc_gemm_nt_kernel<true>, ENC_LDS_BYTES) != KGE_OK ||
        lim_f32.set((const void *)enc_gemm_nt_kernel<false>, ENC_LDS_BYTES) != KGE_OK)
        return KGE_E_HIP;
    EncGemmPair pr{};
    pr.g[0] = g0; pr.g[1] = g1;
    pr.wgs0 = g0.tiles_m * g0.tiles_n * g0.nsplit;
    pr.total = pr.wgs0 + g1.tiles_m * g1.tiles_n * g1.nsplit;
    if (pr.total == 0) return KGE_OK;
    const int grid = (pr.total + 7) / 8 * 8;
    if (bf16) hipLaunchKernelGGL(enc_gemm_nt_kernel<true>, dim3(grid), dim3(256), ENC_LDS_BYTES, st, pr);
    else      hipLaunchKernelGGL(enc_gemm_nt_kernel<false>, dim3(grid), dim3(256), ENC_LDS_BYTES, st, pr);
    return KGE_OK;
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
        take((size_t)(p.nsplit_h + p.nsplit_t + 1) * e.dim * e.feat_dim * 4);     // split partials of both contractions
    }
    return off + 256;
}

int kge_run_encode(const kge_encoder_t &e, const int32_t *h, const int32_t *t, int64_t B, const int32_t *neg, int64_t N,
                   uint64_t seed, uint64_t step, void *e_out, float *proj_out, float *reg_out, void *ws, hipStream_t st) {
    const EncPlan p = enc_plan(e, B, N);
    const bool bf16 = e.dtype == KGE_BF16;
    float *regv = (float *)ws;
    const int ksteps = e.feat_dim * p.es / 32;
    {
        KgeProfScope prof(KGE_PROF_ENC_FWD, st);          // heads against M_H, tails and negatives against M_T: one launch
        const EncGemm gh = enc_gemm_desc(e.feat, e.feat_ld * p.es, true, h, (int)B, nullptr, (int)B, e.m_h, e.m_ld * p.es, e.dim,
                                         proj_out, e.dim, 0, ksteps, ksteps, 1);
        const EncGemm gt = enc_gemm_desc(e.feat, e.feat_ld * p.es, true, t, (int)B, neg, (int)(B + N), e.m_t, e.m_ld * p.es, e.dim,
                                         proj_out + (size_t)B * e.dim, e.dim, 0, ksteps, ksteps, 1);
        if (int rc = enc_launch_pair(bf16, gh, gt, st)) return rc;
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
    // padding columns must read as zero (a fill kernel rather than a memset, so that the call can be captured)
    {
        const int tail_end = p.Bh + (int)(B + N);
        if (bf16) {
            hipLaunchKernelGGL(enc_zero_pad_kernel<true>, dim3(e.dim), dim3(256), 0, st, dPt, e.dim, p.ncols, (int)B, p.Bh, tail_end);
            hipLaunchKernelGGL(enc_zero_pad_kernel<true>, dim3(e.feat_dim), dim3(256), 0, st, Ft, e.feat_dim, p.ncols, (int)B, p.Bh, tail_end);
        } else {
            hipLaunchKernelGGL(enc_zero_pad_kernel<false>, dim3(e.dim), dim3(256), 0, st, dPt, e.dim, p.ncols, (int)B, p.Bh, tail_end);
            hipLaunchKernelGGL(enc_zero_pad_kernel<false>, dim3(e.feat_dim), dim3(256), 0, st, Ft, e.feat_dim, p.ncols, (int)B, p.Bh, tail_end);
        }
    }
    // the row kernels stage 32 rows in the LDS: more than the default dynamic limit for long rows
    static KgeLdsLimit lim_rows_bf16, lim_rows_f32, lim_gt_bf16, lim_gt_f32;
    {
        const int big = 32 * (1024 + 1) * 4;
        if (lim_rows_bf16.set((const void *)enc_bwd_rows_kernel<true>, big) != KGE_OK ||
            lim_rows_f32.set((const void *)enc_bwd_rows_kernel<false>, big) != KGE_OK ||
            lim_gt_bf16.set((const void *)enc_gather_t_kernel<true>, big) != KGE_OK ||
            lim_gt_f32.set((const void *)enc_gather_t_kernel<false>, big) != KGE_OK)
            return KGE_E_HIP;
    }
    const EncRowArgs a = enc_row_args(e, h, t, B, neg, N, seed, step);
    if (p.n > 0) {
        const int grid = (int)((B + 31) / 32 + (B + N + 31) / 32);
        if (bf16) {
            hipLaunchKernelGGL(enc_bwd_rows_kernel<true>, dim3(grid), dim3(256), 32 * (e.dim + 1) * 4, st, a, proj, de, g_es, dPt, p.Bh, p.ncols);
            hipLaunchKernelGGL(enc_gather_t_kernel<true>, dim3(grid), dim3(256), 32 * (e.feat_dim + 1) * 4, st, a, e.feat, e.feat_ld, e.feat_dim, Ft, p.Bh, p.ncols);
        } else {
            hipLaunchKernelGGL(enc_bwd_rows_kernel<false>, dim3(grid), dim3(256), 32 * (e.dim + 1) * 4, st, a, proj, de, g_es, dPt, p.Bh, p.ncols);
            hipLaunchKernelGGL(enc_gather_t_kernel<false>, dim3(grid), dim3(256), 32 * (e.feat_dim + 1) * 4, st, a, e.feat, e.feat_ld, e.feat_dim, Ft, p.Bh, p.ncols);
        }
    }
    // G[d, f] = dP^t[d, cols] . F^t[f, cols]^t over the head columns (M_H) and over the tail / negative columns (M_T):
    // one launch, split over the columns, then the partials are summed in split order
    const int per = 32 / p.es;                             // slots per k-step
    float *part_t = part + (size_t)p.nsplit_h * mcount;
    const EncGemm gh = enc_gemm_desc(dPt, p.ncols * p.es, false, nullptr, 0, nullptr, B > 0 ? e.dim : 0, Ft, p.ncols * p.es, e.feat_dim,
                                     part, e.feat_dim, mcount, p.Bh / per, p.kps, p.nsplit_h);
    const EncGemm gt = enc_gemm_desc((const char *)dPt + (size_t)p.Bh * p.es, p.ncols * p.es, false, nullptr, 0, nullptr,
                                     B + N > 0 ? e.dim : 0, (const char *)Ft + (size_t)p.Bh * p.es, p.ncols * p.es, e.feat_dim,
                                     part_t, e.feat_dim, mcount, p.Th / per, p.kps, p.nsplit_t);
    {
        KgeProfScope prof(KGE_PROF_ENC_BWD, st);
        if (int rc = enc_launch_pair(bf16, gh, gt, st)) return rc;
    }
    hipLaunchKernelGGL(enc_split_reduce_kernel, dim3((unsigned)((mcount + 255) / 256)), dim3(256), 0, st, part, gh.nsplit, mcount, g_mh);
    hipLaunchKernelGGL(enc_split_reduce_kernel, dim3((unsigned)((mcount + 255) / 256)), dim3(256), 0, st, part_t, gt.nsplit, mcount, g_mt);
    return kge_launch_status();
}
