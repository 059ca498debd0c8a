// The pass over the negatives of the sampled-softmax loss for the bilinear scorers (bf16 rows of 512 bytes), WITHOUT
// recomputing the scores: the forward kernel of block_sym.hip has left, for every (query, negative) pair, the weight
// p~ = exp2(log2(e) s - ref) in bf16, ref being the fixed reference of the query's row in that forward workgroup.  The
// gradient coefficient of the pair is p~ exp2(ref + K) with the finished row constant K, and the factor exp2(ref + K)
// depends on the query and on the forward split only - so it is folded into the QUERY rows: for every forward split s the
// row finish writes q'_s[b] = bf16(exp2(ref_s[b] + K[b]) q[b]), and this kernel computes
//     dT[n, :] = sum_b p~[b, n] q'_s(n)[b, :]
// as one contraction per workgroup (half the matrix work of the kernel that recomputes the scores, and no exponentials).
//
// Workgroup: 128 own negatives x all 256 dimensions, four waves as in block_sym.hip: wave (oh, sh) holds
// out^t[dims 128 sh .. + 127][negatives 64 oh .. + 63].  A round takes 64 queries: their scaled rows (32 KB) and the
// weights of 64 queries x 128 negatives (16 KB) come into the LDS by asynchronous copies, three rounds deep.
//
// Layouts.  A forward workgroup (128 queries, one split of the negatives) wrote one 4 KB record per round of 64 negatives
// and wave (oh_f, sh_f): lane (lr, g_f), own block ob, k-step f holds 16 bytes = eight weights of query 64 oh_f + 32 ob + lr
// against the negatives at rows 16 f + 8 h + 2 e + g_f (h = 0, 1 the 8-byte half, e = 0 .. 3) of the wave's 32 rows.
// Here the roles are exchanged - a lane needs, for ONE negative, eight queries - which is what the LDS transpose read
// gives: inside a group of 16 lanes, source lane i = 4 b + a points at the 8-byte unit (query K[b], four negatives of unit
// a), and lane l receives, for the queries K[0 .. 3], negative l % 4 of unit l / 4.  With K[j] = 16 k + 8 hh + 2 j + g
// (k the k-step, g the lane half) the eight queries of a lane are exactly those that the transpose reads of the scaled
// query tile deliver for the other operand (same order as in block_sym.hip), so the contraction index agrees.  Column
// n = lane % 32 of an output block is then the negative at row 8 (2 G + a / 2) + 2 (n % 4) + a % 2 of its 32-row group,
// G = n / 16, a = (n % 16) / 4: the write-out puts every column where it belongs.
#include "block_kernel.hpp"

namespace {

constexpr int GP_RB = 512, GP_DP = 256, GP_ST = 64;
constexpr int GP_QSTAGE = GP_ST * GP_RB;                    // 32 KB: 64 scaled query rows, chunk c of row r at c ^ gp_swz(r)
constexpr int GP_PSTAGE = 16 * 1024;                        // 16 KB: [oh][sh_f][4 KB record]
constexpr int GP_NSTAGE = 3;
constexpr int gp_lds() { return GP_NSTAGE * (GP_QSTAGE + GP_PSTAGE); }
static_assert(gp_lds() <= 160 * 1024, "LDS budget");

__device__ __forceinline__ int gp_swz(int r) { return (((r >> 1) & 3) << 2) | (((r >> 3) & 1) << 1) | (r & 1); }
typedef short gp_i16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void gp_copy16(const void *base, uint32_t off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(off), "s"(base) : "memory");
}
// the same for data that is read once (the weights): no reason to keep it in the caches
__device__ __forceinline__ void gp_copy16_stream(const void *base, uint32_t off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_addr), "v"(off), "s"(base) : "memory");
}

// a pointer that is the same in every lane of the wave, for the compiler's benefit (scalar registers)
__device__ __forceinline__ const char *gp_uniform(const char *p) {
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const char *)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(1, 1)))
void kge_gradp_kernel(const KgeBlockArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    char *pst_base = lds + GP_NSTAGE * GP_QSTAGE;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, g = lane >> 5;
    const int oh = wave >> 1, sh = wave & 1;
    // placement: the own tiles whose negatives one forward split scored stream the same scaled queries (q'_fs) - they go
    // to ONE die (workgroups are dealt to the eight dies in turn), so that a die's L2 holds one q'_fs instead of all
    const int xcd = blockIdx.x & 7, kk = blockIdx.x >> 3;
    const int tpf = a.ps_rounds >> 1, per_group = tpf * a.nsplit;          // own tiles per forward split; work items per group
    const int group = xcd + 8 * (kk / per_group), within = kk % per_group;
    const int own_tile = group * tpf + within / a.nsplit, split = within % a.nsplit;
    if (own_tile >= a.own_tiles) return;
    // rounds of 64 queries; only rounds that hold a valid query are visited
    const int tps = a.tiles_per_split >> 1;
    const int tiles = min(a.str_tiles >> 1, (a.B + GP_ST - 1) / GP_ST);
    const int t0 = split * tps;
    const int t1 = min(tiles, t0 + tps);
    const bool work = t1 > t0;
    // the forward workgroups that scored these 128 negatives: split fs, rounds ft0 and ft0 + 1 of it
    const int fs = (2 * own_tile) / a.ps_rounds, ft0 = 2 * own_tile - fs * a.ps_rounds;
    const char *qsrc = (const char *)a.str + (size_t)fs * a.str_tiles * KGE_STREAM_TILE * GP_RB;   // q'_fs: [Bp][256] bf16

    // ---- staging ---------------------------------------------------------------------------------------------
    // queries: as in block_sym.hip, a copy fills two consecutive LDS rows (1 KB); copy (aa, e) of wave w takes the row pair
    // 8 aa + 4 e + w.  weights: wave w copies the record of (forward round ft0 + w / 2, forward wave (oh_f, w % 2)) as it is.
    uint32_t x_off[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int r = 2 * (4 * e + wave) + g, pos = lane & 31;
        x_off[e] = r * GP_RB + ((pos ^ gp_swz(r)) * 16);
    }
    // (the 16 bytes of forward lane (lr, g_f) land at position 2 lr + g_f of their 1 KB piece: the sixteen 8-byte units that
    // one transpose read touches then lie in sixteen different bank groups)
    const uint32_t p_src = ((lane >> 1) + 32 * (lane & 1)) * 16;
    auto issue = [&](int tile, int slot) {
        tile = __builtin_amdgcn_readfirstlane(tile < t1 ? tile : t1 - 1);   // past the end: a harmless repeat keeps the copy counts uniform
        const uint32_t qbase = lds0 + (slot % GP_NSTAGE) * GP_QSTAGE + wave * 1024;
        const char *src = gp_uniform(qsrc + (size_t)tile * GP_ST * GP_RB);
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            const int aa = jj >> 1, e = jj & 1;
            gp_copy16(src + aa * 16 * GP_RB, x_off[e], __builtin_amdgcn_readfirstlane(qbase + aa * 8192 + e * 4096));
        }
        // 64 queries = half (oh_f) of the forward own tile tile / 2
        const int ftile = tile >> 1, ohf = tile & 1;
        const char *rec = gp_uniform((const char *)a.pstore +
                          ((((size_t)ftile * a.ps_nsplit + fs) * a.ps_rounds + ft0 + (wave >> 1)) * 4 + 2 * ohf + (wave & 1)) * 4096);
        const uint32_t pbase = lds0 + (uint32_t)(pst_base - lds) + (slot % GP_NSTAGE) * GP_PSTAGE + wave * 4096;
#pragma unroll
        for (int c = 0; c < 4; ++c) gp_copy16_stream(rec + c * 1024, p_src, __builtin_amdgcn_readfirstlane(pbase + c * 1024));
    };

    kge_f32x16 acc2[4][2];                                  // out^t[dims 128 sh + 32 blk ..][negatives 64 oh + 32 nb ..]
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc2[blk][nb][i] = 0.f;

    // transpose reads.  Queries (operand A): this lane is source i16 of its group of 16 (dimension sub-block q16, lane half
    // g) and points at row 16 k + 8 hh + rx of the tile, dimensions 128 sh + 32 blk + 16 q16 + 4 (i16 % 4) .. + 3.
    // Weights (operand B): source i16 = 4 b + a points at query 16 k + 8 hh + 2 b + g (own block k / 2 of the record, lane
    // (16 (k % 2) + 8 hh + 2 b + g) + 32 (a % 2), which the copy has put at position 2 lr + g_f of the piece), k-step
    // G = (lane / 16) % 2 of the record, half a / 2.
    const int i16 = lane & 15, q16 = (lane >> 4) & 1, rx = 2 * (i16 >> 2) + g;
    int tr_blk[2][4];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh)
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
            tr_blk[hh][blk] = ((((4 * sh + blk) * 4 + q16 * 2 + ((i16 & 3) >> 1)) ^ gp_swz(8 * hh + rx)) * 16) + (i16 & 1) * 8;
    const int ua = i16 & 3;
    const int p_lane = oh * 8192 + q16 * 1024 + (ua >> 1) * 8 + (2 * rx + (ua & 1)) * 16;

    auto load_a = [&](const char *qs, int k, int blk, uint4 &v4) {
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const gp_i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (gp_i16x4 __attribute__((address_space(3))) *)(qs + (16 * k + 8 * hh + rx) * GP_RB + tr_blk[hh][blk]));
            const uint2 u = __builtin_bit_cast(uint2, v);
            if (hh == 0) { v4.x = u.x; v4.y = u.y; } else { v4.z = u.x; v4.w = u.y; }
        }
    };
    auto load_b = [&](const char *ps, int k, int nb, uint4 &v4) {
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const gp_i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (gp_i16x4 __attribute__((address_space(3))) *)(ps + p_lane + nb * 4096 + (k >> 1) * 2048 + (16 * (k & 1) + 8 * hh) * 32));
            const uint2 u = __builtin_bit_cast(uint2, v);
            if (hh == 0) { v4.x = u.x; v4.y = u.y; } else { v4.z = u.x; v4.w = u.y; }
        }
    };

    if (work) {
        issue(t0, 0);
        if (t0 + 1 < t1) issue(t0 + 1, 1);
        for (int t = t0; t < t1; ++t) {
            const int slot = t - t0;
            // tile t has landed when at most the copies of tile t + 1 (12 per wave) are still in flight
            if (t + 1 < t1) kge_wait_vmcnt<12>(); else kge_wait_vmcnt<0>();
            __syncthreads();                                // ... for every wave; and everyone is done with the slot of tile t - 1
            if (t + 2 < t1) issue(t + 2, slot + 2);
            const char *qs = lds + (slot % GP_NSTAGE) * GP_QSTAGE;
            const char *ps = pst_base + (slot % GP_NSTAGE) * GP_PSTAGE;
            uint4 af[2][4], bf[2][2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) load_b(ps, 0, nb, bf[0][nb]);
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) load_a(qs, 0, blk, af[0][blk]);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (k + 1 < 4) {
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb) load_b(ps, k + 1, nb, bf[(k + 1) & 1][nb]);
#pragma unroll
                    for (int blk = 0; blk < 4; ++blk) load_a(qs, k + 1, blk, af[(k + 1) & 1][blk]);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int blk = 0; blk < 4; ++blk)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb) acc2[blk][nb] = kge_mma16<true>(acc2[blk][nb], af[k & 1][blk], bf[k & 1][nb]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // ---- write-out --------------------------------------------------------------------------------------------
    const int G = (lr >> 4) & 1, ca = (lr & 15) >> 2;
    const int nrow = 8 * (2 * G + (ca >> 1)) + 2 * (lr & 3) + (ca & 1);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int oidx = own_tile * 128 + 64 * oh + 32 * nb + nrow;
        if (sh == 0 && g == 0) a.sum_part[(size_t)split * a.own_pad + oidx] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (a.part_bf16) {
            // bf16 partials in column order.  A lane holds columns 8 q4 + 4 g .. + 3 of every 32-column block; the halves of
            // the wave exchange the odd q4 of the lower with the even q4 of the upper, so that a lane writes eight
            // consecutive columns (16 bytes): the lower half those of the even q4, the upper half those of the odd.
            uint16_t *pr = (uint16_t *)a.acc_part + ((size_t)split * a.own_pad + oidx) * GP_DP + 128 * sh + 8 * g;
#pragma unroll
            for (int blk = 0; blk < 4; ++blk)
#pragma unroll
                for (int q2 = 0; q2 < 2; ++q2) {
                    const int e = 8 * q2;                    // first accumulator of q4 = 2 q2
                    const uint32_t x0 = kge_pack_bf16x2(acc2[blk][nb][e], acc2[blk][nb][e + 1]), x1 = kge_pack_bf16x2(acc2[blk][nb][e + 2], acc2[blk][nb][e + 3]);
                    const uint32_t y0 = kge_pack_bf16x2(acc2[blk][nb][e + 4], acc2[blk][nb][e + 5]), y1 = kge_pack_bf16x2(acc2[blk][nb][e + 6], acc2[blk][nb][e + 7]);
                    // (upper half of x <-> lower half of y)
                    const auto s0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
                    const auto s1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
                    *(uint4 *)(pr + blk * 32 + 16 * q2) = make_uint4(s0[0], s1[0], s0[1], s1[1]);
                }
            continue;
        }
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int dcol = (4 * sh + blk) * 32 + 8 * q4 + 4 * g;
                const size_t o = ((size_t)split * a.own_pad + oidx) * GP_DP + dcol;
                *(float4 *)(a.acc_part + o) = make_float4(acc2[blk][nb][4 * q4], acc2[blk][nb][4 * q4 + 1], acc2[blk][nb][4 * q4 + 2], acc2[blk][nb][4 * q4 + 3]);
            }
    }
}

}  // namespace

int kge_launch_gradp(const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st) {
    auto kern = kge_gradp_kernel;
    static KgeLdsLimit lds_limit;
    if (lds_limit.set((const void *)kern, gp_lds()) != KGE_OK) return KGE_E_HIP;
    // the caller's geometry must match: 128 own negatives per workgroup, query tiles counted in 32 rows with an even number
    // per split; a forward split holds a whole number of own tiles (two of its rounds each)
    if ((int64_t)own_tiles * 128 != a.own_pad || a.dp != GP_DP || (a.tiles_per_split & 1) || (a.str_tiles & 1)) return KGE_E_INVALID_ARG;
    if (!a.pstore || a.ps_rounds < 2 || (a.ps_rounds & 1) || a.ps_nsplit < 1) return KGE_E_INVALID_ARG;
    if ((int64_t)a.ps_nsplit * a.ps_rounds < 2 * (int64_t)own_tiles) return KGE_E_INVALID_ARG;
    KgeBlockArgs b = a;
    b.own_tiles = own_tiles; b.nsplit = nsplit;
    const int tpf = a.ps_rounds / 2, ngroups = (own_tiles + tpf - 1) / tpf;         // see the placement in the kernel
    const int per_die = (ngroups + 7) / 8 * tpf * nsplit;
    hipLaunchKernelGGL(kern, dim3(8 * per_die), dim3(256), gp_lds(), st, b);
    return kge_launch_status();
}
