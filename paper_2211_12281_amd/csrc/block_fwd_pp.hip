// The two passes of a training call over the score block (MODE_FWD and MODE_GRADT of block_kernel.hpp: loss statistics
// of every query row with the unnormalised gradient of the queries in one pass over the shared negatives, then the
// gradient of the negatives from the finished row constants) as a two-role kernel for the hot configuration: bf16
// operands, rows of 512 bytes (d <= 256), bilinear and distance scorers without the TransH operands.
//
// In the one-role kernel a wave owns 32 rows, keeps 64 registers of own fragments AND 128 registers of gradient
// accumulators, so only one wave fits per SIMD, and its contraction over d, its element-wise epilogue (exponentials,
// sums, packing) and its contraction over the stream index run one after another.  Here the two contractions belong
// to two waves that share a SIMD:
//   wave A (waves 0-3)  round t: MFMAs of tile t, acc[32 stream x 32 own] = X_t . own^t, and under them the epilogue
//                       of tile t-1, whose coefficients go to the LDS
//   wave B (waves 4-7)  round t: out^t[d x 32 own] += Xt_{t-2}[d x 32 stream] . coef_{t-2}
// The coefficient tile of a pair (2 KB: the accumulator layout of A is the B-operand layout of B, lane for lane) and
// the rare rescaling factor of the running reference exponent pass through a double-buffered LDS slot; the one
// workgroup barrier per tile that the staging ring needs anyway orders the hand-over.  The ring holds five tiles: B
// reads tile t-2, A reads tile t, tile t+1 has landed or is landing, tile t+2 is requested.
//
// Only the row-major tile X is staged.  Wave B needs it transposed (for a dimension, 8 consecutive stream entries
// per lane) and gets that from the LDS transpose read of gfx950 (ds_read_b64_tr_b16): inside a group of 16 lanes,
// source lane i points at 4 consecutive 16-bit elements, and lane l receives element l % 4 of the source lanes
// l / 4, l / 4 + 4, l / 4 + 8, l / 4 + 12.  With source lane i at row K[i / 4], dimensions 4 (i % 4) .. + 3, lane l
// receives dimension l of the rows K[0 .. 3]: one read transposes a 4 x 16 patch, two reads give the 8 entries of
// an MFMA operand.  Wave A loads stream row pi(m) = (m & ~7) | ((m & 3) << 1) | ((m >> 2) & 1) as row m of its
// contraction: the four rows K[.] of a read are then two apart, and the chunk swizzle pp_swz() below keeps both
// waves' reads free of bank conflicts.
// Geometry (own tiles of 128 rows, splits over the streamed rows, placement on the dies), operand layouts, epilogue
// arithmetic and outputs are those of the one-role kernel, which stays the reference for every other
// configuration.
#include "block_kernel.hpp"

int kge_launch_fwd_pp(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st);
int kge_launch_gradt_pp(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st);

namespace {

constexpr int PP_RB = 512, PP_DP = 256, PP_KS = 16, PP_NB = 8, PP_ST = 32;
constexpr int PP_X_BYTES = PP_ST * PP_RB;                   // 16 KB: [32 rows][512 bytes], chunk c of row r at c ^ pp_swz(r)
constexpr int PP_STAGE = PP_X_BYTES;
constexpr int PP_AHEAD = 2;                                 // tiles requested ahead of wave A's (3 and 4 measured: no gain)
constexpr int PP_NSTAGE = PP_AHEAD + 3;                     // tiles t - 2 (wave B) .. t + PP_AHEAD (requested)
constexpr int PP_VALU_PER_MFMA = 8;                         // vector instructions scheduled after every MFMA of wave A (2 .. 16 measured: level)
constexpr int PP_SIDE_SLOTS = PP_AHEAD + 3;                 // side information of a tile's 32 stream rows, one copy per A wave
constexpr int PP_XCH = 2048 + 256;                          // coefficients (64 lanes x 32 bytes) + rescaling factors (64 x 4 bytes)
constexpr int pp_lds(int mode) { return PP_NSTAGE * PP_STAGE + PP_SIDE_SLOTS * 4 * (mode == KGE_MODE_FWD ? 256 : 1024) + 4 * 2 * PP_XCH; }
constexpr int PP_LPW_A = 3, PP_LPW_B = 2;                   // asynchronous copies per tile of an A / B wave
__device__ __forceinline__ int pp_pi(int m) { return (m & ~7) | ((m & 3) << 1) | ((m >> 2) & 1); }
// 16-byte chunk c of tile row r sits at position c ^ pp_swz(r) of the row: a bit permutation of r % 16 whose upper two bits
// are (r / 2) % 4.  Sixteen consecutive rows at one chunk index then fall into sixteen different bank groups (wave A's
// fragment reads run at the LDS's full 256 bytes per clock instead of the 128 that an XOR with r % 8 gives), and so do
// the four rows two apart x four chunks that one transpose read of wave B touches.
__device__ __forceinline__ int pp_swz(int r) { return (((r >> 1) & 3) << 2) | (((r >> 3) & 1) << 1) | (r & 1); }
typedef short pp_i16x4 __attribute__((ext_vector_type(4)));
// max over a lane and its partner lane ^ 32 without the LDS crossbar (whose counter would make the caller wait for every
// fragment read in flight): v_permlane32_swap exchanges the upper half of one register with the lower half of another
__device__ __forceinline__ float pp_max_halves(float v) {
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
static_assert(pp_lds(KGE_MODE_GRADT) <= 160 * 1024, "LDS budget");

// MODE_FWD: own = queries, stream = negatives (statistics of the loss + gradient of the queries);
// MODE_GRADT: own = negatives, stream = queries (gradient of the negatives from the finished row constants).
template <int MODE, int KIND, int LOSS>
__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void kge_pp_kernel(const KgeBlockArgs a) {
    constexpr bool FWD = MODE == KGE_MODE_FWD;
    constexpr int SIDE_WAVE = FWD ? 256 : 1024;             // per A wave: 64 x 4 bytes of squared norms, or 64 x 16 bytes of row info
    constexpr int SIDE_SLOT = 4 * SIDE_WAVE;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    char *side_ring = lds + PP_NSTAGE * PP_STAGE;
    char *xch_base = side_ring + PP_SIDE_SLOTS * SIDE_SLOT;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, g = lane >> 5;
    const bool role_b = wave >= 4;
    const int pair = wave & 3;
    // placement as in the one-role kernel: workgroups that stream the same negatives share a die
    const int xcd = blockIdx.x & 7, kk = blockIdx.x >> 3;
    int own_tile, split;
    if (a.xcd_per == 1) { own_tile = kk % a.own_tiles; split = xcd + 8 * (kk / a.own_tiles); }
    else { split = xcd / a.xcd_per; own_tile = kk * a.xcd_per + xcd % a.xcd_per; }
    if (own_tile >= a.own_tiles || split >= a.nsplit) return;
    const int oidx = own_tile * 128 + pair * 32 + lr;       // the pair's own row of this lane
    const int str_limit = FWD ? a.N : a.B;                  // valid stream rows
    const int t0 = split * a.tiles_per_split;
    const int t1 = min(a.str_tiles, t0 + a.tiles_per_split);
    const bool work = t1 > t0;

    // ---- staging: every wave copies 2 KB of the tile ------------------------------------------------------
    int x_off[2];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
        const int byte = (wave * 2 + jj) * 1024 + lane * 16;
        const int r = byte / PP_RB, pos = (byte % PP_RB) / 16;
        x_off[jj] = r * PP_RB + ((pos ^ pp_swz(r)) * 16);
    }
    auto issue = [&](int tile, int slot) {
        tile = tile < t1 ? tile : t1 - 1;                   // past the end: a harmless repeat keeps vmcnt uniform
        const uint32_t sbase = lds0 + (slot % PP_NSTAGE) * PP_STAGE;
        const char *src = (const char *)a.str + (size_t)tile * PP_ST * PP_RB;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
            kge_async_copy16(src + x_off[jj], __builtin_amdgcn_readfirstlane(sbase + (wave * 2 + jj) * 1024));
        if (!role_b) {
            const uint32_t sside = lds0 + PP_NSTAGE * PP_STAGE + (slot % PP_SIDE_SLOTS) * SIDE_SLOT + pair * SIDE_WAVE;
            if constexpr (FWD) kge_async_copy4(a.tn + tile * PP_ST + lr, __builtin_amdgcn_readfirstlane(sside));
            else kge_async_copy16(a.rowinfo + tile * PP_ST + lr, __builtin_amdgcn_readfirstlane(sside));
        }
    };

    if (!role_b) {
        // =========================== role A: scores, loss weights, coefficients ===========================
        uint4 own[PP_KS];
        {
            const char *p = (const char *)a.own + (size_t)oidx * PP_RB + g * 16;
#pragma unroll
            for (int ks = 0; ks < PP_KS; ++ks) own[ks] = *(const uint4 *)(p + ks * 32);
        }
        float o_qn = FWD ? a.rowinfo[oidx].qn : a.tn[oidx];   // squared norm of the own row
        float sum1 = 0.f, st_m = -INFINITY, st_l = 0.f, st_acc = 0.f;
        int frag_off[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const int R = pp_pi(lr);                        // row m of the contraction is stream row pi(m) of the tile
            frag_off[b] = R * PP_RB + 16 * ((2 * b + g) ^ pp_swz(R));    // chunk 2 ks + g of k-step ks = b (mod 8)
        }
        const float xscale = (LOSS == KGE_LOGSIGMOID ? a.adv_temp : 1.f) * KGE_LOG2E;
        if (work) {
#pragma unroll
            for (int u = 0; u < PP_AHEAD; ++u) issue(t0 + u, u);
        }
        // the own operand must have arrived before the loop (a wait inside it would drain the ring)
#pragma unroll
        for (int ks = 0; ks < PP_KS; ++ks) asm volatile("" : "+v"(own[ks].x), "+v"(own[ks].y), "+v"(own[ks].z), "+v"(own[ks].w));
        asm volatile("" : "+v"(o_qn));
        // register i holds row 8 (i / 4) + 4 g + i % 4 of the contraction = stream row pi(.) of the tile
        int srow[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) srow[i] = pp_pi(8 * (i >> 2) + 4 * g + (i & 3));
        float sv[16], dv[16], x2[16];
        float rsc = 1.f;
        // first half of the epilogue of tile t: scores (distance scorers: by the norm expansion, entries where it
        // cancels are redone by direct differences), then the exponents x2 of the weights - FWD: relative to the
        // row's running reference st_m, which a tile that exceeds it by more than KGE_TAU raises (rare: what the row
        // has accumulated is rescaled, here and in wave B); GRADT: from the finished row constants of the queries
        // side values of a tile's 32 stream rows (squared norms; GRADT: the row constants K), read BEFORE the next
        // tile's fragments so that waiting for them does not wait for the fragments
        float side_n[16], side_k[16];
        auto load_side = [&](int slot) {
            const char *side = side_ring + (slot % PP_SIDE_SLOTS) * SIDE_SLOT + pair * SIDE_WAVE;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if constexpr (KIND == KGE_KIND_DIST) side_n[i] = FWD ? *(const float *)(side + srow[i] * 4) : *(const float *)(side + srow[i] * 16);
                if constexpr (!FWD) side_k[i] = *(const float *)(side + srow[i] * 16 + 8);      // -inf for padded queries
            }
        };
        auto epi1 = [&](int t, const kge_f32x16 &acc) {
            if constexpr (KIND == KGE_KIND_MULT) {
#pragma unroll
                for (int i = 0; i < 16; ++i) { sv[i] = acc[i]; dv[i] = 0.f; }
            } else {
                float d2[16], thr[16];
                bool cancel = false;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float tnv = side_n[i];                // |t|^2 or |q|^2
                    d2[i] = fmaf(-2.f, acc[i], o_qn + tnv);
                    thr[i] = 1e-3f * (o_qn + tnv);
                    cancel = cancel || d2[i] < thr[i];
                }
                if (__any(cancel)) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        if (d2[i] < thr[i]) {
                            const int sidx = t * PP_ST + srow[i];
                            d2[i] = kge_direct_d2<true, false>((const char *)a.own + (size_t)oidx * PP_RB,
                                                               (const char *)a.str + (size_t)sidx * PP_RB, nullptr, PP_DP);
                        }
                        asm volatile("" ::: "memory");  // keeps the branch from being turned into selects
                    }
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float dd = fmaxf(d2[i], 0.f);
                    const float inv = dd > 0.f ? __builtin_amdgcn_rsqf(dd) : 0.f;
                    dv[i] = inv;
                    sv[i] = -dd * inv;
                }
            }
            rsc = 1.f;
            if constexpr (FWD) {
                const float m_neg = st_m > -INFINITY ? -st_m : 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) x2[i] = fmaf(sv[i], xscale, m_neg);
                if (t * PP_ST + PP_ST > str_limit) {            // padding entries -> -inf
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (t * PP_ST + srow[i] >= str_limit) x2[i] = -INFINITY;
                    asm volatile("" ::: "memory");              // a rarely taken branch, not sixteen selects per tile
                }
                float tm = -INFINITY;
#pragma unroll
                for (int i = 0; i < 16; ++i) tm = fmaxf(tm, x2[i]);
                tm = pp_max_halves(tm);                          // both lanes of an own row share the reference
                const bool have = st_m > -INFINITY;
                const bool trip = tm > (have ? KGE_TAU : -INFINITY);
                if (__any(trip)) {
                    const float m_new = trip ? (have ? tm + st_m : tm) : st_m;
                    const float shift = trip ? -tm : 0.f;
                    rsc = trip ? (have ? kge_exp2(-tm) : 0.f) : 1.f;
                    st_m = m_new;
                    st_l *= rsc; st_acc *= rsc; sum1 *= rsc;
#pragma unroll
                    for (int i = 0; i < 16; ++i) x2[i] += shift;
                }
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) x2[i] = fmaf(sv[i], xscale, side_k[i]);
            }
        };
        // second half: weights, loss sums, coefficients -> LDS (straight-line vector work: it runs under the
        // contraction of the NEXT tile, which the caller issues in the same block)
        auto epi2 = [&](int slot) {
            float coef[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float e = kge_exp2(x2[i]);
                float u = e;
                if constexpr (FWD) st_l += e;
                if constexpr (LOSS == KGE_LOGSIGMOID) {
                    const float y = a.gamma + sv[i];
                    const float tt = kge_exp2(-fabsf(y) * KGE_LOG2E);
                    const float rcp = __builtin_amdgcn_rcpf(1.f + tt);
                    const float sig = y >= 0.f ? rcp : tt * rcp;
                    if constexpr (FWD) {
                        const float softplus = fmaxf(y, 0.f) + KGE_LN2 * kge_log2(1.f + tt);
                        if (e > 0.f) st_acc = fmaf(e, softplus, st_acc);
                    }
                    u = e * sig;
                }
                const float c1 = KIND == KGE_KIND_DIST ? u * dv[i] : u;
                coef[i] = c1;
                if constexpr (KIND == KGE_KIND_DIST) sum1 += c1;
            }
            char *x = xch_base + (pair * 2 + (slot & 1)) * PP_XCH;
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
                *(uint4 *)(x + s2 * 1024 + lane * 16) =
                    make_uint4(kge_pack_bf16x2(coef[8 * s2 + 0], coef[8 * s2 + 1]), kge_pack_bf16x2(coef[8 * s2 + 2], coef[8 * s2 + 3]),
                               kge_pack_bf16x2(coef[8 * s2 + 4], coef[8 * s2 + 5]), kge_pack_bf16x2(coef[8 * s2 + 6], coef[8 * s2 + 7]));
            *(float *)(x + 2048 + lane * 4) = rsc;
        };
        // the sixteen fragments of a tile are requested together, right after the barrier
        auto load_tile = [&](int slot, uint4 (&av)[PP_KS]) {
            const char *stage = lds + (slot % PP_NSTAGE) * PP_STAGE;
#pragma unroll
            for (int k = 0; k < PP_KS; ++k) av[k] = *(const uint4 *)(stage + frag_off[k & 7] + 256 * (k >> 3));
        };
        auto mma_tile = [&](const uint4 (&av)[PP_KS], kge_f32x16 &acc) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
            for (int k = 0; k < PP_KS; ++k) acc = kge_mma16<true>(acc, av[k], own[k]);
        };
        // The wave is one tile ahead with its contraction: round t issues the MFMAs of tile t and, while they run,
        // finishes the epilogue of tile t - 1 (whose coefficients wave B picks up in round t + 1).
        if (work) {
            kge_f32x16 accp;
            kge_wait_vmcnt<(PP_AHEAD - 1) * PP_LPW_A>();                     // tile t0 has landed (this wave's part); tile t0 + 1 may be in flight
            __syncthreads();
            issue(t0 + PP_AHEAD, PP_AHEAD);
            {
                uint4 av[PP_KS];
                load_tile(0, av);
                mma_tile(av, accp);
            }
            for (int t = t0 + 1; t < t1; ++t) {
                kge_wait_vmcnt<(PP_AHEAD - 1) * PP_LPW_A>();
                __syncthreads();
                issue(t + PP_AHEAD, t - t0 + PP_AHEAD);
                uint4 av[PP_KS];
                load_side(t - 1 - t0);
                load_tile(t - t0, av);
                epi1(t - 1, accp);
                kge_f32x16 acc;
                mma_tile(av, acc);
                epi2(t - 1 - t0);
                // one MFMA, then a share of the epilogue's vector instructions, sixteen times
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, PP_VALU_PER_MFMA, 0);
                }
                accp = acc;
            }
            kge_wait_vmcnt<(PP_AHEAD - 1) * PP_LPW_A>();
            __syncthreads();
            issue(t1 + PP_AHEAD, t1 - t0 + PP_AHEAD);
            load_side(t1 - 1 - t0);
            epi1(t1 - 1, accp);
            epi2(t1 - 1 - t0);
            kge_wait_vmcnt<(PP_AHEAD - 1) * PP_LPW_A>();                     // the last round belongs to the B waves
            __syncthreads();
            issue(t1 + 1 + PP_AHEAD, t1 - t0 + 1 + PP_AHEAD);
            kge_wait_vmcnt<0>();                            // no copy may be in flight when the LDS is released
        }
        st_l += __shfl_xor(st_l, 32); st_acc += __shfl_xor(st_acc, 32); sum1 += __shfl_xor(sum1, 32);
        if (g == 0) {
            a.sum_part[(size_t)split * a.own_pad + oidx] = make_float4(sum1, 0.f, 0.f, 0.f);
            if constexpr (FWD) a.stat_part[(size_t)split * a.own_pad + oidx] = make_float4(st_m, st_l, st_acc, 0.f);
        }
    } else {
        // =========================== role B: gradient of the queries =====================================
        kge_f32x16 acc2[PP_NB];
#pragma unroll
        for (int b = 0; b < PP_NB; ++b)
            for (int i = 0; i < 16; ++i) acc2[b][i] = 0.f;
        // transpose reads: this lane is source i16 of its group of 16 (dimension sub-block q16 of a 32-block, lane half g):
        // it points at row 16 f + 8 hh + rx of the tile, dimensions blk 32 + q16 16 + 4 (i16 % 4) .. + 3
        const int i16 = lane & 15, q16 = (lane >> 4) & 1, rx = 2 * (i16 >> 2) + g;
        int tr_off[2][2], tr_blk[2][PP_NB];
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) tr_off[f][hh] = (16 * f + 8 * hh + rx) * PP_RB;
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
#pragma unroll
            for (int blk = 0; blk < PP_NB; ++blk)
                tr_blk[hh][blk] = (((blk * 4 + q16 * 2 + ((i16 & 3) >> 1)) ^ pp_swz(8 * hh + rx)) * 16) + (i16 & 1) * 8;
        if (work) {
#pragma unroll
            for (int u = 0; u < PP_AHEAD; ++u) issue(t0 + u, u);
            for (int t = t0; t <= t1 + 1; ++t) {
                kge_wait_vmcnt<(PP_AHEAD - 1) * PP_LPW_B>();
                __syncthreads();
                issue(t + PP_AHEAD, t - t0 + PP_AHEAD);
                if (t < t0 + 2) continue;                   // nothing to consume yet: wave A hands tile t - 2 over in round t - 1
                const int slot = t - 2 - t0;
                const char *xs = lds + (slot % PP_NSTAGE) * PP_STAGE;
                const char *x = xch_base + (pair * 2 + (slot & 1)) * PP_XCH;
                uint4 bf[2];
                bf[0] = *(const uint4 *)(x + lane * 16);
                bf[1] = *(const uint4 *)(x + 1024 + lane * 16);
                const float rsc = *(const float *)(x + 2048 + lane * 4);
                if (__any(rsc != 1.f)) {
#pragma unroll
                    for (int b = 0; b < PP_NB; ++b) {
                        for (int i = 0; i < 16; ++i) acc2[b][i] *= rsc;
                        asm volatile("" ::: "memory");      // rarely executed: keep it out of the selects
                    }
                }
                // dimension block blk: two k-steps f, each operand two transpose reads hh (entries 4 hh .. + 3 of this lane
                // half: rows 16 f + 8 hh + 2 kk + g = pi of the contraction rows 16 f + 8 hh + 4 g + kk).  The reads run two
                // blocks ahead of the MFMAs; the scheduling barriers keep that order.
                uint4 av2[PP_NB][2];
                auto load_blk = [&](int blk) {
#pragma unroll
                    for (int f = 0; f < 2; ++f)
#pragma unroll
                        for (int hh = 0; hh < 2; ++hh) {
                            const pp_i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                (pp_i16x4 __attribute__((address_space(3))) *)(xs + tr_off[f][hh] + tr_blk[hh][blk]));
                            const uint2 u = __builtin_bit_cast(uint2, v);
                            if (hh == 0) { av2[blk][f].x = u.x; av2[blk][f].y = u.y; } else { av2[blk][f].z = u.x; av2[blk][f].w = u.y; }
                        }
                };
                load_blk(0); load_blk(1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int blk = 0; blk < PP_NB; ++blk) {
                    if (blk + 2 < PP_NB) load_blk(blk + 2);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int f = 0; f < 2; ++f) acc2[blk] = kge_mma16<true>(acc2[blk], av2[blk][f], bf[f]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            kge_wait_vmcnt<0>();
        }
#pragma unroll
        for (int blk = 0; blk < PP_NB; ++blk)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int dcol = blk * 32 + 8 * q4 + 4 * g;
                const size_t o = ((size_t)split * a.own_pad + oidx) * PP_DP + dcol;
                *(float4 *)(a.acc_part + o) = make_float4(acc2[blk][4 * q4], acc2[blk][4 * q4 + 1], acc2[blk][4 * q4 + 2], acc2[blk][4 * q4 + 3]);
            }
    }
}

template <int MODE, int KIND, int LOSS>
int pp_launch(const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st) {
    auto kern = kge_pp_kernel<MODE, KIND, LOSS>;
    constexpr int LDS = pp_lds(MODE);
    static KgeLdsLimit lds_limit;
    if (lds_limit.set((const void *)kern, LDS) != KGE_OK) return KGE_E_HIP;
    if ((int64_t)own_tiles * 128 != a.own_pad || a.dp != PP_DP) return KGE_E_INVALID_ARG;
    KgeBlockArgs b = a;
    b.own_tiles = own_tiles; b.nsplit = nsplit;
    int groups;
    if (nsplit >= 8) { b.xcd_per = 1; groups = own_tiles * ((nsplit + 7) / 8); }
    else {
        int s2 = 1;
        while (s2 < nsplit) s2 <<= 1;
        b.xcd_per = 8 / s2;
        groups = (own_tiles + b.xcd_per - 1) / b.xcd_per;
    }
    hipLaunchKernelGGL(kern, dim3(8 * groups), dim3(512), LDS, st, b);
    return kge_launch_status();
}

template <int MODE>
int pp_dispatch(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st) {
    if (kind == KGE_KIND_MULT) return loss == KGE_LOGSIGMOID ? pp_launch<MODE, KGE_KIND_MULT, 0>(a, own_tiles, nsplit, st)
                                                             : pp_launch<MODE, KGE_KIND_MULT, 1>(a, own_tiles, nsplit, st);
    return loss == KGE_LOGSIGMOID ? pp_launch<MODE, KGE_KIND_DIST, 0>(a, own_tiles, nsplit, st)
                                  : pp_launch<MODE, KGE_KIND_DIST, 1>(a, own_tiles, nsplit, st);
}

}  // namespace

int kge_launch_fwd_pp(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st) {
    return pp_dispatch<KGE_MODE_FWD>(kind, loss, a, own_tiles, nsplit, st);
}
int kge_launch_gradt_pp(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st) {
    return pp_dispatch<KGE_MODE_GRADT>(kind, loss, a, own_tiles, nsplit, st);
}
