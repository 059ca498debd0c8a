// The two passes of a training call over the score block for the hot configuration (bf16 operands, rows of 512 bytes,
// bilinear scorers - DistMult, ComplEx): MODE_FWD (sampled softmax) gives the loss statistics of every query row and the
// unnormalised gradient of the queries in one pass over the shared negatives (arXiv 2211.12281, Section 3.1 "Loss
// Functions"; the negatives are shared by the micro-batch, eq. (negsamples)), MODE_GRADT (both losses) the gradient of
// the negatives from the finished row constants.  Every other configuration keeps the kernels of block_fwd_pp.hip and
// block_kernel.hpp.
//
// What bounds such a pass on a compute unit is the LDS: a 32 x 32 x 16 MFMA takes 32 cycles, and the 1 KB operand
// fragment that it reads from the staged tile takes 6-8 cycles of the LDS, which four SIMDs share - so a fragment has to
// feed TWO MFMAs.  That needs 64 own rows per wave in both contractions.  One wave cannot hold 64 rows of operand
// fragments (128 registers) AND their 64 x 256 gradient accumulators (256 registers), so two waves share 64 own rows:
//   workgroup = 4 waves, one per SIMD (up to 512 registers each), 128 own rows, stream tiles of 64 rows
//   wave (oh, sh), oh = own half (64 rows), sh = 0 / 1:
//     phase 1   S^t[32 stream rows (half sh of the tile) x 64 own] = X . own^t        16 fragments, 32 MFMAs
//     epilogue  scores -> loss weights -> coefficients P (bf16), own half kept in registers, copy to the LDS
//     phase 2   out^t[128 dims (half sh) x 64 own] += X^t[128 dims x 64 stream] . P[64 stream x 64 own]
//               P = own half + the partner wave's half from the LDS               16 fragments, 32 MFMAs
// The accumulator layout of phase 1 is the B-operand layout of phase 2 lane for lane (the stream rows of a tile enter
// phase 1 under the permutation pi, as in block_fwd_pp.hip, whose tile layout, chunk swizzle and transpose reads are
// reused here), so the coefficients never change lanes.  Every byte of a tile is read from the LDS exactly once per
// phase and wave.
//
// Pipeline: one barrier per tile; the ring holds three tiles of 32 KB: t - 1, t and t + 1 (landing).  A wave is alone on
// its SIMD and issues in order, so the order of a round is written out (see `round`): the MFMAs form four stages of
// sixteen, the LDS requests and the copies of the next tile go under the first two, the epilogue under the last two.
//
// MODE_FWD weights a score x with exp2(x - ref), ref a reference exponent per own row.  The two waves of a pair see
// different stream rows but feed the same accumulators, so they use the SAME reference: the exact maximum of the
// workgroup's first tile over both waves (exchanged through the LDS once).  It is never raised: the weights of later
// tiles may exceed 1, which costs nothing while they stay finite.  A score that exceeds the reference by more than about
// 2^SY_GUARD (69 in natural units) cannot be handled this way: when a lane's sum of weights ends above 2^SY_GUARD (or is
// not a number), the workgroup does its pass a second time, the reference now being the exact maximum of every row over
// the whole split (one more walk over the tiles finds it).  (The check is on the sums at the end, not on every score: a
// weight that overflowed leaves an infinite sum, and a sum below 2^SY_GUARD bounds every weight.)
#include "block_kernel.hpp"

int kge_launch_fwd_sym(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st);
int kge_launch_gradt_sym(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st);

namespace {

constexpr int SY_RB = 512, SY_DP = 256, SY_KS = 16, SY_ST = 64;
constexpr int SY_STAGE = SY_ST * SY_RB;                     // 32 KB: [64 rows][512 bytes], chunk c of row r at c ^ sy_swz(r)
constexpr int SY_NSTAGE = 3;
constexpr int SY_LPW = SY_STAGE / 1024 / 4;                 // 1 KB copies per wave and tile (8)
constexpr int SY_XCH_WAVE = 4096;                           // coefficients of one wave and tile: [2 own blocks][2 k-steps][64 lanes x 16 bytes]
constexpr int SY_XCH = 4 * SY_XCH_WAVE;
constexpr int SY_POST = 4 * 64 * 4;                         // the first tile's row maxima, 64 own rows per wave (later: the pair's sums at the end)
constexpr float SY_GUARD = 100.f;                           // log2 of the largest weight a fixed reference may produce
constexpr int sy_side_wave(int) { return 256; }             // per wave and stage: 64 x 4 bytes of side values
constexpr int sy_lds(int mode) { return SY_NSTAGE * SY_STAGE + 2 * SY_XCH + 2 * SY_POST + SY_NSTAGE * 4 * sy_side_wave(mode); }
static_assert(sy_lds(KGE_MODE_GRADT) <= 160 * 1024, "LDS budget");

__device__ __forceinline__ int sy_pi(int m) { return (m & ~7) | ((m & 3) << 1) | ((m >> 2) & 1); }
__device__ __forceinline__ int sy_swz(int r) { return (((r >> 1) & 3) << 2) | (((r >> 3) & 1) << 1) | (r & 1); }
typedef short sy_i16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float sy_max_halves(float v) {
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Asynchronous global -> LDS copies with a wave-uniform base address and a 32-bit offset per lane (no vector arithmetic
// per copy): lane l's 16 (4) bytes at base + off go to LDS byte m0 + 16 l (4 l).
__device__ __forceinline__ void sy_copy16(const void *base, uint32_t off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(off), "s"(base) : "memory");
}
__device__ __forceinline__ void sy_copy4(const void *base, uint32_t off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_addr), "v"(off), "s"(base) : "memory");
}

template <int MODE, int LOSS>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(1, 1)))
void kge_sym_kernel(const KgeBlockArgs a) {
    constexpr bool FWD = MODE == KGE_MODE_FWD;
    static_assert(!FWD || LOSS == KGE_SAMPLED_SOFTMAX, "the forward pass of the log-sigmoid loss keeps the two-role kernel");
    // FWD: the score accumulators START from the rows' 0 / -inf, which masks the padding rows for free (the exponent of a
    // weight is log2(e) s - ref)
    constexpr int SIDE_WAVE = sy_side_wave(MODE);
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    char *xch_base = lds + SY_NSTAGE * SY_STAGE;
    char *post_base = xch_base + 2 * SY_XCH;
    char *side_ring = post_base + 2 * SY_POST;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, g = lane >> 5;
    const int oh = wave >> 1, sh = wave & 1, partner = wave ^ 1;
    // placement: workgroups that stream the same rows share a die
    const int xcd = blockIdx.x & 7, kk = blockIdx.x >> 3;
    int own_tile, split;
    if (a.xcd_per == 1) { own_tile = kk % a.own_tiles; split = xcd + 8 * (kk / a.own_tiles); }
    else { split = xcd / a.xcd_per; own_tile = kk * a.xcd_per + xcd % a.xcd_per; }
    if (own_tile >= a.own_tiles || split >= a.nsplit) return;
    const int obase = own_tile * 128 + oh * 64 + lr;        // own row of block ob: obase + 32 ob
    const int str_limit = FWD ? a.N : a.B;                  // valid stream rows
    // tiles of 64 rows; only tiles that hold a valid row are visited
    const int tps = a.tiles_per_split >> 1;
    const int tiles = min(a.str_tiles >> 1, (str_limit + SY_ST - 1) / SY_ST);
    const int t0 = split * tps;
    const int t1 = min(tiles, t0 + tps);
    const bool work = t1 > t0;

    // ---- staging: every wave copies 8 KB of the tile ------------------------------------------------------
    // A copy instruction fills two consecutive LDS rows (1 KB).  Copy jj = (a, e) of wave w takes the row pair
    // 8 a + 4 e + w: the rows' swizzle depends on (e, w, lane) only, so two per-lane offsets serve all eight copies and
    // the rest of the address is wave-uniform.
    uint32_t x_off[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int r = 2 * (4 * e + wave) + g, pos = lane & 31;              // row mod 16, 16-byte position
        x_off[e] = r * SY_RB + ((pos ^ sy_swz(r)) * 16);
    }
    // side values of the wave's 32 stream rows in the order the lanes need them: position 16 g + i holds the value of
    // the row that register i of lane half g scores, so a lane reads its sixteen values as 64 contiguous bytes
    const uint32_t side_row = 32 * sh + 8 * (((lane & 31) >> 2) & 3) + 2 * (lane & 3) + ((lane & 31) >> 4);
    // part jj of the copies of a tile: 0 .. 7 the wave's eight row pairs, 8 the side values.  The vector memory path of a
    // compute unit moves 64 bytes per clock: the 32 KB of a tile keep it busy for 512 cycles, and a wave that issues its
    // copies back to back sits at the issue for most of that - so a round issues them one at a time between its MFMAs.
    auto issue_part = [&](int tile, int slot, int jj) {
        tile = __builtin_amdgcn_readfirstlane(tile < t1 ? tile : t1 - 1);   // past the end: a harmless repeat keeps the copy counts uniform
        if (jj < SY_LPW) {
            const uint32_t sbase = lds0 + (slot % SY_NSTAGE) * SY_STAGE + wave * 1024;
            const char *src = (const char *)a.str + (size_t)tile * SY_ST * SY_RB;
            const int aa = jj >> 1, e = jj & 1;
            sy_copy16(src + aa * 16 * SY_RB, x_off[e], __builtin_amdgcn_readfirstlane(sbase + aa * 8192 + e * 4096));
        } else {
            const uint32_t sside = lds0 + (uint32_t)(side_ring - lds) + ((slot % SY_NSTAGE) * 4 + wave) * SIDE_WAVE;
            // GRADT: the finished row constant K of a query (-inf for a padded one); FWD: 0, or -inf for a padding row
            if constexpr (FWD) sy_copy4(a.str_bias + (size_t)tile * SY_ST, side_row * 4, __builtin_amdgcn_readfirstlane(sside));
            else sy_copy4(&a.rowinfo[(size_t)tile * SY_ST].K, side_row * 16, __builtin_amdgcn_readfirstlane(sside));
        }
    };
    auto issue = [&](int tile, int slot) {
#pragma unroll
        for (int jj = 0; jj <= SY_LPW; ++jj) issue_part(tile, slot, jj);
    };

    // ---- own operand: two blocks of 32 rows as B fragments ------------------------------------------------
    uint4 own[2][SY_KS];
#pragma unroll
    for (int ob = 0; ob < 2; ++ob) {
        const char *p = (const char *)a.own + (size_t)(obase + 32 * ob) * SY_RB + g * 16;
#pragma unroll
        for (int ks = 0; ks < SY_KS; ++ks) own[ob][ks] = *(const uint4 *)(p + ks * 32);
    }
    kge_f32x16 acc2[4][2];                                  // out^t[dims 128 sh + 32 blk ..][own block ob]
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int ob = 0; ob < 2; ++ob)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc2[blk][ob][i] = 0.f;
    float ref[2] = {-INFINITY, -INFINITY}, st_l[2] = {0.f, 0.f};

    // phase 1 fragments: row m of the contraction is row 32 sh + pi(m) of the tile
    int frag_off[8];
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const int R = 32 * sh + sy_pi(lr);
        frag_off[b] = R * SY_RB + 16 * ((2 * b + g) ^ sy_swz(R));
    }
    // (register i of a score block holds contraction row 8 (i / 4) + 4 g + i % 4 = row 8 (i / 4) + 2 (i % 4) + g of the
    // wave's half tile)
    // phase 2 transpose reads (see block_fwd_pp.hip): source lane i16 of a group of 16, dimension sub-block q16
    const int i16 = lane & 15, q16 = (lane >> 4) & 1, rx = 2 * (i16 >> 2) + g;
    int tr_row[2][2][2], tr_blk[2][4];                      // [0: own half of the tile, 1: partner's][k-step][hh] row offsets, [hh][blk] chunk offsets
#pragma unroll
    for (int w = 0; w < 2; ++w)
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) tr_row[w][f][hh] = (32 * (w == 0 ? sh : 1 - sh) + 16 * f + 8 * hh + rx) * SY_RB;
#pragma unroll
    for (int hh = 0; hh < 2; ++hh)
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
            tr_blk[hh][blk] = ((((4 * sh + blk) * 4 + q16 * 2 + ((i16 & 3) >> 1)) ^ sy_swz(8 * hh + rx)) * 16) + (i16 & 1) * 8;

    const float xscale = (LOSS == KGE_LOGSIGMOID ? a.adv_temp : 1.f) * KGE_LOG2E;

    // the own operand must have arrived before the loop (a wait inside it would wait for the ring's copies too)
#pragma unroll
    for (int ob = 0; ob < 2; ++ob) {
#pragma unroll
        for (int ks = 0; ks < SY_KS; ++ks) {
            // 96 of the 128 registers are pinned to the accumulator file, which holds the 128 gradient accumulators and
            // the 32 of a score block besides (MFMA operands may come from either file; nothing else reads these)
            if (ob == 0 || ks < 8) asm volatile("" : "+a"(own[ob][ks].x), "+a"(own[ob][ks].y), "+a"(own[ob][ks].z), "+a"(own[ob][ks].w));
            else asm volatile("" : "+v"(own[ob][ks].x), "+v"(own[ob][ks].y), "+v"(own[ob][ks].z), "+v"(own[ob][ks].w));
        }
    }

    // ---- pieces of a round --------------------------------------------------------------------------------
    // GRADT: the row constants K of the wave's 32 streamed queries, in the order of the lane's sixteen entries
    float side_k[16];
    auto load_side = [&](int slot) {
        const float4 *side = (const float4 *)(side_ring + ((slot % SY_NSTAGE) * 4 + wave) * SIDE_WAVE + 64 * g);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 v = side[q];
            side_k[4 * q] = v.x; side_k[4 * q + 1] = v.y; side_k[4 * q + 2] = v.z; side_k[4 * q + 3] = v.w;
        }
    };
    // weight, loss sum and coefficient of one entry with score sv and exponent x2
    auto entry_coef = [&](int ob, float sv, float x2) -> float {
        const float e = kge_exp2(x2);
        if constexpr (FWD) st_l[ob] += e;
        if constexpr (LOSS == KGE_LOGSIGMOID) {
            const float y = a.gamma + sv;
            const float tt = kge_exp2(-fabsf(y) * KGE_LOG2E);
            const float rcp = __builtin_amdgcn_rcpf(1.f + tt);
            return e * (y >= 0.f ? rcp : tt * rcp);
        }
        return e;
    };
    // phase 2 fragment (w: 0 own half of the tile / 1 partner's, k-step f, blk): two transpose reads hh
    auto load_frag = [&](const char *xs, int w, int f, int blk, uint4 &v4) {
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const sy_i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (sy_i16x4 __attribute__((address_space(3))) *)(xs + tr_row[w][f][hh] + tr_blk[hh][blk]));
            const uint2 u = __builtin_bit_cast(uint2, v);
            if (hh == 0) { v4.x = u.x; v4.y = u.y; } else { v4.z = u.x; v4.w = u.y; }
        }
    };
    using yes = std::true_type;
    using no = std::false_type;
    // FWD: the coefficients of tile t (exp2 of the score's exponent less the reference, bf16) go to memory as the wave holds
    // them, for the pass over the negatives: 4 KB per wave and tile.  They are stored at the START of the next round (from
    // the registers that phase 2 still reads), so that the wait for the ring's copies at the top of a round finds the
    // stores of the round before long finished.
    auto store_coefs = [&](int t, const uint4 (&pc)[2][2]) {
        if constexpr (FWD) {
            if (a.pstore) {
                char *dst = (char *)a.pstore + ((((size_t)own_tile * a.ps_nsplit + split) * a.ps_rounds + (t - t0)) * 4 + wave) * 4096 + lane * 16;
#pragma unroll
                for (int ob = 0; ob < 2; ++ob)
#pragma unroll
                    for (int f = 0; f < 2; ++f) {           // (read once, much later: no reason to keep it in the caches)
                        typedef unsigned sy_u32x4 __attribute__((ext_vector_type(4)));
                        const sy_u32x4 v = { pc[ob][f].x, pc[ob][f].y, pc[ob][f].z, pc[ob][f].w };
                        __builtin_nontemporal_store(v, (sy_u32x4 *)(dst + ob * 2048 + f * 1024));
                    }
            }
        }
    };

    // One round.  Tile t (ring slot `slot`) gets its scores and its coefficients; tile t - 1 its phase 2.  The order
    // keeps the matrix pipe fed while everything else is in flight:
    //   A  phase 2 of tile t - 1, own half: its eight fragments were requested before the barrier (trf), the coefficients
    //      are the wave's own (pown) - nothing to wait for, while the fragments of tile t, the partner's coefficients
    //      and the side values arrive
    //   B  phase 1, own block 0            (16 MFMAs)
    //   C  phase 1, own block 1            (16 MFMAs) with the epilogue of block 0, one entry per MFMA
    //   D  phase 2 of tile t - 1, partner's half (16 MFMAs) with the epilogue of block 1; the own-half fragments of
    //      tile t are requested for the next round
    // HAVE_P2 false: the first round (no tile before it).
    auto round = [&](auto have_p2, int t, int slot, kge_f32x16 (&accs)[2], uint4 (&trf)[8], uint4 (&pown)[2][2]) {
        constexpr bool P2 = decltype(have_p2)::value;
        const char *stage = lds + (slot % SY_NSTAGE) * SY_STAGE;
        const char *xs = lds + ((slot + SY_NSTAGE - 1) % SY_NSTAGE) * SY_STAGE;
        uint4 av[SY_KS], pp[2][2], trp[8];
        uint32_t pk[4];
        uint4 pnew[2][2];
        // ---- requests of the round ----
        const char *xprev = xch_base + ((slot - 1) & 1) * SY_XCH;
#pragma unroll
        for (int k = 0; k < 8; ++k) av[k] = *(const uint4 *)(stage + frag_off[k]);
        if constexpr (!FWD) load_side(slot);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (P2) store_coefs(t - 1, pown);
        // ---- A ----
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int f = n >> 2, blk = n & 3;
            av[8 + n] = *(const uint4 *)(stage + frag_off[n] + 256);    // (the sixteen fragments serve both own blocks: every byte of the tile is read once)
            if (!(n & 1)) issue_part(t + 1, slot + 1, n >> 1);      // the next tile's copies, spread over the stages A and B
            if constexpr (P2) {
#pragma unroll
                for (int ob = 0; ob < 2; ++ob)
                    acc2[blk][ob] = kge_mma16<true>(acc2[blk][ob], trf[n], pown[ob][f]);
                load_frag(xs, 1, f, blk, trp[n]);           // the partner half's fragments, for stage D
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // one entry of the epilogue of block ob (entries come in pairs: a pair is one packed register)
        float cprev = 0.f;
        auto entry = [&](int ob, int i) {
            const float s1 = accs[ob][i];
            const float x1 = FWD ? fmaf(s1, xscale, -ref[ob])            // (-inf for a padding row: its accumulator started there)
                                 : fmaf(s1, xscale, side_k[i]);
            const float c1 = entry_coef(ob, s1, x1);
            if (i & 1) {
                pk[(i >> 1) & 3] = kge_pack_bf16x2(cprev, c1);
                if ((i & 7) == 7) {                         // a k-step's eight entries: one B fragment, kept for the next round and handed to the partner
                    pnew[ob][i >> 3] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                    *(uint4 *)(xch_base + (slot & 1) * SY_XCH + wave * SY_XCH_WAVE + ob * 2048 + (i >> 3) * 1024 + lane * 16) = pnew[ob][i >> 3];
                }
            } else cprev = c1;
        };
        // FWD: a score block's accumulators start from the rows' 0 / -inf, read from the LDS for each block (straight into
        // the accumulator registers: nothing is held in between)
        auto start_value = [&]() {
            kge_f32x16 v = {};
            if constexpr (FWD) {
                const float4 *side = (const float4 *)(side_ring + ((slot % SY_NSTAGE) * 4 + wave) * SIDE_WAVE + 64 * g);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 x = side[q];
                    v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
                }
            }
            return v;
        };
        // ---- B ----
        kge_f32x16 init = start_value();
#pragma unroll
        for (int k = 0; k < SY_KS; ++k) {
            if ((k & 3) == 1) issue_part(t + 1, slot + 1, 4 + (k >> 2));
            if (k == 15) issue_part(t + 1, slot + 1, SY_LPW);
            if constexpr (P2) {                             // the partner's coefficients of tile t - 1
                if (k < 4) pp[k >> 1][k & 1] = *(const uint4 *)(xprev + partner * SY_XCH_WAVE + (k >> 1) * 2048 + (k & 1) * 1024 + lane * 16);
            }
            if (k >= 8) load_frag(stage, 0, (k - 8) >> 2, (k - 8) & 3, trf[k - 8]);   // own half of tile t: phase 2 of the next round starts with it
            accs[0] = kge_mma16<true>(k == 0 ? init : accs[0], av[k], own[0][k]);
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- C ----
        init = start_value();
#pragma unroll
        for (int k = 0; k < SY_KS; ++k) {
            accs[1] = kge_mma16<true>(k == 0 ? init : accs[1], av[k], own[1][k]);
            entry(0, k);
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- D ----
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int f = n >> 2, blk = n & 3;
            if constexpr (P2) {
#pragma unroll
                for (int ob = 0; ob < 2; ++ob)
                    acc2[blk][ob] = kge_mma16<true>(acc2[blk][ob], trp[n], pp[ob][f]);
            }
            entry(1, 2 * n);
            entry(1, 2 * n + 1);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int ob = 0; ob < 2; ++ob)
#pragma unroll
            for (int f = 0; f < 2; ++f) pown[ob][f] = pnew[ob][f];
    };

    // FWD: a pass whose weights outgrow the first tile's reference (see the head of the file) is done a second time, with the
    // exact row maxima of the whole split as reference - nothing can overflow then.  The decision is the workgroup's.
    for (int attempt = 0; work && attempt < (FWD ? 2 : 1); ++attempt) {
        kge_f32x16 accs[2];
        uint4 trf[8], pown[2][2];
        if constexpr (FWD) {
            if (attempt == 1) {
                // (rare, and written for brevity, not speed: one tile in flight at a time)
                float tm[2] = {-INFINITY, -INFINITY};
                for (int t = t0; t < t1; ++t) {
                    __syncthreads();                        // everyone is done with stage 0
                    issue(t, 0);
                    kge_wait_vmcnt<0>();
                    __syncthreads();
                    load_side(0);
#pragma unroll
                    for (int ob = 0; ob < 2; ++ob) {
                        kge_f32x16 acc;
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[i] = side_k[i];
#pragma unroll
                        for (int k = 0; k < SY_KS; ++k)
                            acc = kge_mma16<true>(acc, *(const uint4 *)(lds + frag_off[k & 7] + 256 * (k >> 3)), own[ob][k]);
#pragma unroll
                        for (int i = 0; i < 16; ++i) tm[ob] = fmaxf(tm[ob], acc[i] * xscale);
                    }
                }
                __syncthreads();
#pragma unroll
                for (int ob = 0; ob < 2; ++ob) {
                    tm[ob] = sy_max_halves(tm[ob]);
                    *(float *)(post_base + wave * 256 + (32 * ob + lr) * 4) = tm[ob];
                }
                __syncthreads();
#pragma unroll
                for (int ob = 0; ob < 2; ++ob) {
                    ref[ob] = fmaxf(tm[ob], *(const float *)(post_base + partner * 256 + (32 * ob + lr) * 4));
                    st_l[ob] = 0.f;
                }
#pragma unroll
                for (int blk = 0; blk < 4; ++blk)
#pragma unroll
                    for (int ob = 0; ob < 2; ++ob)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc2[blk][ob][i] = 0.f;
                __syncthreads();
            }
        }
        issue(t0, 0);
        kge_wait_vmcnt<0>();
        __syncthreads();                                    // tile t0 has landed
        if constexpr (FWD) {
            if (attempt == 0) {
                // the reference starts as the exact maximum of the first tile over both waves of the pair
                const char *stage = lds;
                load_side(0);                               // (0 / -inf of the tile's rows)
                float tm[2];
#pragma unroll
                for (int ob = 0; ob < 2; ++ob) {
                    kge_f32x16 acc;
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[i] = side_k[i];
#pragma unroll
                    for (int k = 0; k < SY_KS; ++k)
                        acc = kge_mma16<true>(acc, *(const uint4 *)(stage + frag_off[k & 7] + 256 * (k >> 3)), own[ob][k]);
                    tm[ob] = -INFINITY;
#pragma unroll
                    for (int i = 0; i < 16; ++i) tm[ob] = fmaxf(tm[ob], acc[i] * xscale);
                    tm[ob] = sy_max_halves(tm[ob]);
                    *(float *)(post_base + wave * 256 + (32 * ob + lr) * 4) = tm[ob];
                }
                __syncthreads();
#pragma unroll
                for (int ob = 0; ob < 2; ++ob)
                    ref[ob] = fmaxf(tm[ob], *(const float *)(post_base + partner * 256 + (32 * ob + lr) * 4));
            }
        }
        round(no{}, t0, 0, accs, trf, pown);
        for (int t = t0 + 1; t < t1; ++t) {
            const int slot = t - t0;
            kge_wait_vmcnt<0>();                            // this wave's part of tile t has landed
            __syncthreads();
            round(yes{}, t, slot, accs, trf, pown);
            // the score blocks keep accumulator registers of their own for the whole loop (else the register allocator
            // parks gradient accumulators elsewhere around every phase 1)
#pragma unroll
            for (int ob = 0; ob < 2; ++ob)
#pragma unroll
                for (int i = 0; i < 16; i += 4)
                    asm volatile("" ::"a"(accs[ob][i]), "a"(accs[ob][i + 1]), "a"(accs[ob][i + 2]), "a"(accs[ob][i + 3]));
        }
        kge_wait_vmcnt<0>();                                // no copy may be in flight when the LDS is released
        __syncthreads();
        // phase 2 of the last tile
        store_coefs(t1 - 1, pown);
        {
            const int pslot = t1 - 1 - t0;
            const char *xs = lds + (pslot % SY_NSTAGE) * SY_STAGE;
            const char *x = xch_base + (pslot & 1) * SY_XCH;
            uint4 pp[2][2], trp[8];
#pragma unroll
            for (int ob = 0; ob < 2; ++ob)
#pragma unroll
                for (int f = 0; f < 2; ++f) pp[ob][f] = *(const uint4 *)(x + partner * SY_XCH_WAVE + ob * 2048 + f * 1024 + lane * 16);
#pragma unroll
            for (int n = 0; n < 8; ++n) load_frag(xs, 1, n >> 2, n & 3, trp[n]);
#pragma unroll
            for (int n = 0; n < 8; ++n)
#pragma unroll
                for (int ob = 0; ob < 2; ++ob) {
                    acc2[n & 3][ob] = kge_mma16<true>(acc2[n & 3][ob], trf[n], pown[ob][n >> 2]);
                    acc2[n & 3][ob] = kge_mma16<true>(acc2[n & 3][ob], trp[n], pp[ob][n >> 2]);
                }
        }
        if constexpr (FWD) {
            const float lim = __builtin_amdgcn_ldexpf(1.f, (int)SY_GUARD);
            if (!__syncthreads_or(!(st_l[0] <= lim) || !(st_l[1] <= lim))) break;
        }
    }

    // ---- write-out: the pair's sums are added through the LDS ----------------------------------------------
    __syncthreads();
    float *fin = (float *)post_base;                        // [wave][64]
#pragma unroll
    for (int ob = 0; ob < 2; ++ob) {
        st_l[ob] += __shfl_xor(st_l[ob], 32);
        if (sh == 1 && g == 0) fin[wave * 64 + 32 * ob + lr] = st_l[ob];
    }
    __syncthreads();
#pragma unroll
    for (int ob = 0; ob < 2; ++ob) {
        const int oidx = obase + 32 * ob;
        if (sh == 0 && g == 0) {
            a.sum_part[(size_t)split * a.own_pad + oidx] = make_float4(0.f, 0.f, 0.f, 0.f);     // (distance scorers' sums: none here)
            if constexpr (FWD) a.stat_part[(size_t)split * a.own_pad + oidx] = make_float4(ref[ob], st_l[ob] + fin[partner * 64 + 32 * ob + lr], 0.f, 0.f);
        }
        if (a.part_bf16) {
            // bf16 partials: a lane holds columns c .. c + 3 (blk) and c + 64 .. c + 67 (blk + 2): four words of the row
            uint32_t *pw = (uint32_t *)a.acc_part + ((size_t)split * a.own_pad + oidx) * (SY_DP / 2) + 64 * sh + 4 * g;
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *(uint4 *)(pw + blk * 32 + 8 * q4) =
                        make_uint4(kge_pack_bf16x2(acc2[blk][ob][4 * q4], acc2[blk + 2][ob][4 * q4]),
                                   kge_pack_bf16x2(acc2[blk][ob][4 * q4 + 1], acc2[blk + 2][ob][4 * q4 + 1]),
                                   kge_pack_bf16x2(acc2[blk][ob][4 * q4 + 2], acc2[blk + 2][ob][4 * q4 + 2]),
                                   kge_pack_bf16x2(acc2[blk][ob][4 * q4 + 3], acc2[blk + 2][ob][4 * q4 + 3]));
            continue;
        }
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int dcol = (4 * sh + blk) * 32 + 8 * q4 + 4 * g;
                const size_t o = ((size_t)split * a.own_pad + oidx) * SY_DP + dcol;
                *(float4 *)(a.acc_part + o) = make_float4(acc2[blk][ob][4 * q4], acc2[blk][ob][4 * q4 + 1], acc2[blk][ob][4 * q4 + 2], acc2[blk][ob][4 * q4 + 3]);
            }
    }
}

template <int MODE, int LOSS>
int sym_launch(const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st) {
    auto kern = kge_sym_kernel<MODE, LOSS>;
    constexpr int LDS = sy_lds(MODE);
    static KgeLdsLimit lds_limit;
    if (lds_limit.set((const void *)kern, LDS) != KGE_OK) return KGE_E_HIP;
    // the caller's geometry must match: 128 own rows per workgroup, stream tiles counted in 32 rows, an even number per split
    if ((int64_t)own_tiles * 128 != a.own_pad || a.dp != SY_DP || (a.tiles_per_split & 1) || (a.str_tiles & 1)) return KGE_E_INVALID_ARG;
    if (MODE == KGE_MODE_FWD && !a.str_bias) return KGE_E_INVALID_ARG;
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
    hipLaunchKernelGGL(kern, dim3(8 * groups), dim3(256), LDS, st, b);
    return kge_launch_status();
}

}  // namespace

int kge_launch_fwd_sym(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st) {
    if (kind != KGE_KIND_MULT || loss != KGE_SAMPLED_SOFTMAX) return KGE_E_INVALID_ARG;
    return sym_launch<KGE_MODE_FWD, KGE_SAMPLED_SOFTMAX>(a, own_tiles, nsplit, st);
}
int kge_launch_gradt_sym(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st) {
    if (kind != KGE_KIND_MULT) return KGE_E_INVALID_ARG;
    return loss == KGE_LOGSIGMOID ? sym_launch<KGE_MODE_GRADT, KGE_LOGSIGMOID>(a, own_tiles, nsplit, st)
                                  : sym_launch<KGE_MODE_GRADT, KGE_SAMPLED_SOFTMAX>(a, own_tiles, nsplit, st);
}
