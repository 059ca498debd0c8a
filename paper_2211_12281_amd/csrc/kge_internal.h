// Internal declarations shared by the translation units of the gfx950 library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <mutex>
#include "../../include/kge.h"

#define KGE_HIP_TRY(expr)                                   \
    do {                                                    \
        hipError_t e__ = (expr);                            \
        if (e__ != hipSuccess) return KGE_E_HIP;            \
    } while (0)

static inline int kge_launch_status() {
    return hipGetLastError() == hipSuccess ? KGE_OK : KGE_E_HIP;
}

// RAII pair of HIP events around a kernel launch; a no-op unless kge_profile_enable(1) was called.
struct KgeProfScope {
    KgeProfScope(int slot, hipStream_t st);
    ~KgeProfScope();
    int slot_; hipStream_t st_; void *a_, *b_;
};

// Raises a kernel's dynamic LDS limit once per process; safe when several threads make the first launch together.
struct KgeLdsLimit {
    std::once_flag once;
    hipError_t err = hipSuccess;
    int set(const void *kern, int bytes) {
        std::call_once(once, [&] { err = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); });
        return err == hipSuccess ? KGE_OK : KGE_E_HIP;
    }
};

// Kernel choices that only tests and benchmarks override (kge_debug_select); 0 = the library's own choice.
enum { KGE_KNOB_FWD_ONE_ROLE = 0, KGE_KNOB_GRADT_ONE_ROLE = 1, KGE_KNOB_SCORE_F32_MFMA = 2, KGE_KNOB_TWO_ROLE = 3,
       KGE_KNOB_GRADT_RECOMPUTE = 4, KGE_KNOBS = 5 };
int kge_knob(int knob);

static inline int64_t kge_round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// ---------------------------------------------------------------------------------------------
// Tile geometry of the block kernels
// ---------------------------------------------------------------------------------------------
constexpr int KGE_STREAM_TILE = 32;   // rows streamed through LDS per iteration
constexpr int KGE_PAD = 256;          // B and N are padded to this in the workspace copies

enum { KGE_MODE_SCORE = 0, KGE_MODE_FWD = 1, KGE_MODE_GRADT = 2 };
enum { KGE_KIND_MULT = 0, KGE_KIND_DIST = 1 };

// 32-row fragments of its operand that each of a workgroup's four waves owns (the workgroup owns
// 128 times this many rows).  Two where the registers allow it: every fragment read from the LDS then
// feeds two MFMAs, which halves the LDS traffic per flop.  Not with the TransH operands; not in the
// FWD pass, whose gradient accumulators for two fragments of 256 dimensions would take the whole
// accumulator file and more; not in the GRADT pass of the distance scorers, whose epilogue needs
// the registers.
constexpr int kge_block_ow(bool bf16, int rb, bool transh, int mode, int kind) {
    if (!bf16 || rb != 512 || transh || mode == KGE_MODE_FWD) return 1;
    return (mode == KGE_MODE_GRADT && kind == KGE_KIND_DIST) ? 1 : 2;
}

// Workgroups of a block-kernel pass that share a compute unit: the SCORE pass keeps no gradient
// accumulators and fits two, where two ring stages of its tiles fit in half of the LDS.
constexpr int kge_block_occ(bool bf16, int rb, bool transh, int mode) {
    (void)bf16;
    return (mode == KGE_MODE_SCORE && !transh && KGE_STREAM_TILE * rb <= 32 * 1024) ? 2 : 1;
}

// Per-row side information of the queries: squared norm of q, c = w.q (TransH), the per-row
// constant K of the gradient coefficient exp2(x * log2e + K) (log2 domain), squared norm of the
// (rounded) TransH normal.
struct __attribute__((aligned(16))) KgeRowInfo { float qn, c, K, wn; };

// Arguments of one block-kernel launch.  "own" is the operand a workgroup keeps in registers
// (queries when OWN_ROW, negatives otherwise); "str" is the operand streamed through LDS.
struct KgeBlockArgs {
    const void *own, *own2;        // [own_pad][dp]; own2: TransH normals when OWN_ROW
    const void *str, *str2;        // [str_pad][dp]; str2: TransH normals when !OWN_ROW
    const void *strT, *strT2;      // [dp][strT_ld] transposed stream operand(s), GRAD only
    int64_t strT_ld;               // elements
    const KgeRowInfo *rowinfo;     // [Bp]
    const float *tn;               // [Np] squared norms of the negatives
    int32_t B, N;                  // true sizes (padding is masked)
    int32_t dp;                    // padded dim (elements) = RB / sizeof(elem)
    int32_t str_tiles;             // number of stream tiles in total
    int32_t tiles_per_split;       // stream tiles handled by one workgroup
    int32_t kind;                  // KGE_KIND_*
    int32_t loss;                  // kge_loss_t
    float gamma, adv_temp, c_corr; // c_corr: sampled-softmax correction c
    // outputs
    float *S_out;                  // SCORE: [B][N]
    float4 *stat_part;             // FWD: [nsplit][Bp] {running max (log2 domain), sum of weights, weighted loss, 0}
    float *acc_part, *acc_part2;   // FWD / GRADT: [nsplit][own_pad][dp]
    float4 *sum_part;              // FWD / GRADT: [nsplit][own_pad] {s1, s2, s3, 0}
    int32_t own_pad;
    int32_t own_tiles, nsplit;     // launch geometry (the grid is one-dimensional in (split, own tile))
    int32_t xcd_per;               // XCDs that share one split (1 when there are 8 or more splits)
    const float *str_bias;         // FWD, kernel of block_sym.hip: [Np] 0 for a negative, -inf for a padding row (added to its scores)
    // the coefficients of the forward pass, kept for the pass over the negatives (block_sym.hip writes, block_gradp.hip reads):
    // one 4 KB record per (own tile of 128 queries, split, round of 64 negatives, wave), in the writer's register layout
    void *pstore;
    int32_t ps_nsplit, ps_rounds;  // splits and rounds per split of the forward pass that wrote them
    // block_sym.hip (forward pass that keeps its weights) and block_gradp.hip: the split partials of the gradient rows are
    // written as bf16 (round to nearest even), half the bytes that the finishing launch reads back.  acc_part then holds
    // [nsplit][own_pad][dp] bf16: the pass over the negatives in column order; the pass over the queries as dp/2 32-bit
    // words per row, word 64 (c / 128) + c % 64 = columns c (low half) and c + 64 (high half) for c % 128 < 64 - the
    // pairs that one lane of the chain-rule kernel holds.
    int32_t part_bf16;
};

// arguments of the rows' finish that also scales the query rows per forward split (row_finish.hpp)
struct KgeRowFinishQArgs {
    const float4 *stat_part; int nsplit, Bp, B, N, loss; float gamma, c_corr, scale; const float *pos;
    KgeRowInfo *rowinfo; float *lossb, *gpos; const uint16_t *Q; uint16_t *Qs;
};

bool kge_fwd_pp_applies(bool bf16, int rb, bool transh, int dsplit);
bool kge_gradt_pp_applies(bool bf16, int rb, bool transh, int dsplit);
// the kernel of block_sym.hip serves both passes of the same configurations; it walks the stream in tiles of 64 rows
bool kge_sym_applies(bool bf16, int rb, bool transh, int dsplit);
// sampled softmax, bilinear scorers: the pass over the negatives without recomputing the scores (block_gradp.hip);
// kge_gradp_applies: the configurations whose forward pass keeps its weights for it
bool kge_gradp_applies(bool bf16, int rb, bool transh, int dsplit, int kind);
int kge_launch_gradp(const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st);
// launchers implemented in block_*.hip (one file per element type and pass to bound compile time)
int kge_launch_block(bool bf16, int rb, int mode, bool transh, int kind, int loss, int dsplit, const KgeBlockArgs &a,
                     int own_tiles, int nsplit, hipStream_t st);
