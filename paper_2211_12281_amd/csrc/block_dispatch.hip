// Dispatch of the block-kernel instantiations.
#include "kge_internal.h"
#include <atomic>

int kge_launch_fwd_pp(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st);
int kge_launch_gradt_pp(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st);
int kge_launch_fwd_sym(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st);
int kge_launch_gradt_sym(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st);

// Every job has ONE kernel in the library's own dispatch.  Tests and benchmarks that compare two kernels of one job
// override the choice through kge_debug_select (process-wide, off by default).
static std::atomic<int> g_knobs[KGE_KNOBS];
int kge_knob(int knob) { return g_knobs[knob].load(std::memory_order_relaxed); }
extern "C" int kge_debug_select(int knob, int value) {
    if (knob < 0 || knob >= KGE_KNOBS || value < 0 || value > 1) return KGE_E_INVALID_ARG;
    g_knobs[knob].store(value, std::memory_order_relaxed);
    return KGE_OK;
}

#define KGE_DECL(name) int kge_launch_block_##name(int, int, bool, int, int, int, const KgeBlockArgs &, int, int, hipStream_t);
KGE_DECL(f32_score) KGE_DECL(f32_fwd_ls) KGE_DECL(f32_fwd_sm) KGE_DECL(f32_gradt_ls) KGE_DECL(f32_gradt_sm)
KGE_DECL(bf16_score) KGE_DECL(bf16_fwd_ls) KGE_DECL(bf16_fwd_sm) KGE_DECL(bf16_gradt_ls) KGE_DECL(bf16_gradt_sm)

// whether the row-owner pass of this configuration runs the two-role kernel (which needs no transposed negatives)
bool kge_fwd_pp_applies(bool bf16, int rb, bool transh, int dsplit) {
    return bf16 && rb == 512 && !transh && dsplit == 1 && !kge_knob(KGE_KNOB_FWD_ONE_ROLE);
}

// Bilinear scorers in these configurations run the kernel of block_sym.hip (64 own rows per pair of waves): the pass over
// the negatives with both losses, the pass over the queries with the sampled softmax (whose weights it keeps, so that the
// pass over the negatives of that loss is the contraction of block_gradp.hip).  The two-role kernels serve the distance
// scorers and the log-sigmoid forward pass, and stand in for the others in comparisons (KGE_KNOB_TWO_ROLE).
bool kge_sym_applies(bool bf16, int rb, bool transh, int dsplit) {
    return bf16 && rb == 512 && !transh && dsplit == 1 && !kge_knob(KGE_KNOB_FWD_ONE_ROLE) && !kge_knob(KGE_KNOB_GRADT_ONE_ROLE) &&
           !kge_knob(KGE_KNOB_TWO_ROLE);
}
bool kge_gradp_applies(bool bf16, int rb, bool transh, int dsplit, int kind) {
    return kge_sym_applies(bf16, rb, transh, dsplit) && kind == KGE_KIND_MULT && !kge_knob(KGE_KNOB_GRADT_RECOMPUTE);
}
static bool sym_serves(int mode, int kind, int loss) {
    return kind == KGE_KIND_MULT && (mode == KGE_MODE_GRADT || loss == KGE_SAMPLED_SOFTMAX);
}

// the same for the pass over the negatives (one own fragment per wave there; needs no transposed queries)
bool kge_gradt_pp_applies(bool bf16, int rb, bool transh, int dsplit) {
    return bf16 && rb == 512 && !transh && dsplit == 1 && !kge_knob(KGE_KNOB_GRADT_ONE_ROLE);
}

int kge_launch_block(bool bf16, int rb, int mode, bool transh, int kind, int loss, int dsplit, const KgeBlockArgs &a,
                     int own_tiles, int nsplit, hipStream_t st) {
    const int slot = mode == KGE_MODE_SCORE ? KGE_PROF_BLOCK_SCORE : mode == KGE_MODE_FWD ? KGE_PROF_BLOCK_FWD : KGE_PROF_BLOCK_GRADT;
    KgeProfScope prof(slot, st);
    if (mode == KGE_MODE_FWD && kge_sym_applies(bf16, rb, transh, dsplit) && sym_serves(mode, kind, loss))
        return kge_launch_fwd_sym(kind, loss, a, own_tiles, nsplit, st);
    if (mode == KGE_MODE_GRADT && loss == KGE_SAMPLED_SOFTMAX && a.pstore && kge_gradp_applies(bf16, rb, transh, dsplit, kind)) {
        // the forward pass kept its weights: no scores are recomputed
        KgeBlockArgs b = a;
        b.str = a.str2; b.str2 = nullptr;                    // the queries scaled per forward split
        return kge_launch_gradp(b, own_tiles, nsplit, st);
    }
    if (mode == KGE_MODE_SCORE)
        return bf16 ? kge_launch_block_bf16_score(rb, mode, transh, kind, 0, dsplit, a, own_tiles, nsplit, st)
                    : kge_launch_block_f32_score(rb, mode, transh, kind, 0, dsplit, a, own_tiles, nsplit, st);
    const bool ls = loss == KGE_LOGSIGMOID;
    if (mode == KGE_MODE_FWD) {
        if (kge_fwd_pp_applies(bf16, rb, transh, dsplit)) return kge_launch_fwd_pp(kind, loss, a, own_tiles, nsplit, st);
        if (bf16) return ls ? kge_launch_block_bf16_fwd_ls(rb, mode, transh, kind, loss, dsplit, a, own_tiles, nsplit, st)
                            : kge_launch_block_bf16_fwd_sm(rb, mode, transh, kind, loss, dsplit, a, own_tiles, nsplit, st);
        return ls ? kge_launch_block_f32_fwd_ls(rb, mode, transh, kind, loss, dsplit, a, own_tiles, nsplit, st)
                  : kge_launch_block_f32_fwd_sm(rb, mode, transh, kind, loss, dsplit, a, own_tiles, nsplit, st);
    }
    if (kge_sym_applies(bf16, rb, transh, dsplit) && sym_serves(mode, kind, loss)) return kge_launch_gradt_sym(kind, loss, a, own_tiles, nsplit, st);
    if (kge_gradt_pp_applies(bf16, rb, transh, dsplit)) return kge_launch_gradt_pp(kind, loss, a, own_tiles, nsplit, st);
    if (bf16) return ls ? kge_launch_block_bf16_gradt_ls(rb, mode, transh, kind, loss, dsplit, a, own_tiles, nsplit, st)
                        : kge_launch_block_bf16_gradt_sm(rb, mode, transh, kind, loss, dsplit, a, own_tiles, nsplit, st);
    return ls ? kge_launch_block_f32_gradt_ls(rb, mode, transh, kind, loss, dsplit, a, own_tiles, nsplit, st)
              : kge_launch_block_f32_gradt_sm(rb, mode, transh, kind, loss, dsplit, a, own_tiles, nsplit, st);
}
