// Dispatch of the block-kernel instantiations.
#include "kge_internal.h"
#include <stdlib.h>

int kge_launch_fwd_pp(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st);
int kge_launch_gradt_pp(int kind, int loss, const KgeBlockArgs &a, int own_tiles, int nsplit, hipStream_t st);

// The two-role row-owner kernel serves bf16 rows of 512 bytes without the TransH operands; the environment variable
// KGE_FWD_ONE_ROLE=1 selects the one-role kernel instead (for comparisons).
static bool kge_use_fwd_pp() {
    static const bool on = [] { const char *e = getenv("KGE_FWD_ONE_ROLE"); return !(e && e[0] == '1'); }();
    return on;
}

#define KGE_DECL(name) int kge_launch_block_##name(int, int, bool, int, int, int, const KgeBlockArgs &, int, int, hipStream_t);
KGE_DECL(f32_score) KGE_DECL(f32_fwd_ls) KGE_DECL(f32_fwd_sm) KGE_DECL(f32_gradt_ls) KGE_DECL(f32_gradt_sm)
KGE_DECL(bf16_score) KGE_DECL(bf16_fwd_ls) KGE_DECL(bf16_fwd_sm) KGE_DECL(bf16_gradt_ls) KGE_DECL(bf16_gradt_sm)

// whether the row-owner pass of this configuration runs the two-role kernel (which needs no transposed negatives)
bool kge_fwd_pp_applies(bool bf16, int rb, bool transh, int dsplit) {
    return bf16 && rb == 512 && !transh && dsplit == 1 && kge_use_fwd_pp();
}

// the same for the pass over the negatives (one own fragment per wave there; needs no transposed queries);
// KGE_GRADT_ONE_ROLE=1 selects the one-role kernel
bool kge_gradt_pp_applies(bool bf16, int rb, bool transh, int dsplit) {
    static const bool on = [] { const char *e = getenv("KGE_GRADT_ONE_ROLE"); return !(e && e[0] == '1'); }();
    return bf16 && rb == 512 && !transh && dsplit == 1 && on;
}

int kge_launch_block(bool bf16, int rb, int mode, bool transh, int kind, int loss, int dsplit, const KgeBlockArgs &a,
                     int own_tiles, int nsplit, hipStream_t st) {
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
    if (kge_gradt_pp_applies(bf16, rb, transh, dsplit)) return kge_launch_gradt_pp(kind, loss, a, own_tiles, nsplit, st);
    if (bf16) return ls ? kge_launch_block_bf16_gradt_ls(rb, mode, transh, kind, loss, dsplit, a, own_tiles, nsplit, st)
                        : kge_launch_block_bf16_gradt_sm(rb, mode, transh, kind, loss, dsplit, a, own_tiles, nsplit, st);
    return ls ? kge_launch_block_f32_gradt_ls(rb, mode, transh, kind, loss, dsplit, a, own_tiles, nsplit, st)
              : kge_launch_block_f32_gradt_sm(rb, mode, transh, kind, loss, dsplit, a, own_tiles, nsplit, st);
}
