// Instantiations of the block kernel: f32 operands, pass "fwd_sm" (split over files to bound compile time).
#include "block_kernel.hpp"

#define KGE_INST(RB, MODE, TH, KIND, LOSS, DS) \
    if (rb == RB && mode == MODE && transh == TH && kind == KIND && loss == LOSS && dsplit == DS) \
        return kge_block_launch<false, RB, MODE, TH, KIND, LOSS, DS>(a, own_tiles, nsplit, st);

int kge_launch_block_f32_fwd_sm(int rb, int mode, bool transh, int kind, int loss, int dsplit, const KgeBlockArgs &a,
                         int own_tiles, int nsplit, hipStream_t st) {
    KGE_INST(512, KGE_MODE_FWD, false, KGE_KIND_MULT, 1, 1)
    KGE_INST(512, KGE_MODE_FWD, false, KGE_KIND_DIST, 1, 1)
    KGE_INST(1024, KGE_MODE_FWD, false, KGE_KIND_MULT, 1, 1)
    KGE_INST(1024, KGE_MODE_FWD, false, KGE_KIND_DIST, 1, 1)
    KGE_INST(512, KGE_MODE_FWD, true, KGE_KIND_DIST, 1, 1)
    return KGE_E_UNSUPPORTED;
}
