// Instantiations of the block kernel for f32 operands (split over files to bound compile time).
#include "block_kernel.hpp"

#define KGE_INST(RB, OWN, MODE, TH, DS) \
    if (rb == RB && own_row == OWN && mode == MODE && transh == TH && dsplit == DS) \
        return kge_block_launch<false, RB, OWN, MODE, TH, DS>(a, own_tiles, nsplit, st);

int kge_launch_block_f32_gradt(int rb, bool own_row, int mode, bool transh, const KgeBlockArgs &a,
                         int own_tiles, int nsplit, int dsplit, hipStream_t st) {
    KGE_INST(512, false, KGE_MODE_GRAD, false, 1)
    KGE_INST(1024, false, KGE_MODE_GRAD, false, 1)
    KGE_INST(512, false, KGE_MODE_GRAD, true, 1)
    return KGE_E_UNSUPPORTED;
}
