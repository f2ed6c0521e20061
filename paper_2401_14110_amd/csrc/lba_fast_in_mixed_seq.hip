// lba_fast_in_mixed_seq.hip -- instantiations of lba_fast_in_mixed_kernel (other operand formats / rounded products on
// the mixed grid) for the sequential order.
#include "lba_launch_fast.h"

namespace lba {
hipError_t launch_fast_in_mixed_seq(const Plan& pl, hipStream_t st) {
    if (pl.amode != 1 || pl.events || pl.kp.batch != 1 || pl.mix_tail <= 0 || pl.order != LBA_ORDER_SEQ) return hipErrorInvalidValue;
    const dim3 grid(pl.grid_x, 1, 1), block(256);
    const KParams& kp = pl.kp;
#define LBA_MIX(PM, RND) hipLaunchKernelGGL((lba_fast_in_mixed_kernel<LBA_FAST_BK, PM, RND, LBA_ORDER_SEQ>), grid, block, 0, st, kp)
#define LBA_MIX_ROUNDING(RND)                                         \
    switch (pl.prod_mode) {                                           \
        case PM_IDENT:       LBA_MIX(PM_IDENT, RND); break;           \
        case PM_FLUSH:       LBA_MIX(PM_FLUSH, RND); break;           \
        case PM_FLUSH_CLAMP: LBA_MIX(PM_FLUSH_CLAMP, RND); break;     \
        case PM_TRUNC:       LBA_MIX(PM_TRUNC, RND); break;           \
        case PM_TRUNC_CLAMP: LBA_MIX(PM_TRUNC_CLAMP, RND); break;     \
        case PM_RNE:         LBA_MIX(PM_RNE, RND); break;             \
        default:             LBA_MIX(PM_RNE_CLAMP, RND); break;       \
    }
    if (pl.round == LBA_ROUND_FLOOR) { LBA_MIX_ROUNDING(LBA_ROUND_FLOOR) } else { LBA_MIX_ROUNDING(LBA_ROUND_RNE) }
#undef LBA_MIX_ROUNDING
#undef LBA_MIX
    return hipGetLastError();
}
}  // namespace lba
