// lba_fast_odd.hip -- instantiations of lba_fast_kernel with the round-to-odd nearest-even rounding
// (RND_RNE_ODD: accumulator formats whose nearest-even rounding is not exact after one FP32 rounding).
#include "lba_launch_fast.h"

namespace lba {
template <int ORDER>
static hipError_t launch_odd(const Plan& pl, hipStream_t st) {
    const dim3 grid(pl.grid_x, pl.grid_y, pl.kp.batch), block(256);
#define LBA_ODD(PM) hipLaunchKernelGGL((lba_fast_kernel<4, 4, LBA_FAST_BK, PM, RND_RNE_ODD, ORDER, 0>), grid, block, 0, st, pl.kp)
    switch (pl.prod_mode) {
        case PM_IDENT:       LBA_ODD(PM_IDENT); break;
        case PM_FLUSH:       LBA_ODD(PM_FLUSH); break;
        case PM_FLUSH_CLAMP: LBA_ODD(PM_FLUSH_CLAMP); break;
        default: return hipErrorInvalidValue;
    }
#undef LBA_ODD
    return hipGetLastError();
}

hipError_t launch_fast_odd(const Plan& pl, hipStream_t st) {
    if (pl.tm != 4 || pl.tn != 4 || pl.amode || pl.round != LBA_ROUND_RNE) return hipErrorInvalidValue;
    return pl.order == LBA_ORDER_CHUNK16 ? launch_odd<LBA_ORDER_CHUNK16>(pl, st) : launch_odd<LBA_ORDER_SEQ>(pl, st);
}
}  // namespace lba
