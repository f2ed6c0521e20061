// lba_diff.hip -- instantiations of lba_fast_diff_kernel (the DIFF plane in the scaled domain).
#include "lba_device.h"
#include "lba_launch.h"

namespace lba {
template <int RND>
static hipError_t launch_diff_rounding(const Plan& pl, hipStream_t st) {
    const bool mixed = pl.mix_tail > 0;                     // 64 x 64 workgroups, then 32 x 32 ones on the last rows
    const dim3 grid(pl.grid_x, mixed ? 1 : pl.grid_y, mixed ? 1 : pl.kp.batch), block(256);
#define LBA_DIFF(PM, ORDER)                                                                                      \
    do {                                                                                                        \
        if (mixed) hipLaunchKernelGGL((lba_fast_diff_mixed_kernel<PM, RND, ORDER>), grid, block, 0, st, pl.kp);      \
        else       hipLaunchKernelGGL((lba_fast_diff_kernel<PM, RND, ORDER>), grid, block, 0, st, pl.kp);            \
    } while (0)
    if (pl.amode || (pl.prod_mode != PM_FLUSH && pl.prod_mode != PM_FLUSH_CLAMP)) return hipErrorInvalidValue;
    if (pl.order == LBA_ORDER_CHUNK16) {
        if (pl.prod_mode == PM_FLUSH) LBA_DIFF(PM_FLUSH, LBA_ORDER_CHUNK16); else LBA_DIFF(PM_FLUSH_CLAMP, LBA_ORDER_CHUNK16);
    } else {
        if (pl.prod_mode == PM_FLUSH) LBA_DIFF(PM_FLUSH, LBA_ORDER_SEQ); else LBA_DIFF(PM_FLUSH_CLAMP, LBA_ORDER_SEQ);
    }
#undef LBA_DIFF
    return hipGetLastError();
}

hipError_t launch_fast_diff(const Plan& pl, hipStream_t st) {
    return pl.round == LBA_ROUND_FLOOR ? launch_diff_rounding<LBA_ROUND_FLOOR>(pl, st) : launch_diff_rounding<LBA_ROUND_RNE>(pl, st);
}
}  // namespace lba
