// lba_bwd_in_mixed.hip -- the recompute call for other operand formats (AMODE 1) on the mixed grid: floor rounding,
// sequential order, 64 x 64 workgroups for the full rounds and 32 x 32 ones behind them (or throughout).
#include "lba_device.h"
#include "lba_launch.h"

namespace lba {
hipError_t launch_fast_bwd_in_mixed(const Plan& pl, hipStream_t st) {
    if (pl.amode != 1 || pl.events != 1 || pl.round != LBA_ROUND_FLOOR || pl.order != LBA_ORDER_SEQ || pl.kp.batch != 1 ||
        pl.mix_tail <= 0)
        return hipErrorInvalidValue;
    const dim3 grid(pl.grid_x, 1, 1), block(256);
    const int uf = pl.kp.uf_mask != nullptr ? (pl.uf_class ? 2 : 1) : 0;   // as launch_fast_bwd_rounding
#define LBA_BWDM(PM) do { if (uf == 2)      hipLaunchKernelGGL((lba_fast_bwd_in_mixed_kernel<PM, LBA_ROUND_FLOOR, 2>), grid, block, 0, st, pl.kp); \
                          else if (uf == 1) hipLaunchKernelGGL((lba_fast_bwd_in_mixed_kernel<PM, LBA_ROUND_FLOOR, 1>), grid, block, 0, st, pl.kp); \
                          else              hipLaunchKernelGGL((lba_fast_bwd_in_mixed_kernel<PM, LBA_ROUND_FLOOR, 0>), grid, block, 0, st, pl.kp); } while (0)
    switch (pl.prod_mode) {
        case PM_FLUSH:       LBA_BWDM(PM_FLUSH); break;
        case PM_FLUSH_CLAMP: LBA_BWDM(PM_FLUSH_CLAMP); break;
        case PM_TRUNC:       LBA_BWDM(PM_TRUNC); break;
        case PM_TRUNC_CLAMP: LBA_BWDM(PM_TRUNC_CLAMP); break;
        default: return hipErrorInvalidValue;
    }
#undef LBA_BWDM
    return hipGetLastError();
}
}  // namespace lba
