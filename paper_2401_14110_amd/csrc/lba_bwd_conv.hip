// lba_bwd_conv.hip -- the recompute call reading A as im2col rows of an NHWC tensor of E4M3 codes (AMODE 2):
// floor rounding, sequential order, plain and mixed grids.
#include "lba_device.h"
#include "lba_launch.h"

namespace lba {
hipError_t launch_fast_bwd_conv(const Plan& pl, hipStream_t st) {
    if (pl.amode != 2 || pl.events != 1 || pl.round != LBA_ROUND_FLOOR || pl.order != LBA_ORDER_SEQ || pl.kp.batch != 1)
        return hipErrorInvalidValue;
    if (pl.prod_mode != PM_FLUSH && pl.prod_mode != PM_FLUSH_CLAMP) return hipErrorInvalidValue;
    const dim3 block(256);
    const bool uf = pl.kp.uf_mask != nullptr;
    if (pl.mix_tail > 0) {
        const dim3 grid(pl.grid_x, 1, 1);
#define LBA_BWDM(PM) do { if (uf) hipLaunchKernelGGL((lba_fast_bwd_conv_mixed_kernel<PM, LBA_ROUND_FLOOR, true>), grid, block, 0, st, pl.kp); \
                          else    hipLaunchKernelGGL((lba_fast_bwd_conv_mixed_kernel<PM, LBA_ROUND_FLOOR, false>), grid, block, 0, st, pl.kp); } while (0)
        if (pl.prod_mode == PM_FLUSH) LBA_BWDM(PM_FLUSH); else LBA_BWDM(PM_FLUSH_CLAMP);
#undef LBA_BWDM
    } else {
        const dim3 grid(pl.grid_x, pl.grid_y, 1);
#define LBA_BWD(PM) do { if (uf) hipLaunchKernelGGL((lba_fast_bwd_kernel<PM, LBA_ROUND_FLOOR, LBA_ORDER_SEQ, true, 2>), grid, block, 0, st, pl.kp); \
                         else    hipLaunchKernelGGL((lba_fast_bwd_kernel<PM, LBA_ROUND_FLOOR, LBA_ORDER_SEQ, false, 2>), grid, block, 0, st, pl.kp); } while (0)
        if (pl.prod_mode == PM_FLUSH) LBA_BWD(PM_FLUSH); else LBA_BWD(PM_FLUSH_CLAMP);
#undef LBA_BWD
    }
    return hipGetLastError();
}
}  // namespace lba
