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
    const int uf = pl.kp.uf_mask != nullptr ? (pl.uf_class ? 2 : 1) : 0;   // as launch_fast_bwd_rounding
#define LBA_UF3(CALL, PM) do { if (uf == 2) CALL(PM, 2); else if (uf == 1) CALL(PM, 1); else CALL(PM, 0); } while (0)
    if (pl.mix_tail > 0) {
        const dim3 grid(pl.grid_x, 1, 1);
#define LBA_BWDM(PM, UF) hipLaunchKernelGGL((lba_fast_bwd_conv_mixed_kernel<PM, LBA_ROUND_FLOOR, UF>), grid, block, 0, st, pl.kp)
        if (pl.prod_mode == PM_FLUSH) LBA_UF3(LBA_BWDM, PM_FLUSH); else LBA_UF3(LBA_BWDM, PM_FLUSH_CLAMP);
#undef LBA_BWDM
    } else {
        const dim3 grid(pl.grid_x, pl.grid_y, 1);
#define LBA_BWD(PM, UF) hipLaunchKernelGGL((lba_fast_bwd_kernel<PM, LBA_ROUND_FLOOR, LBA_ORDER_SEQ, UF, 2>), grid, block, 0, st, pl.kp)
        if (pl.prod_mode == PM_FLUSH) LBA_UF3(LBA_BWD, PM_FLUSH); else LBA_UF3(LBA_BWD, PM_FLUSH_CLAMP);
#undef LBA_BWD
    }
#undef LBA_UF3
    return hipGetLastError();
}
}  // namespace lba
