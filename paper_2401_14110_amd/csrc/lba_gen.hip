// lba_gen.hip -- instantiations of lba_gen_kernel (every format, forward and recompute).
#include "lba_device.h"
#include "lba_launch.h"

namespace lba {
hipError_t launch_gen(const Plan& pl, hipStream_t st) {
    const dim3 grid(pl.grid_x, pl.grid_y, pl.kp.batch), block(256);
    const KParams& kp = pl.kp;
    if (pl.events == 2) {                                      // the DIFF plane
        if (pl.order == LBA_ORDER_CHUNK16) {
            if (pl.round == LBA_ROUND_FLOOR) hipLaunchKernelGGL((lba_gen_kernel<LBA_ROUND_FLOOR, false, LBA_ORDER_CHUNK16, true>), grid, block, 0, st, kp);
            else                             hipLaunchKernelGGL((lba_gen_kernel<LBA_ROUND_RNE, false, LBA_ORDER_CHUNK16, true>), grid, block, 0, st, kp);
        } else {
            if (pl.round == LBA_ROUND_FLOOR) hipLaunchKernelGGL((lba_gen_kernel<LBA_ROUND_FLOOR, false, LBA_ORDER_SEQ, true>), grid, block, 0, st, kp);
            else                             hipLaunchKernelGGL((lba_gen_kernel<LBA_ROUND_RNE, false, LBA_ORDER_SEQ, true>), grid, block, 0, st, kp);
        }
    } else if (pl.order == LBA_ORDER_CHUNK16 && pl.events) {
        if (pl.round == LBA_ROUND_FLOOR) hipLaunchKernelGGL((lba_gen_kernel<LBA_ROUND_FLOOR, true, LBA_ORDER_CHUNK16>), grid, block, 0, st, kp);
        else                             hipLaunchKernelGGL((lba_gen_kernel<LBA_ROUND_RNE, true, LBA_ORDER_CHUNK16>), grid, block, 0, st, kp);
    } else if (pl.order == LBA_ORDER_CHUNK16) {
        if (pl.round == LBA_ROUND_FLOOR) hipLaunchKernelGGL((lba_gen_kernel<LBA_ROUND_FLOOR, false, LBA_ORDER_CHUNK16>), grid, block, 0, st, kp);
        else                             hipLaunchKernelGGL((lba_gen_kernel<LBA_ROUND_RNE, false, LBA_ORDER_CHUNK16>), grid, block, 0, st, kp);
    } else if (pl.round == LBA_ROUND_FLOOR) {
        if (pl.events) hipLaunchKernelGGL((lba_gen_kernel<LBA_ROUND_FLOOR, true, LBA_ORDER_SEQ>), grid, block, 0, st, kp);
        else           hipLaunchKernelGGL((lba_gen_kernel<LBA_ROUND_FLOOR, false, LBA_ORDER_SEQ>), grid, block, 0, st, kp);
    } else {
        if (pl.events) hipLaunchKernelGGL((lba_gen_kernel<LBA_ROUND_RNE, true, LBA_ORDER_SEQ>), grid, block, 0, st, kp);
        else           hipLaunchKernelGGL((lba_gen_kernel<LBA_ROUND_RNE, false, LBA_ORDER_SEQ>), grid, block, 0, st, kp);
    }
    return hipGetLastError();
}
}  // namespace lba
