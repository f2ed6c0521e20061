// lba_launch_bwd.h -- the launcher template of lba_fast_bwd_kernel, included by lba_bwd.hip (floor) and
// lba_bwd_rne.hip (nearest-even), which instantiate it for their rounding.
#ifndef LBA_LAUNCH_BWD_H_
#define LBA_LAUNCH_BWD_H_

#include "lba_device.h"
#include "lba_launch.h"

namespace lba {

template <int RND>
static hipError_t launch_fast_bwd_rounding(const Plan& pl, hipStream_t st) {
    const dim3 grid(pl.grid_x, pl.grid_y, pl.kp.batch), block(256);
    // 0: no underflow plane; 1: product underflow from the operands' and the product's zero tests; 2: from the product's class
    const int uf = (pl.kp.uf_mask != nullptr || pl.kp.uf_mask2 != nullptr) ? (pl.uf_class ? 2 : 1) : 0;
#define LBA_UF3(CALL, ...) do { if (uf == 2) CALL(__VA_ARGS__, 2); else if (uf == 1) CALL(__VA_ARGS__, 1); else CALL(__VA_ARGS__, 0); } while (0)
    if (pl.amode == 2) return hipErrorInvalidValue;        // launch_fast_bwd_conv
    if (pl.amode) {                                        // im2col rows / other operand formats: floor, sequential order only
        if constexpr (RND == LBA_ROUND_FLOOR) {
#define LBA_BWD1(PM, UF) hipLaunchKernelGGL((lba_fast_bwd_kernel<PM, RND, LBA_ORDER_SEQ, UF, 1>), grid, block, 0, st, pl.kp)
            if (pl.order != LBA_ORDER_SEQ) return hipErrorInvalidValue;
            switch (pl.prod_mode) {
                case PM_FLUSH:       LBA_UF3(LBA_BWD1, PM_FLUSH); break;
                case PM_FLUSH_CLAMP: LBA_UF3(LBA_BWD1, PM_FLUSH_CLAMP); break;
                case PM_TRUNC:       LBA_UF3(LBA_BWD1, PM_TRUNC); break;
                case PM_TRUNC_CLAMP: LBA_UF3(LBA_BWD1, PM_TRUNC_CLAMP); break;
                default: return hipErrorInvalidValue;
            }
#undef LBA_BWD1
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;
        }
    }
    if (pl.prod_mode != PM_FLUSH && pl.prod_mode != PM_FLUSH_CLAMP) return hipErrorInvalidValue;
    if (pl.mix_tail > 0) {                                 // sequential order: mixed grid
        if (pl.order != LBA_ORDER_SEQ) return hipErrorInvalidValue;
        const dim3 mgrid(pl.grid_x, 1, 1);
#define LBA_BWDM(PM, UF) hipLaunchKernelGGL((lba_fast_bwd_mixed_kernel<PM, RND, UF>), mgrid, block, 0, st, pl.kp)
        if (pl.prod_mode == PM_FLUSH) LBA_UF3(LBA_BWDM, PM_FLUSH); else LBA_UF3(LBA_BWDM, PM_FLUSH_CLAMP);
#undef LBA_BWDM
        return hipGetLastError();
    }
#define LBA_BWD(PM, ORDER, UF) hipLaunchKernelGGL((lba_fast_bwd_kernel<PM, RND, ORDER, UF>), grid, block, 0, st, pl.kp)
    if (pl.order == LBA_ORDER_CHUNK16) {
        if (pl.prod_mode == PM_FLUSH) LBA_UF3(LBA_BWD, PM_FLUSH, LBA_ORDER_CHUNK16); else LBA_UF3(LBA_BWD, PM_FLUSH_CLAMP, LBA_ORDER_CHUNK16);
    } else {
        if (pl.prod_mode == PM_FLUSH) LBA_UF3(LBA_BWD, PM_FLUSH, LBA_ORDER_SEQ); else LBA_UF3(LBA_BWD, PM_FLUSH_CLAMP, LBA_ORDER_SEQ);
    }
#undef LBA_BWD
#undef LBA_UF3
    return hipGetLastError();
}

}  // namespace lba
#endif
