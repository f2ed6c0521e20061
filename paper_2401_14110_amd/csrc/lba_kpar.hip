// lba_kpar.hip -- instantiations of lba_kpar_kernel (chunked order, several chunks of an output side by side:
// forward launches with too few outputs to fill the chip otherwise).
#include "lba_device.h"
#include "lba_launch.h"

namespace lba {

template <int TM, int TN, int CPW>
static hipError_t launch_kpar_shape(const Plan& pl, hipStream_t st) {
    const dim3 grid(pl.grid_x, pl.grid_y, 1), block(256);
    const KParams& kp = pl.kp;
#define LBA_KPAR(PM, RND) hipLaunchKernelGGL((lba_kpar_kernel<TM, TN, CPW, PM, RND>), grid, block, 0, st, kp)
#define LBA_KPAR_ROUNDING(RND)                                  \
    switch (pl.prod_mode) {                                     \
        case PM_IDENT: LBA_KPAR(PM_IDENT, RND); break;          \
        case PM_FLUSH: LBA_KPAR(PM_FLUSH, RND); break;          \
        case PM_FLUSH_CLAMP: LBA_KPAR(PM_FLUSH_CLAMP, RND); break; \
        default: return hipErrorInvalidValue;                   \
    }
    if (pl.round == LBA_ROUND_FLOOR) {
        LBA_KPAR_ROUNDING(LBA_ROUND_FLOOR)
    } else if (pl.kp.sh_a == 16) {                          // M = 7: rounding by the bfloat16 conversion
        LBA_KPAR_ROUNDING(RND_RNE_BF16)
    } else {
        LBA_KPAR_ROUNDING(LBA_ROUND_RNE)
    }
#undef LBA_KPAR_ROUNDING
#undef LBA_KPAR
    return hipGetLastError();
}

hipError_t launch_kpar(const Plan& pl, hipStream_t st) {
    if (pl.order != LBA_ORDER_CHUNK16 || pl.events || pl.amode || pl.rne_odd || pl.kp.batch != 1) return hipErrorInvalidValue;
    switch (pl.kpar) {
        case 1: return launch_kpar_shape<4, 4, 1>(pl, st);      // 32 x 32 outputs, 4 chunks in flight
        case 3: return launch_kpar_shape<2, 4, 4>(pl, st);      //  8 x 16 outputs, 16 chunks in flight
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lba
