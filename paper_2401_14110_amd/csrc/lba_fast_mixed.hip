// lba_fast_mixed.hip -- instantiations of lba_fast_mixed_kernel (64 x 64 workgroups, then 32 x 32 ones on the
// last rows of the launch).
#include "lba_device.h"
#include "lba_launch.h"

#ifndef LBA_FAST_BK
#define LBA_FAST_BK 32
#endif

namespace lba {

template <int ORDER>
static hipError_t launch_mixed_order(const Plan& pl, hipStream_t st) {
    const dim3 grid(pl.grid_x, 1, 1), block(256);
    const KParams& kp = pl.kp;
#define LBA_MIX(PM, RND) hipLaunchKernelGGL((lba_fast_mixed_kernel<LBA_FAST_BK, PM, RND, ORDER>), grid, block, 0, st, kp)
#define LBA_MIX_ROUNDING(RND)                                   \
    switch (pl.prod_mode) {                                     \
        case PM_IDENT: LBA_MIX(PM_IDENT, RND); break;           \
        case PM_FLUSH: LBA_MIX(PM_FLUSH, RND); break;           \
        case PM_FLUSH_CLAMP: LBA_MIX(PM_FLUSH_CLAMP, RND); break; \
        default: return hipErrorInvalidValue;                   \
    }
    if (pl.round == LBA_ROUND_FLOOR) {
        LBA_MIX_ROUNDING(LBA_ROUND_FLOOR)
    } else if (pl.kp.sh_a == 16) {
        LBA_MIX_ROUNDING(RND_RNE_BF16)
    } else {
        LBA_MIX_ROUNDING(LBA_ROUND_RNE)
    }
#undef LBA_MIX_ROUNDING
#undef LBA_MIX
    return hipGetLastError();
}

hipError_t launch_fast_mixed(const Plan& pl, hipStream_t st) {
    return pl.order == LBA_ORDER_CHUNK16 ? launch_mixed_order<LBA_ORDER_CHUNK16>(pl, st)
                                         : launch_mixed_order<LBA_ORDER_SEQ>(pl, st);
}

}  // namespace lba
