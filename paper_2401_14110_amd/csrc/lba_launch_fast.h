// lba_launch_fast.h -- the launcher template of lba_fast_kernel, included by the lba_fast_*.hip units.
#ifndef LBA_LAUNCH_FAST_H_
#define LBA_LAUNCH_FAST_H_

#include "lba_device.h"
#include "lba_launch.h"

namespace lba {

#ifndef LBA_FAST_BK
#define LBA_FAST_BK 32              // k-depth of a tile of the fast kernel (a multiple of 16)
#endif

template <int TM, int TN, int ORDER, int AMODE = 0>
static hipError_t launch_fast(const Plan& pl, hipStream_t st) {
    const dim3 grid(pl.grid_x, pl.grid_y, pl.kp.batch), block(256);
    const KParams& kp = pl.kp;
#define LBA_LAUNCH(PM, RND) hipLaunchKernelGGL((lba_fast_kernel<TM, TN, LBA_FAST_BK, PM, RND, ORDER, AMODE>), grid, block, 0, st, kp)
    // the truncating product modes (operand formats whose products exceed Q_prod's mantissa) exist for
    // the 4 x 4 lane block of AMODE 0 and 1 only, the nearest-even ones for AMODE = 1 only; the planner never asks for them otherwise
#define LBA_LAUNCH_ROUNDING(RND)                                                        \
    switch (pl.prod_mode) {                                                             \
        case PM_IDENT:       LBA_LAUNCH(PM_IDENT, RND); break;                          \
        case PM_FLUSH:       LBA_LAUNCH(PM_FLUSH, RND); break;                          \
        case PM_FLUSH_CLAMP: LBA_LAUNCH(PM_FLUSH_CLAMP, RND); break;                    \
        case PM_TRUNC:       if constexpr (TM == 4 && TN == 4 && AMODE != 2) { LBA_LAUNCH(PM_TRUNC, RND); break; } else return hipErrorInvalidValue;        \
        case PM_TRUNC_CLAMP: if constexpr (TM == 4 && TN == 4 && AMODE != 2) { LBA_LAUNCH(PM_TRUNC_CLAMP, RND); break; } else return hipErrorInvalidValue;  \
        case PM_RNE:         if constexpr (AMODE == 1) { LBA_LAUNCH(PM_RNE, RND); break; } else return hipErrorInvalidValue;                  \
        default:             if constexpr (AMODE == 1) { LBA_LAUNCH(PM_RNE_CLAMP, RND); break; } else return hipErrorInvalidValue;            \
    }
    if (pl.round == LBA_ROUND_FLOOR) {
        LBA_LAUNCH_ROUNDING(LBA_ROUND_FLOOR)
    } else if (pl.kp.sh_a == 16 && AMODE != 1) {             // M = 7: rounding by the bfloat16 conversion
        LBA_LAUNCH_ROUNDING(RND_RNE_BF16)
    } else {
        LBA_LAUNCH_ROUNDING(LBA_ROUND_RNE)
    }
#undef LBA_LAUNCH_ROUNDING
#undef LBA_LAUNCH
    return hipGetLastError();
}

template <int TM, int TN, int AMODE>
static hipError_t launch_fast_orders(const Plan& pl, hipStream_t st) {
    return pl.order == LBA_ORDER_CHUNK16 ? launch_fast<TM, TN, LBA_ORDER_CHUNK16, AMODE>(pl, st)
                                         : launch_fast<TM, TN, LBA_ORDER_SEQ, AMODE>(pl, st);
}

// lba_fast_mixed_kernel: plans with a mixed grid (64 x 64 workgroups, then 48 x 64 ones, then 32 x 32 ones)
template <int ORDER, int AMODE>
static hipError_t launch_mixed_order(const Plan& pl, hipStream_t st) {
    const dim3 grid(pl.grid_x, 1, 1), block(256);
    const KParams& kp = pl.kp;
#define LBA_MIX(PM, RND)                                                                                              \
    do {                                                                                                              \
        if constexpr (AMODE == 2) hipLaunchKernelGGL((lba_fast_conv_mixed_kernel<LBA_FAST_BK, PM, RND, ORDER>), grid, block, 0, st, kp); \
        else hipLaunchKernelGGL((lba_fast_mixed_kernel<LBA_FAST_BK, PM, RND, ORDER>), grid, block, 0, st, kp);         \
    } while (0)
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

template <int AMODE>
static hipError_t launch_mixed(const Plan& pl, hipStream_t st) {
    return pl.order == LBA_ORDER_CHUNK16 ? launch_mixed_order<LBA_ORDER_CHUNK16, AMODE>(pl, st)
                                         : launch_mixed_order<LBA_ORDER_SEQ, AMODE>(pl, st);
}

}  // namespace lba
#endif
