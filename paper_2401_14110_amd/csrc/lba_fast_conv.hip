// lba_fast_conv.hip -- forward kernels that read A as im2col rows of an NHWC tensor of E4M3 codes (AMODE 2):
// the mixed-grid kernel and the 4 x 4 lane block; the smaller lane blocks are in lba_fast_conv_small.hip.
#include "lba_launch_fast.h"

namespace lba {
hipError_t launch_fast_conv_small(const Plan& pl, hipStream_t st);

hipError_t launch_fast_conv(const Plan& pl, hipStream_t st) {
    if (pl.amode != 2 || pl.events || pl.kp.batch != 1) return hipErrorInvalidValue;
    if (pl.mix_tail > 0) return launch_mixed<2>(pl, st);
    if (pl.tm == 2) return launch_fast_conv_small(pl, st);
    return launch_fast_orders<4, 4, 2>(pl, st);
}
}  // namespace lba
