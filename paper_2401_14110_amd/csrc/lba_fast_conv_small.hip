// lba_fast_conv_small.hip -- the 2 x 4 and 2 x 2 lane blocks of the forward kernel reading im2col rows (AMODE 2).
#include "lba_launch_fast.h"

namespace lba {
hipError_t launch_fast_conv_small(const Plan& pl, hipStream_t st) {
    if (pl.tm == 2 && pl.tn == 2) return launch_fast_orders<2, 2, 2>(pl, st);
    if (pl.tm == 2 && pl.tn == 4) return launch_fast_orders<2, 4, 2>(pl, st);
    return hipErrorInvalidValue;
}
}  // namespace lba
