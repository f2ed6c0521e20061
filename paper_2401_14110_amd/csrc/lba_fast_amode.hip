// lba_fast_amode.hip -- instantiations of lba_fast_kernel for the 4 x 4 lane block reading im2col rows / other operand formats.
#include "lba_launch_fast.h"

namespace lba {
hipError_t launch_fast_amode(const Plan& pl, hipStream_t st) { return launch_fast_orders<4, 4, 1>(pl, st); }
}  // namespace lba
