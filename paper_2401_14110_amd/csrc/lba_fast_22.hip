// lba_fast_22.hip -- instantiations of lba_fast_kernel for the 2 x 2 lane block.
#include "lba_launch_fast.h"

namespace lba {
hipError_t launch_fast_22(const Plan& pl, hipStream_t st) { return launch_fast_orders<2, 2, 0>(pl, st); }
}  // namespace lba
