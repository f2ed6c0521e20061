// lba_fast_44.hip -- instantiations of lba_fast_kernel for the 4 x 4 lane block.
#include "lba_launch_fast.h"

namespace lba {
hipError_t launch_fast_44(const Plan& pl, hipStream_t st) { return launch_fast_orders<4, 4, 0>(pl, st); }
}  // namespace lba
