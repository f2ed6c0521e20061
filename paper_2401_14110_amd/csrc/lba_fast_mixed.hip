// lba_fast_mixed.hip -- instantiations of lba_fast_mixed_kernel for row-major operands (64 x 64 workgroups, then
// 48 x 64 ones, then 32 x 32 ones on the last rows of the launch).
#include "lba_launch_fast.h"

namespace lba {
hipError_t launch_fast_mixed(const Plan& pl, hipStream_t st) { return launch_mixed<0>(pl, st); }
}  // namespace lba
