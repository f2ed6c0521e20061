// lba_bwd_rne.hip -- instantiations of lba_fast_bwd_kernel for nearest-even rounding of the accumulator.
#include "lba_launch_bwd.h"

namespace lba {
hipError_t launch_fast_bwd_rne(const Plan& pl, hipStream_t st) {
    if (pl.round != LBA_ROUND_RNE || pl.amode) return hipErrorInvalidValue;
    return launch_fast_bwd_rounding<LBA_ROUND_RNE>(pl, st);
}
}  // namespace lba
