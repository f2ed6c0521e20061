// lba_bwd.hip -- instantiations of lba_fast_bwd_kernel (the recompute call in the scaled domain) for floor
// rounding; the nearest-even ones are in lba_bwd_rne.hip.
#include "lba_launch_bwd.h"

namespace lba {
hipError_t launch_fast_bwd(const Plan& pl, hipStream_t st) {
    if (pl.amode == 2) return launch_fast_bwd_conv(pl, st);
    if (pl.amode == 1 && pl.mix_tail > 0) return launch_fast_bwd_in_mixed(pl, st);
    if (pl.round != LBA_ROUND_FLOOR) return launch_fast_bwd_rne(pl, st);
    return launch_fast_bwd_rounding<LBA_ROUND_FLOOR>(pl, st);
}
}  // namespace lba
