// lba_launch.h -- launchers of the kernel instantiations.  The instantiations are spread over several
// translation units (lba_fast_*.hip, lba_bwd.hip, lba_gen.hip) so that they compile in parallel; each
// defines the launchers declared here for its group of template arguments.
#ifndef LBA_LAUNCH_H_
#define LBA_LAUNCH_H_

#include <hip/hip_runtime.h>

#include "lba_internal.h"

namespace lba {

// forward, scaled-domain kernel; lane block tm x tn of the plan (amode plans: 4 x 4)
hipError_t launch_fast_44(const Plan& pl, hipStream_t st);
hipError_t launch_fast_24(const Plan& pl, hipStream_t st);
hipError_t launch_fast_22(const Plan& pl, hipStream_t st);
hipError_t launch_fast_amode(const Plan& pl, hipStream_t st);
hipError_t launch_fast_mixed(const Plan& pl, hipStream_t st);   // plans with mix_tail > 0
hipError_t launch_fast_conv(const Plan& pl, hipStream_t st);    // plans with amode == 2 (any lane block, mixed or not)
hipError_t launch_fast_in_mixed_seq(const Plan& pl, hipStream_t st);    // plans with amode == 1 and mix_tail > 0, by order
hipError_t launch_fast_in_mixed_chunk(const Plan& pl, hipStream_t st);
hipError_t launch_fast_odd(const Plan& pl, hipStream_t st);     // plans with rne_odd
// forward, chunked order, several chunks of an output side by side (plans with kpar > 0)
hipError_t launch_kpar(const Plan& pl, hipStream_t st);
// recompute call, scaled-domain kernel (launch_fast_bwd hands nearest-even plans to launch_fast_bwd_rne)
hipError_t launch_fast_bwd(const Plan& pl, hipStream_t st);
hipError_t launch_fast_bwd_rne(const Plan& pl, hipStream_t st);
hipError_t launch_fast_bwd_conv(const Plan& pl, hipStream_t st);   // plans with amode == 2
hipError_t launch_fast_bwd_in_mixed(const Plan& pl, hipStream_t st);   // plans with amode == 1 on a mixed grid
// the DIFF plane, scaled-domain kernel (plans with events == 2)
hipError_t launch_fast_diff(const Plan& pl, hipStream_t st);
// general kernel (forward and recompute)
hipError_t launch_gen(const Plan& pl, hipStream_t st);

// Brick maps of an overflow plane (lba_grad.hip): two byte maps in a caller-given workspace, the dX side first, each
// padded to a multiple of 256 bytes.  All return LBA_OK or LBA_ERR_LAUNCH / LBA_ERR_SHAPE.
void brick_bytes(int64_t M, int64_t N, int64_t K, size_t* dx_bytes, size_t* dw_bytes);
int brick_maps_fill(void* workspace, int64_t M, int64_t N, int64_t K, bool dirty, hipStream_t st);   // all clean / all dirty
// zeroes the maps, then marks them in one pass over the plane (N % 4 == 0, plane 16-byte aligned); flip: 0 for a
// plane of overflow bits, all ones for a plane of coefficients
int brick_maps_scan(const uint32_t* plane, void* workspace, int64_t M, int64_t N, int64_t K, uint32_t flip, hipStream_t st);
void brick_map_params(void* workspace, int64_t M, int64_t N, int64_t K, KParams* kp);   // for a kernel that marks them itself

}  // namespace lba
#endif
