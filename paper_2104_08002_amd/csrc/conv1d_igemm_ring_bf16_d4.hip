// Forward / backward-data, bfloat16, many channels, dilation 4: the resident-weight kernels of this dilation.
#include "conv1d_igemm_ring_bf16.h"

namespace conv1d {
namespace rg {

#ifdef CONV1D_DEV_FEW_KERNELS
hipError_t launch_d4(const RgPlan&, hipStream_t) { return hipErrorInvalidValue; }
#else
hipError_t launch_d4(const RgPlan& pl, hipStream_t st) { return rg_launch_d<4>(pl, st); }
#endif

}  // namespace rg
}  // namespace conv1d
