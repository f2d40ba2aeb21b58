// Backward-weight, bfloat16, dilation 16: the register-ring kernels of this dilation (all shapes).
#include "conv1d_toeplitz_wgrad_bf16.h"

namespace conv1d {
namespace tz {

#ifdef CONV1D_DEV_FEW_KERNELS
hipError_t launch_d16(const TzPlan&, hipStream_t) { return hipErrorInvalidValue; }
#else
hipError_t launch_d16(const TzPlan& pl, hipStream_t st) { return launch_dilation<16>(pl, st); }
#endif

}  // namespace tz
}  // namespace conv1d
