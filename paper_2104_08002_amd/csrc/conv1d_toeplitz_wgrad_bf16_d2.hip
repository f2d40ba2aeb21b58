// Backward-weight, bfloat16, dilation 2: the register-ring kernels of this dilation (all shapes).
#include "conv1d_toeplitz_wgrad_bf16.h"

namespace conv1d {
namespace tz {

hipError_t launch_d2(const TzPlan& pl, hipStream_t st) { return launch_dilation<2>(pl, st); }

}  // namespace tz
}  // namespace conv1d
