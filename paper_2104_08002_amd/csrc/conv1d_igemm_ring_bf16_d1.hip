// Forward / backward-data, bfloat16, many channels, dilation 1: the resident-weight kernels of this dilation.
#include "conv1d_igemm_ring_bf16.h"

namespace conv1d {
namespace rg {

hipError_t launch_d1(const RgPlan& pl, hipStream_t st) { return rg_launch_d<1>(pl, st); }

}  // namespace rg
}  // namespace conv1d
