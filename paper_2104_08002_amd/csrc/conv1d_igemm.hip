#include "conv1d_internal.h"
namespace conv1d {
bool igemm_corr_supported(const CorrProblem&) { return false; }
hipError_t igemm_corr_launch(const CorrProblem&, hipStream_t) { return hipErrorInvalidValue; }
bool igemm_wgrad_supported(const WgradProblem&) { return false; }
size_t igemm_wgrad_workspace(const WgradProblem&) { return 0; }
hipError_t igemm_wgrad_launch(const WgradProblem&, hipStream_t) { return hipErrorInvalidValue; }
}  // namespace conv1d
