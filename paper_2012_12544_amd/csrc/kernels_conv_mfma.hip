// placeholder until the MFMA kernels land
#include "kernels.h"
namespace bapipe {
bool conv_gather_mfma_supported(const GatherConv &) { return false; }
hipError_t conv_gather_mfma(const void *, const void *, const float *, void *, int, GradEpi, const GatherConv &, hipStream_t) { return hipErrorNotSupported; }
bool conv_wgrad_mfma_supported(const ConvShape &) { return false; }
size_t conv_wgrad_mfma_workspace(const ConvShape &) { return 0; }
hipError_t conv_wgrad_mfma(const void *, const void *, float *, void *, const ConvShape &, hipStream_t) { return hipErrorNotSupported; }
}
