#include "sa_internal.h"
namespace sa {
bool bwd_mfma_supported(const StepArgs&, int) { return false; }
hipError_t launch_bwd_mfma(const StepArgs&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace sa
