#include "sa_internal.h"
namespace sa {
bool fwd_mfma_supported(const StepArgs&, int) { return false; }
hipError_t launch_fwd_mfma(const StepArgs&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace sa
