// placeholder until the MFMA append/prefill kernel lands
#include "kernels.h"
namespace fi355 {
hipError_t launch_append(const RunParams&, bool, hipStream_t) { return hipErrorNotSupported; }
}  // namespace fi355
