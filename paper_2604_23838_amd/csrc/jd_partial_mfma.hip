#include "jd_internal.h"
namespace jd {
int mfma_waves_per_cu() { return 4; }
int mfma_waves_per_block() { return 4; }
hipError_t launch_partial_mfma(const Params&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace jd
