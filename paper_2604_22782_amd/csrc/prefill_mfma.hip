#include "skv_internal.h"
namespace skv {
bool prefill_mfma_supported(int, int, int) { return false; }
hipError_t launch_prefill_mfma(const AttnArgs &, int, int, int, hipStream_t) { return hipErrorNotSupported; }
} // namespace skv
