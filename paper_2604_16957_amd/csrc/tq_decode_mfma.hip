// Matrix-core (MFMA) fused decode kernel: placeholder until the kernel lands.
#include "tq_internal.h"

namespace tq {

bool mfma_supported(int, int) { return false; }

hipError_t launch_partial_mfma(const DecodeParams&, int, int, hipStream_t) { return hipErrorNotSupported; }

}  // namespace tq
