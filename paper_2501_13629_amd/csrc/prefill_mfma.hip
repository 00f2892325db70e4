// Causal prefill on the matrix cores (placeholder until the kernel lands: nothing is supported,
// so the boundary takes the portable kernel).
#include "kernels.h"

namespace diffqkv {

bool prefill_mfma_supported(const PrefillParams&, int) { return false; }
hipError_t launch_prefill_mfma(const PrefillParams&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace diffqkv
