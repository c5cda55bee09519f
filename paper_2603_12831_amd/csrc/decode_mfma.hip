// Matrix-core decode attention (placeholder until the MFMA kernel lands).
#include "omni_internal.hpp"

namespace omni {
bool decode_mfma_supports(const DecodeParams&, bool) { return false; }
hipError_t launch_decode_mfma(const DecodeParams&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace omni
