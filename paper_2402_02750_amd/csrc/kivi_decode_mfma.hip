// Decode attention, matrix-core family: placeholder until the MFMA kernels land.
#include "kivi_internal.h"

namespace kivi {

hipError_t launch_decode_mfma(const DecodeParams&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace kivi
