// Matrix-core decode kernel (placeholder until the MFMA path lands).
#include "kvq_internal.h"
namespace kvq {
hipError_t launch_decode_mfma(const DecodeArgs &, hipStream_t) { return hipErrorNotSupported; }
}  // namespace kvq
