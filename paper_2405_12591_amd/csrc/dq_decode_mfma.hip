// Matrix-core decode kernel (placeholder until the fast path lands).
#include "dq_decode.h"

namespace dq {
bool mfma_supported(const dq_format*, int, int) { return false; }
int32_t launch_decode_mfma(const DecodeArgs&, hipStream_t) { return DQ_EINVAL; }
}  // namespace dq
