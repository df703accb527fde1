// Instantiations of the matrix-core decode kernel for 4-bit codes.
#include "dq_decode_mfma_kernel.h"

namespace dq {

int32_t launch_decode_mfma_b4(const DecodeArgs& a, hipStream_t st) { return launch_bits<4>(a, st); }

}  // namespace dq
