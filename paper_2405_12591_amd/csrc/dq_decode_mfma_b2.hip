// Instantiations of the matrix-core decode kernel for 2-bit codes.
#include "dq_decode_mfma_kernel.h"

namespace dq {

int32_t launch_decode_mfma_b2(const DecodeArgs& a, hipStream_t st) { return launch_bits<2>(a, st); }

}  // namespace dq
