// Instantiations of the matrix-core decode kernel for 8-bit codes.
#include "dq_decode_mfma_kernel.h"

namespace dq {

int32_t launch_decode_mfma_b8(const DecodeArgs& a, hipStream_t st) { return launch_bits<8>(a, st); }

}  // namespace dq
