// Host side of the matrix-core decode path: which formats it takes, and the launch.  The kernel
// template lives in dq_decode_mfma_kernel.h; its instantiations are spread over one source file per
// code width so that they compile in parallel.
#include "dq_decode.h"

namespace dq {

bool mfma_supported(const dq_format* f, int q_heads, int kv_heads) {
  if (!format_ok(f) || kv_heads <= 0 || q_heads % kv_heads) return false;
  if (f->head_dim != 128 || f->j1 != 16 || f->j2 != 8) return false;
  const int rep = q_heads / kv_heads;
  if (f->bits != 8 && f->bits != 4 && f->bits != 2) return false;
  // a head takes four B columns per step group of the sixteen
  if (f->group == 128) return rep == 1 || rep == 2 || rep == 4;
  if (f->group == 64) return rep == 1 || rep == 2;
  return false;
}

// defined in dq_decode_mfma_b8.hip, _b4.hip, _b2.hip
int32_t launch_decode_mfma_b8(const DecodeArgs& a, hipStream_t st);
int32_t launch_decode_mfma_b4(const DecodeArgs& a, hipStream_t st);
int32_t launch_decode_mfma_b2(const DecodeArgs& a, hipStream_t st);

int32_t launch_decode_mfma(const DecodeArgs& a, hipStream_t st) {
  const int32_t rc = (a.fmt.bits == 8) ? launch_decode_mfma_b8(a, st)
                     : (a.fmt.bits == 4) ? launch_decode_mfma_b4(a, st) : launch_decode_mfma_b2(a, st);
  if (rc != DQ_OK) return rc;
  DQ_HIP_CHECK(hipGetLastError());
  return DQ_OK;
}

}  // namespace dq
