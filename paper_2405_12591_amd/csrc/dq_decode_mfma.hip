// Host side of the matrix-core decode path: which formats it takes, and the launch.  The kernel
// template lives in dq_decode_mfma_kernel.h; its instantiations are spread over one source file per
// code width so that they compile in parallel.
#include "dq_decode.h"

namespace dq {

// Query heads per kv head that one workgroup takes: four B columns per head and step group of the
// sixteen, so at most 4 (one step group) or 2 (two); the kernel is built for 1, 2 and 4.  More heads
// are served in groups of that many, the last group taking what is left (7 = 4 + 3); a number that
// is not a power of two takes the next size up (3 heads run in a workgroup built for 4).
static int heads_per_workgroup(const dq_format* f, int rep) {
  const int most = (f->group == 128) ? 4 : 2;
  int r = 1;
  while (r < rep && r < most) r <<= 1;
  return ((rep + r - 1) / r <= kMaxHeadGroups) ? r : 0;
}

// Heads of 64 channels are worked in pairs of neighbouring kv heads (as one head of 128 channels and
// two step groups): j1 = j2 = 8, one step per row, one query head per kv head, an even number of
// heads, two local tensors.
bool mfma_pair_heads(const dq_format* f, int q_heads, int kv_heads) {
  if (!format_ok(f) || kv_heads <= 0 || q_heads != kv_heads || (kv_heads & 1)) return false;
  return f->head_dim == 64 && f->j1 == 8 && f->j2 == 8 && f->group == 64 && f->i3 == 1 && f->i1 == 1;
}

bool mfma_supported(const dq_format* f, int q_heads, int kv_heads) {
  if (!format_ok(f) || kv_heads <= 0 || q_heads <= 0 || q_heads % kv_heads) return false;
  if (f->i1 != 1) return false;   // a token factor on the small tensor: the plain kernel's
  if (mfma_pair_heads(f, q_heads, kv_heads)) return true;
  if (f->head_dim != 128 || f->j1 != 16 || f->j2 != 8) return false;
  if (f->bits != 8 && f->bits != 4 && f->bits != 2) return false;
  if (f->group != 128 && f->group != 64) return false;
  return heads_per_workgroup(f, q_heads / kv_heads) > 0;
}

int mfma_head_groups(const dq_format* f, int q_heads, int kv_heads, int* heads_per_group) {
  if (mfma_pair_heads(f, q_heads, kv_heads)) {
    if (heads_per_group) *heads_per_group = 1;
    return 1;
  }
  const int rep = q_heads / kv_heads;
  const int r = heads_per_workgroup(f, rep);
  if (heads_per_group) *heads_per_group = r;
  return (rep + r - 1) / r;
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
