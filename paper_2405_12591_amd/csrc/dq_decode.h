// Internal launch interfaces of the decode kernels.
#pragma once
#include "dq_common.h"

namespace dq {

struct DecodeArgs {
  dq_format fmt;
  dq_cache cache;
  const uint16_t* q;       // [B, Hq, d] fp16 bits
  int q_heads;
  const int32_t* seq_lens; // [B]
  int max_seq_len;
  float scale;             // softmax scale (already defaulted)
  uint16_t* out;           // [B, Hq, d] fp16 bits
  float* out_f32;          // optional
  float* partials;         // [B*Hq, n_split, d + 2]
  int32_t* counters;       // [B*Hkv] zero between calls
  int n_split;
  int n_slots;             // partial slots per (b, head): n_split, plus one for the fp16 tail
  dq_tail tail;            // k_tail == nullptr: no tail
  int nw;                  // waves per workgroup of the matrix-core kernel (4 or 8)
  hipEvent_t ev_start;     // optional: recorded around the main kernel
  hipEvent_t ev_stop;
};

// Workspace carve-up shared by the host entry points.
inline size_t decode_counter_bytes(int batch, int kv_heads) {
  return align_up((size_t)batch * kv_heads * sizeof(int32_t), 256);
}
inline size_t decode_partial_bytes(const dq_format* f, int batch, int q_heads) {
  return (size_t)batch * q_heads * (kMaxSplits + 1) * (f->head_dim + 2) * sizeof(float);
}

int32_t launch_decode_generic(const DecodeArgs& a, hipStream_t st);
int32_t launch_tail_partial(const DecodeArgs& a, float m_unit, hipStream_t st);
int32_t launch_decode_mfma(const DecodeArgs& a, hipStream_t st);
bool mfma_supported(const dq_format* f, int q_heads, int kv_heads);
int choose_splits(const dq_format* f, int batch, int q_heads, int kv_heads, int max_seq_len, bool mfma,
                  int* nw_out);

}  // namespace dq
