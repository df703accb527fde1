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
  int32_t* counters;       // [B*Hkv*head_groups] zero between calls
  int n_split;
  int n_slots;             // partial slots per (b, head): n_split, plus one for the fp16 tail
  dq_tail tail;            // k_tail == nullptr: no tail
  int nw;                  // waves per workgroup of the matrix-core kernel (4 or 8)
  int head_groups;         // matrix-core kernel: workgroups per (sequence, kv head, split) ...
  int heads_per_group;     // ... each with this many query heads (1, 2 or 4; the last one what is left)
  int pair_heads;          // matrix-core kernel: 1 = two kv heads of 64 channels per workgroup (one query head each)
  int unit_map;            // which (sequence, kv head) a workgroup row takes: 0 = its own index, see unit_of_row()
  int rows_on_x;           // 0: grid (splits, rows); 1: grid (rows, splits), for more rows than a grid's y extent takes
  hipEvent_t ev_start;     // optional: recorded around the main kernel
  hipEvent_t ev_stop;
#ifdef DQ_TIMELINE
  // Instrumented build only (-DDQ_TIMELINE, see timeline.py): every wave of the matrix-core kernel
  // leaves kTimelineSlots time stamps of the 100 MHz real-time counter here, or nothing if null.
  unsigned long long* timeline;
#endif
};

#ifdef DQ_TIMELINE
// slot 0: wave entry; 1: lengths known, first tile's arithmetic starts; 2 + k: the wave's k-th tile
// starts (k < 16, later tiles overwrite the last of them); 18: its last tile is done; 19: exit (merge and
// output done); 20: not a time, the number of waves per workgroup
constexpr int kTimelineSlots = 21;
extern unsigned long long* g_timeline;   // set by dq_debug_timeline(), read by the decode entry points
#endif

// Which (sequence, kv head) unit the workgroups with blockIdx.y == row work on.  Workgroups go to
// the XCDs round-robin, so with the plain mapping an XCD only ever sees the units of one residue
// class mod 8, whose data sit at a fixed offset pattern in memory; the other mappings (bijections on
// [0, units) whenever units is a multiple of 8) give it a different class, all of them, or a
// contiguous range of units.  Measured on the 256-unit benchmark shape (us per step): 0: 27.0,
// 2: 25.9, 3: 25.7, 4: 26.5, 5: 25.7.
__host__ __device__ inline int unit_of_row(int row, int units, int unit_map) {
  if (unit_map == 0 || (units & 7)) return row;
  const int j = row >> 3, k = row & 7;
  if (unit_map == 1) return 8 * j + ((5 * k) & 7);   // another class per XCD
  if (unit_map == 3) return 8 * j + ((k + 3 * j) & 7);   // every class on every XCD (the default where it is used)
  if (unit_map == 4 && (units & (units - 1)) == 0) return (row * 37) & (units - 1);   // scattered
  if (unit_map == 5) return k * (units >> 3) + j;    // a contiguous range of units per XCD
  return 8 * j + ((k + j) & 7);                        // every class on every XCD, neighbours shifted by one
}

// Workspace carve-up shared by the host entry points.
inline size_t decode_counter_bytes(int batch, int q_heads) {   // one per (sequence, kv head, head group) at most
  return align_up((size_t)batch * q_heads * sizeof(int32_t), 256);
}
inline size_t decode_partial_bytes(const dq_format* f, int batch, int q_heads) {
  return (size_t)batch * q_heads * (kMaxSplits + 1) * (f->head_dim + 2) * sizeof(float);
}

int32_t launch_decode_generic(const DecodeArgs& a, hipStream_t st);
int32_t launch_tail_partial(const DecodeArgs& a, float m_unit, hipStream_t st);
int32_t launch_decode_mfma(const DecodeArgs& a, hipStream_t st);
bool mfma_supported(const dq_format* f, int q_heads, int kv_heads);
bool mfma_pair_heads(const dq_format* f, int q_heads, int kv_heads);
int mfma_head_groups(const dq_format* f, int q_heads, int kv_heads, int* heads_per_group);
int choose_splits(const dq_format* f, int batch, int q_heads, int kv_heads, int max_seq_len, bool mfma,
                  uint32_t flags, int* nw_out);

}  // namespace dq
