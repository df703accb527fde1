// The cache policy of Section 3.2 (arXiv 2405.12591) on the device: newly generated key/value rows
// are buffered in fp16, and a sequence's buffer is compressed into its next block slot as soon as
// it holds a block's worth of rows.  Every decision (where a row goes, whether a tail is full,
// which slot it is compressed into, how the lengths move) is taken by kernels from device-side
// lengths, so the host reads nothing back and any step can be captured in a graph.
#include "dq_common.h"

namespace dq {

// Append area behind the compression workspace: four int32 arrays of one entry per sequence.
struct AppendArea {
  int32_t* tickets;   // zero between calls
  int32_t* blk_idx;   // slot the tail is compressed into, or -1
  int32_t* take;      // rows of this call that went to the tail before it was compressed
  int32_t* rest;      // rows of this call that go to the emptied tail afterwards
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kAppendThreads = 256;

// One workgroup per (sequence, kv head, chunk of rows): copies its rows behind the tail's current
// end.  The last workgroup of a sequence to finish (a ticket per sequence) then moves the
// sequence's lengths and leaves the plan for the kernels that follow.  All workgroups of a sequence
// read its old tail length before they take their ticket, and only the holder of the last ticket
// writes the new one.
template <int D>
__global__ __launch_bounds__(kAppendThreads) void append_rows_kernel(
    dq_format fmt, int batch, int kv_heads, int block_capacity, uint16_t* __restrict__ k_tail,
    uint16_t* __restrict__ v_tail, int32_t* __restrict__ tail_lens, int32_t* __restrict__ seq_lens,
    const uint16_t* __restrict__ k_rows, const uint16_t* __restrict__ v_rows, int n_rows,
    const int32_t* __restrict__ counts, AppendArea area, int32_t* __restrict__ status, int chunks,
    int may_compress) {
  constexpr int LPR = D / 8;                      // lanes per row, 16 bytes each
  constexpr int RPB = kAppendThreads / LPR;       // rows per workgroup
  const int chunk = blockIdx.x % chunks;
  const int bh = blockIdx.x / chunks;
  const int b = bh / kv_heads;
  const int tb = fmt.block_tokens;
  const int tl = min(max(tail_lens[b], 0), tb);
  const int c = counts ? min(max(counts[b], 0), n_rows) : n_rows;
  const int take = min(c, tb - tl);
  const int r = chunk * RPB + (int)threadIdx.x / LPR, l = threadIdx.x % LPR;
  if (r < take) {
    const long src = ((long)bh * n_rows + r) * D + 8 * l;
    const long dst = ((long)bh * tb + tl + r) * D + 8 * l;
    *reinterpret_cast<u32x4*>(k_tail + dst) = *reinterpret_cast<const u32x4*>(k_rows + src);
    *reinterpret_cast<u32x4*>(v_tail + dst) = *reinterpret_cast<const u32x4*>(v_rows + src);
  }
  __syncthreads();
  if (threadIdx.x != 0) return;
  const int ticket = __hip_atomic_fetch_add(area.tickets + b, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (ticket != kv_heads * chunks - 1) return;
  __hip_atomic_store(area.tickets + b, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // clean for the next call
  int blk = -1, rest = 0, new_tl = tl + take;
  if (new_tl == tb) {                             // the tail holds a whole block: compress it
    const int slot = max(seq_lens[b], 0) / tb;
    if (!may_compress) {
      atomicOr(status + 3, 2);                    // the caller said no tail would fill: it stays full, further rows are dropped
    } else if (slot < block_capacity) {
      blk = slot;
      seq_lens[b] = (slot + 1) * tb;
      rest = c - take;
      new_tl = rest;                              // what is left of this call's rows restarts the tail
    } else {
      atomicOr(status + 3, 1);                    // no free slot: the tail stays full, further rows are dropped
    }
  }
  area.blk_idx[b] = blk;
  area.take[b] = take;
  area.rest[b] = rest;
  tail_lens[b] = new_tl;
}

// After the compression: the rows of this call that did not fit before the tail was compressed go
// to the start of the emptied tail.
template <int D>
__global__ __launch_bounds__(kAppendThreads) void append_rest_kernel(
    dq_format fmt, int kv_heads, uint16_t* __restrict__ k_tail, uint16_t* __restrict__ v_tail,
    const uint16_t* __restrict__ k_rows, const uint16_t* __restrict__ v_rows, int n_rows, AppendArea area,
    int chunks) {
  constexpr int LPR = D / 8;
  constexpr int RPB = kAppendThreads / LPR;
  const int chunk = blockIdx.x % chunks;
  const int bh = blockIdx.x / chunks;
  const int b = bh / kv_heads;
  const int rest = area.rest[b];
  const int r = chunk * RPB + (int)threadIdx.x / LPR, l = threadIdx.x % LPR;
  if (r >= rest) return;
  const long src = ((long)bh * n_rows + area.take[b] + r) * D + 8 * l;
  const long dst = ((long)bh * fmt.block_tokens + r) * D + 8 * l;
  *reinterpret_cast<u32x4*>(k_tail + dst) = *reinterpret_cast<const u32x4*>(k_rows + src);
  *reinterpret_cast<u32x4*>(v_tail + dst) = *reinterpret_cast<const u32x4*>(v_rows + src);
}

static size_t append_area_bytes(int batch) { return align_up((size_t)batch * 4 * sizeof(int32_t), 256); }

}  // namespace dq

using namespace dq;

extern "C" size_t dq_cache_append_workspace_bytes(const dq_format* fmt, int32_t batch, int32_t kv_heads) {
  const size_t c = dq_compress_workspace_bytes(fmt, batch, kv_heads);
  if (c == 0 || fmt->block_tokens > kMaxTailRows) return 0;
  return align_up(c, 256) + append_area_bytes(batch);
}

extern "C" int32_t dq_cache_append(const dq_format* fmt, dq_cache* cache, const dq_kv_state* state,
                                   const uint16_t* k_rows, const uint16_t* v_rows, int32_t n_rows,
                                   const int32_t* counts, void* workspace, size_t workspace_bytes,
                                   uint32_t flags, void* hip_stream) {
  if (!format_ok(fmt) || !cache || !state || !k_rows || !v_rows || !workspace) return DQ_EINVAL;
  if (!state->k_tail || !state->v_tail || !state->tail_lens || !state->seq_lens) return DQ_EINVAL;
  if (cache->batch <= 0 || cache->kv_heads <= 0 || cache->block_capacity <= 0) return DQ_EINVAL;
  if (fmt->block_tokens > kMaxTailRows) return DQ_EINVAL;   // the tail must fit what a decode call takes
  if (n_rows < 1 || n_rows > fmt->block_tokens) return DQ_EINVAL;
  if (flags & ~DQ_APPEND_NO_COMPRESS) return DQ_EINVAL;
  if (((uintptr_t)k_rows | (uintptr_t)v_rows | (uintptr_t)state->k_tail | (uintptr_t)state->v_tail) & 15) return DQ_EINVAL;
  const size_t need = dq_cache_append_workspace_bytes(fmt, cache->batch, cache->kv_heads);
  if (need == 0) return DQ_EINVAL;
  if (workspace_bytes < need) return DQ_ENOSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const int B = cache->batch, H = cache->kv_heads;
  const size_t cbytes = align_up(dq_compress_workspace_bytes(fmt, B, H), 256);
  int32_t* base = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(workspace) + cbytes);
  const AppendArea area = {base, base + B, base + 2 * B, base + 3 * B};
  int32_t* status = reinterpret_cast<int32_t*>(workspace);
  const int rpb = kAppendThreads / (fmt->head_dim / 8);
  const int chunks = (n_rows + rpb - 1) / rpb;
  const dim3 grid((unsigned)(B * H * chunks));
  if (fmt->head_dim == 128)
    hipLaunchKernelGGL(append_rows_kernel<128>, grid, dim3(kAppendThreads), 0, st, *fmt, B, H, cache->block_capacity,
                       state->k_tail, state->v_tail, state->tail_lens, state->seq_lens, k_rows, v_rows, n_rows,
                       counts, area, status, chunks, (flags & DQ_APPEND_NO_COMPRESS) ? 0 : 1);
  else
    hipLaunchKernelGGL(append_rows_kernel<64>, grid, dim3(kAppendThreads), 0, st, *fmt, B, H, cache->block_capacity,
                       state->k_tail, state->v_tail, state->tail_lens, state->seq_lens, k_rows, v_rows, n_rows,
                       counts, area, status, chunks, (flags & DQ_APPEND_NO_COMPRESS) ? 0 : 1);
  DQ_HIP_CHECK(hipGetLastError());
  if (flags & DQ_APPEND_NO_COMPRESS) return DQ_OK;
  // every sequence whose tail filled (a slot index in the plan; -1 skips the others) is compressed
  // from its tail buffer; the fp32 large tensors are not kept
  const int32_t rc = dq_compress_kv_ex(fmt, cache, state->k_tail, state->v_tail, fmt->block_tokens, area.blk_idx,
                                       nullptr, workspace, cbytes, DQ_COMPRESS_NO_LARGE, hip_stream);
  if (rc != DQ_OK) return rc;
  if (n_rows > 1) {
    if (fmt->head_dim == 128)
      hipLaunchKernelGGL(append_rest_kernel<128>, grid, dim3(kAppendThreads), 0, st, *fmt, H, state->k_tail,
                         state->v_tail, k_rows, v_rows, n_rows, area, chunks);
    else
      hipLaunchKernelGGL(append_rest_kernel<64>, grid, dim3(kAppendThreads), 0, st, *fmt, H, state->k_tail,
                         state->v_tail, k_rows, v_rows, n_rows, area, chunks);
    DQ_HIP_CHECK(hipGetLastError());
  }
  return DQ_OK;
}
