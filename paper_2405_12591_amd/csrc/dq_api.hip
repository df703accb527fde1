// Host side of the C ABI: argument checks, workspace carve-up, kernel selection.
#include <atomic>
#include <mutex>

#include "dq_decode.h"

namespace dq {

static std::atomic<int> g_last_hip_error{0};
void set_last_hip_error(hipError_t e) { g_last_hip_error.store((int)e); }

// Launch shape of the matrix-core kernel: n splits of every (sequence, kv head) and nw waves per
// workgroup.  Measured on MI355X: a wave needs about eight 128-token tiles to amortise its start-up
// and its share of the merge (four when it serves four query heads: more arithmetic per tile to
// overlap); about 2048 resident waves (8 per CU) stream fastest when they can be had at that depth,
// 1024 (one 4-wave workgroup per CU) otherwise; every extra split costs a partial write, a ticket
// and a merge.  Small problems are bound by the fixed start-up and merge latencies: there one tile
// per wave is best as long as every workgroup finds a compute unit of its own.
static void choose_mfma_shape(int units, int max_tiles, int rep, int bits, int* n_out, int* nw_out) {
  auto tiles_per_wave = [&](int n, int nw) { return max_tiles / (n * nw); };
  const int deep = rep >= 4 ? 4 : 8;
  // A: deep and wide (8-bit codes: a wave's ring of chunks is twice as large and an 8-wave
  // workgroup would run out of registers)
  for (int nw = (bits == 8 ? 4 : 8); nw >= 4; nw -= 4) {
    const int cap = 256 * (8 / nw);            // workgroups resident on the chip
    for (int n = cap / units; n >= 1; --n) {
      if (n > kMaxSplits) continue;
      if (tiles_per_wave(n, nw) >= deep && (long)units * n * nw >= 1536) { *n_out = n; *nw_out = nw; return; }
    }
  }
  // B: deep, at least half the chip
  for (int n = 512 / units; n >= 1; --n) {
    if (n > kMaxSplits) continue;
    if (tiles_per_wave(n, 4) >= 8 && (long)units * n * 4 >= 512) { *n_out = n; *nw_out = 4; return; }
  }
  // C: small problem: one tile per wave while a workgroup per compute unit is enough, else two
  for (int n = (512 / units < kMaxSplits ? 512 / units : kMaxSplits); n >= 1; --n) {
    const int need = (units * n <= 256) ? 1 : 2;
    if (tiles_per_wave(n, 4) >= need) { *n_out = n; *nw_out = 4; return; }
  }
  *n_out = 1; *nw_out = 4;
}

int choose_splits(const dq_format* f, int batch, int q_heads, int kv_heads, int max_seq_len, bool mfma,
                  uint32_t flags, int* nw_out) {
  const int max_tiles = (max_seq_len + kTileTokens - 1) / kTileTokens;
  int n = 1, nw = 4;
  if (max_tiles > 0) {
    if (mfma) {
      int per_group = 1;
      const int hg = mfma_head_groups(f, q_heads, kv_heads, &per_group);   // each head group is a workgroup of its own
      if (mfma_pair_heads(f, q_heads, kv_heads))   // two kv heads, one query head each, per workgroup
        choose_mfma_shape(batch * kv_heads / 2, max_tiles, 2, f->bits, &n, &nw);
      else
        choose_mfma_shape(batch * kv_heads * hg, max_tiles, per_group, f->bits, &n, &nw);
    } else {
      const int units = batch * q_heads;
      n = (2048 + units - 1) / units;
      const int by_len = (max_tiles + 1) / 2;
      if (n > by_len) n = by_len;
    }
  }
  // the caller's overrides (validated by the entry point)
  if (const int v = (int)((flags >> 8) & 0x7Fu)) n = v;
  if (const int v = (int)((flags >> 16) & 0xFu)) nw = v;
  if (n < 1) n = 1;
  if (n > kMaxSplits) n = kMaxSplits;
  if (max_tiles > 0 && n > max_tiles) n = max_tiles;
  if (nw_out) *nw_out = nw;
  return n;
}

__global__ void fill_zero_kernel(uint4* p, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Each wave reads its own contiguous slice with sixteen 1 KB loads in flight: the access shape
// that gave the highest read rate of the shapes tried on this chip.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, size_t n16,
                                                          uint32_t* __restrict__ sink) {
  constexpr int INF = 16;
  const size_t waves = (size_t)gridDim.x * 4;
  const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  // slices are multiples of one load group (INF * 64 elements); what is left over after the
  // slices is dealt out in 64-element pieces
  const size_t group = (size_t)INF * 64;
  const size_t per_wave = (n16 / waves) / group * group;
  const size_t begin = wave * per_wave;
  const size_t end = begin + per_wave;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t i = begin + lane; i < end; i += group) {
    u32x4 v[INF];
#pragma unroll
    for (int k = 0; k < INF; ++k) v[k] = __builtin_nontemporal_load(src + i + k * 64);
#pragma unroll
    for (int k = 0; k < INF; ++k) acc ^= v[k];
  }
  for (size_t i = waves * per_wave + wave * 64 + lane; i < n16; i += waves * 64)
    acc ^= __builtin_nontemporal_load(src + i);
  // a data-dependent store that practically never happens keeps the loads alive
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) {
    sink[0] = acc.x; sink[1] = acc.y; sink[2] = acc.z; sink[3] = acc.w;
  }
}

}  // namespace dq

using namespace dq;

#ifdef DQ_TIMELINE
namespace dq { unsigned long long* g_timeline = nullptr; }
// Instrumented build only: the device buffer ([workgroups * waves, kTimelineSlots] u64, zero-filled by the
// caller) the matrix-core decode kernel's waves stamp their time line into; NULL switches it off.
extern "C" void dq_debug_timeline(void* buffer) { dq::g_timeline = reinterpret_cast<unsigned long long*>(buffer); }
extern "C" int32_t dq_debug_timeline_slots(void) { return dq::kTimelineSlots; }
#endif

extern "C" int32_t dq_version(void) { return 6; }

extern "C" const char* dq_status_string(int32_t status) {
  switch (status) {
    case DQ_OK: return "ok";
    case DQ_EINVAL: return "invalid argument or unsupported format";
    case DQ_ENOSPACE: return "workspace too small";
    case DQ_EHIP: return "HIP runtime error";
    case DQ_ELIMIT: return "sizes beyond the limit of the allocation-free entry point";
    default: return "unknown status";
  }
}

extern "C" int32_t dq_last_hip_error(void) { return g_last_hip_error.load(); }

extern "C" int32_t dq_decode_mfma_supported(const dq_format* fmt, int32_t q_heads, int32_t kv_heads) {
  return mfma_supported(fmt, q_heads, kv_heads) ? 1 : 0;
}

extern "C" size_t dq_decode_workspace_bytes(const dq_format* fmt, int32_t batch, int32_t q_heads,
                                            int32_t kv_heads, int32_t max_seq_len) {
  if (!format_ok(fmt) || batch <= 0 || q_heads <= 0 || kv_heads <= 0 || q_heads % kv_heads ||
      max_seq_len < 0)
    return 0;
  return (size_t)kWsHeaderBytes + decode_counter_bytes(batch, q_heads) +
         decode_partial_bytes(fmt, batch, q_heads);
}

extern "C" int32_t dq_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!workspace || workspace_bytes % 16 || ((uintptr_t)workspace & 15)) return DQ_EINVAL;
  if (workspace_bytes == 0) return DQ_OK;
  const size_t n16 = workspace_bytes / 16;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream,
                     reinterpret_cast<uint4*>(workspace), n16);
  DQ_HIP_CHECK(hipGetLastError());
  return DQ_OK;
}

static int32_t decode_impl(const dq_format* fmt, const dq_cache* cache, const uint16_t* q,
                           int32_t q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                           const dq_tail* tail, float softmax_scale, uint16_t* out, float* out_f32,
                           void* workspace, size_t workspace_bytes, uint32_t flags, void* hip_stream,
                           void* ev_kernel_start, void* ev_kernel_stop) {
  if (!format_ok(fmt) || !cache || !q || !seq_lens || !out || !workspace) return DQ_EINVAL;
  if (!cache->k_codes || !cache->k_scales || !cache->k_small || !cache->v_codes || !cache->v_scales ||
      !cache->v_small)
    return DQ_EINVAL;
  if (fmt->i3 != 1 && (!cache->k_small3 || !cache->v_small3)) return DQ_EINVAL;
  if (cache->batch <= 0 || cache->kv_heads <= 0 || cache->block_capacity <= 0) return DQ_EINVAL;
  if (q_heads <= 0 || q_heads % cache->kv_heads) return DQ_EINVAL;
  if ((long)cache->batch * q_heads > kMaxDecodeRows) return DQ_EINVAL;
  if (max_seq_len < 0 || (long)max_seq_len > (long)cache->block_capacity * fmt->block_tokens) return DQ_EINVAL;
  if ((flags & DQ_DECODE_FORCE_GENERIC) && (flags & DQ_DECODE_FORCE_MFMA)) return DQ_EINVAL;
  {
    const uint32_t splits = (flags >> 8) & 0x7Fu, waves = (flags >> 16) & 0xFu, umap = (flags >> 20) & 0xFu;
    if (flags & ~(3u | DQ_DECODE_SPLITS(0x7F) | DQ_DECODE_WAVES(0xF) | (0xFu << 20))) return DQ_EINVAL;
    if (splits > (uint32_t)kMaxSplits || (waves != 0 && waves != 4 && waves != 8) || umap > 6) return DQ_EINVAL;
  }
  const size_t need = dq_decode_workspace_bytes(fmt, cache->batch, q_heads, cache->kv_heads, max_seq_len);
  if (need == 0) return DQ_EINVAL;
  if (workspace_bytes < need) return DQ_ENOSPACE;
  if (tail && (!tail->k_tail || !tail->v_tail || !tail->tail_lens || tail->capacity < 1 || tail->capacity > kMaxTailRows))
    return DQ_EINVAL;
  const bool can_mfma = mfma_supported(fmt, q_heads, cache->kv_heads);
  if ((flags & DQ_DECODE_FORCE_MFMA) && !can_mfma) return DQ_EINVAL;
  const bool use_mfma = can_mfma && !(flags & DQ_DECODE_FORCE_GENERIC);

  DecodeArgs a;
  a.fmt = *fmt;
  a.cache = *cache;
  a.q = q;
  a.q_heads = q_heads;
  a.seq_lens = seq_lens;
  a.max_seq_len = max_seq_len;
  a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)fmt->head_dim);
  a.out = out;
  a.out_f32 = out_f32;
  char* ws = reinterpret_cast<char*>(workspace);
  a.counters = reinterpret_cast<int32_t*>(ws + kWsHeaderBytes);
  a.partials = reinterpret_cast<float*>(ws + kWsHeaderBytes + decode_counter_bytes(cache->batch, q_heads));
  a.heads_per_group = q_heads / cache->kv_heads;
  a.head_groups = use_mfma ? mfma_head_groups(fmt, q_heads, cache->kv_heads, &a.heads_per_group) : 1;
  a.n_split = choose_splits(fmt, cache->batch, q_heads, cache->kv_heads, max_seq_len, use_mfma, flags, &a.nw);
  // With one workgroup per compute unit and equal shares, a launch ends with its slowest XCD.
  // Dealing the units so that every XCD sees every residue class of them (mod 8) brings the XCDs
  // closer together: measured 4 - 5 % faster on the 256-unit benchmark shapes (4- and 8-bit), neutral
  // or within half a percent either way on the other workloads, where the plain order stays.
  a.pair_heads = (use_mfma && mfma_pair_heads(fmt, q_heads, cache->kv_heads)) ? 1 : 0;
  const int units = cache->batch * cache->kv_heads / (a.pair_heads ? 2 : 1);
  a.unit_map = (a.n_split == 1 && a.head_groups == 1 && units <= 256) ? 3 : 0;
  if (const uint32_t umap = (flags >> 20) & 0xFu) a.unit_map = (int)umap - 1;   // the caller's override
  a.rows_on_x = ((long)cache->batch * q_heads > kMaxGridY) ? 1 : 0;   // rows: at most batch * q_heads of them
  a.n_slots = a.n_split + (tail ? 1 : 0);
  if (tail) a.tail = *tail;
  else a.tail = dq_tail{nullptr, nullptr, nullptr, 0};
#ifdef DQ_TIMELINE
  a.timeline = g_timeline;
#endif
  a.ev_start = (hipEvent_t)ev_kernel_start;
  a.ev_stop = (hipEvent_t)ev_kernel_stop;
  hipStream_t st = (hipStream_t)hip_stream;
  return use_mfma ? launch_decode_mfma(a, st) : launch_decode_generic(a, st);
}

extern "C" int32_t dq_attn_decode_timed(const dq_format* fmt, const dq_cache* cache, const uint16_t* q,
                                        int32_t q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                                        float softmax_scale, uint16_t* out, float* out_f32, void* workspace,
                                        size_t workspace_bytes, uint32_t flags, void* hip_stream,
                                        void* ev_kernel_start, void* ev_kernel_stop) {
  return decode_impl(fmt, cache, q, q_heads, seq_lens, max_seq_len, nullptr, softmax_scale, out, out_f32,
                     workspace, workspace_bytes, flags, hip_stream, ev_kernel_start, ev_kernel_stop);
}

extern "C" int32_t dq_attn_decode_tail(const dq_format* fmt, const dq_cache* cache, const uint16_t* q,
                                       int32_t q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                                       const dq_tail* tail, float softmax_scale, uint16_t* out,
                                       float* out_f32, void* workspace, size_t workspace_bytes,
                                       uint32_t flags, void* hip_stream) {
  return decode_impl(fmt, cache, q, q_heads, seq_lens, max_seq_len, tail, softmax_scale, out, out_f32,
                     workspace, workspace_bytes, flags, hip_stream, nullptr, nullptr);
}

extern "C" int32_t dq_attn_decode(const dq_format* fmt, const dq_cache* cache, const uint16_t* q,
                                  int32_t q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                                  float softmax_scale, uint16_t* out, float* out_f32, void* workspace,
                                  size_t workspace_bytes, uint32_t flags, void* hip_stream) {
  return dq_attn_decode_timed(fmt, cache, q, q_heads, seq_lens, max_seq_len, softmax_scale, out, out_f32,
                              workspace, workspace_bytes, flags, hip_stream, nullptr, nullptr);
}

// ---- decode without a workspace argument: for callers that cannot allocate -------------------
// The split partials and tickets live in a file-scope device array.  Every GPU the library runs on
// holds its own copy at its own address, which is looked up once per device; host code uses that
// address only, never the array's name.
constexpr int kStaticMaxPairs = 512;   // (sequence, query head) pairs one call may hold
constexpr size_t kStaticScratchBytes =
    (size_t)kWsHeaderBytes + (size_t)kStaticMaxPairs * sizeof(int32_t) /* tickets, a multiple of 256 */ +
    (size_t)kStaticMaxPairs * (kMaxSplits + 1) * (128 + 2) * sizeof(float);
static_assert(((size_t)kStaticMaxPairs * sizeof(int32_t)) % 256 == 0, "ticket area is a multiple of 256 bytes");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];   // the array's device address, per device; null until looked up

// The current device's copy of the array; on its first use the ticket area is cleared on `st` (a
// small kernel, safe under stream capture).  The kernels leave the tickets at zero afterwards.
static int32_t static_scratch(hipStream_t st, void** out) {
  int dev = -1;
  DQ_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return DQ_EINVAL;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    DQ_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return DQ_EHIP;
    const size_t head = (size_t)kWsHeaderBytes + (size_t)kStaticMaxPairs * sizeof(int32_t);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(256), 0, st, reinterpret_cast<uint4*>(ptr), head / 16);
    DQ_HIP_CHECK(hipGetLastError());
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return DQ_OK;
}

extern "C" int32_t dq_attn_decode_static(const dq_format* fmt, const dq_cache* cache, const uint16_t* q,
                                         int32_t q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                                         const dq_tail* tail, float softmax_scale, uint16_t* out,
                                         float* out_f32, uint32_t flags, void* hip_stream) {
  if (!format_ok(fmt) || !cache || cache->batch <= 0 || q_heads <= 0) return DQ_EINVAL;
  if ((long)cache->batch * q_heads > kStaticMaxPairs) return DQ_ELIMIT;
  const size_t need = dq_decode_workspace_bytes(fmt, cache->batch, q_heads, cache->kv_heads, max_seq_len);
  if (need == 0) return DQ_EINVAL;
  if (need > kStaticScratchBytes) return DQ_ELIMIT;
  void* ptr = nullptr;
  const int32_t rc = static_scratch((hipStream_t)hip_stream, &ptr);
  if (rc != DQ_OK) return rc;
  return decode_impl(fmt, cache, q, q_heads, seq_lens, max_seq_len, tail, softmax_scale, out, out_f32, ptr,
                     kStaticScratchBytes, flags, hip_stream, nullptr, nullptr);
}

extern "C" int32_t dq_stream_read(const void* src, size_t bytes, uint32_t* sink, void* hip_stream) {
  if (!src || !sink || bytes % 16 || ((uintptr_t)src & 15)) return DQ_EINVAL;
  if (bytes == 0) return DQ_OK;
  const size_t n16 = bytes / 16;
  size_t blocks = n16 / (16 * 64 * 4);   // at least one full load group per wave
  if (blocks > 1024) blocks = 1024;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream,
                     reinterpret_cast<const u32x4*>(src), n16, sink);
  DQ_HIP_CHECK(hipGetLastError());
  return DQ_OK;
}
