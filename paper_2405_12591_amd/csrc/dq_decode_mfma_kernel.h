// Matrix-core decode attention over the compressed cache for the formats
//   bits in {2, 4, 8};  group = 128 with 1, 2 or 4 query heads of a kv head per workgroup,
//                       group = 64  with 1 or 2
// with head_dim = 128, j1 = 16, j2 = 8, block_tokens % 128 == 0, two or three local tensors.
// More query heads per kv head are served by several workgroups (head groups) over the same codes.
// Heads of 64 channels (j1 = 8, j2 = 8, group = 64, one query head per kv head) ride in pairs: two
// neighbouring kv heads are worked as one head of 128 channels whose small tensors are block-diagonal
// and whose two query heads are the real ones padded with zeros (see P2 below).
//
// This is the fusion of dequantization with the product of the local tensors of Section 3.2 (arXiv
// 2405.12591) carried through the attention that follows it.  The low-bit codes never become
// floating point: a 32-bit word of codes is split into words of four bytes each
// (4-bit: x & 0x0F0F0F0F, (x >> 4) & 0x0F0F0F0F; 2-bit: (x >> 2k) & 0x03030303; 8-bit: x ^ 0x80808080) and fed to the
// int8 matrix cores; the other operand (the folded query, then the softmax weights times the
// value steps) is expressed as 7-bit integer limbs (four and three) relative to a per-tile power of two,
// one B column per limb, so the contraction is exact integer arithmetic.  Per 128-token tile,
// one wavefront
//   1. folds the keys' small tensor into the query,  q'[r, b2] = sum_b1 T_S^K[b1, r] q[b1, b2]
//      (one 16x16x16 f16 MFMA per two heads; T_S and q are fp16, so the products are exact),
//      and writes the limbs of q' * scale * log2(e) as B operands;
//   2. streams the key codes: S[t][limb] = sum_c (u[t, c] - offset) limb[c]  (16x16x64 i8 MFMA,
//      u = code + offset as stored; the offset's share comes from a constant-A MFMA and is the
//      accumulators' starting value);
//   3. online softmax with two tokens per lane (scores cross from the MFMA layout through
//      wave-private LDS); w_t = p_t * step^V_t is cut into limbs, again B columns;
//   4. streams the value codes (stored token-contiguous): o'[r, b2] = sum_t u[t, r, b2] limb[t];
//   5. applies the values' small tensor with fp32 16x16x4 MFMAs,
//      acc[b1, b2] = alpha * acc + sum_r T_S^V[b1, r] o'[r, b2]
//      (the limb columns of several b2 packed side by side first, so that the sixteen columns
//      of these MFMAs are all in use).
// With two step groups per token row (group = 64: rows r < 8 and r >= 8 of the large tensor)
// every limb gets one B column per group: the key side zeroes the limbs of the other group's
// channels, the value side takes each row of o' from the column of that row's group.
// A query head takes 4 (one group) or 8 (two groups) of the sixteen B columns.
//
// MFMA operand layouts (lane l: n = l % 16, g = l / 16):
//   A[m][k]: lane holds row m = n, k = S*g + i (S values per lane);  B[k][n]: column n, same k;
//   D[m][n]: lane holds column n, rows m = 4*g + i.
#pragma once

#include <hip/hip_ext.h>

#include <type_traits>

#include "dq_decode.h"
#include "dq_tail.h"

namespace dq {

typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kLimbBits = 7;
constexpr int kMantBits = 3 * kLimbBits;  // weights: 21-bit integers, limb0 * 2^14 + limb1 * 2^7 + limb2
// The folded query takes all four columns of its group of four: 28 bits relative to the tile's
// largest |q'|.  With three limbs the rounding of the small entries of q' (2^-21 of the largest one,
// times 128 channels) was the largest error of the whole kernel on peaked softmaxes.
constexpr int kQueryBits = 4 * kLimbBits;
// With three local tensors the weights are signed mixtures over a run of tokens and what they
// multiply cancels across the run: they take all four columns as well (27 bits and a sign relative
// to the tile's largest weight, i.e. every bit an fp32 weight has).
constexpr int kSignedWeightBits = 4 * kLimbBits;

// ---- per-bit-width pieces -------------------------------------------------------------------
// Chunk: what one lane loads of a 16-row piece of codes (32 bytes at 8 bits, 16 at 4, 8 at 2); it
// feeds two int8 MFMAs of 16 codes per lane each.  `slot(e)` is the byte position, inside the 16
// bytes a lane hands to one MFMA, of the e-th of its 16 consecutive codes.
template <int BITS> struct Codec;
template <> struct Codec<4> {
  typedef u32x4 chunk_t;
  static constexpr int kOffset = 8;
  // first MFMA: words x, y (codes 0..15 of the lane's 32); second: words z, w
  static __device__ __forceinline__ i32x4 half(const chunk_t& c, int which) {
    const uint32_t M = 0x0F0F0F0Fu;
    const uint32_t x0 = which ? c.z : c.x, x1 = which ? c.w : c.y;
    i32x4 v;
    v.x = (int)(x0 & M);          // codes 0, 2, 4, 6
    v.y = (int)((x0 >> 4) & M);   // codes 1, 3, 5, 7
    v.z = (int)(x1 & M);          // codes 8, 10, 12, 14
    v.w = (int)((x1 >> 4) & M);   // codes 9, 11, 13, 15
    return v;
  }
  static __device__ __forceinline__ int slot(int e) { return (e & 8) + (e & 1) * 4 + ((e & 7) >> 1); }
};
template <> struct Codec<2> {
  typedef u32x2 chunk_t;
  static constexpr int kOffset = 2;
  static __device__ __forceinline__ i32x4 half(const chunk_t& c, int which) {
    const uint32_t M = 0x03030303u;
    const uint32_t x = which ? c.y : c.x;
    i32x4 v;
    v.x = (int)(x & M);           // codes 0, 4, 8, 12
    v.y = (int)((x >> 2) & M);    // codes 1, 5, 9, 13
    v.z = (int)((x >> 4) & M);    // codes 2, 6, 10, 14
    v.w = (int)((x >> 6) & M);    // codes 3, 7, 11, 15
    return v;
  }
  static __device__ __forceinline__ int slot(int e) { return (e & 3) * 4 + (e >> 2); }
};

template <> struct Codec<8> {
  typedef uint32_t chunk_t __attribute__((ext_vector_type(8)));
  static constexpr int kOffset = 0;   // the stored byte becomes the signed code by flipping its top bit
  static __device__ __forceinline__ i32x4 half(const chunk_t& c, int which) {
    const uint32_t F = 0x80808080u;
    i32x4 v;
    v.x = (int)((which ? c.s4 : c.s0) ^ F);
    v.y = (int)((which ? c.s5 : c.s1) ^ F);
    v.z = (int)((which ? c.s6 : c.s2) ^ F);
    v.w = (int)((which ? c.s7 : c.s3) ^ F);
    return v;
  }
  static __device__ __forceinline__ int slot(int e) { return e; }
};

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float lane_f(float v, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
// Maximum over the wave, taken on integer keys that order like the floats (for v >= 0 the bit
// pattern itself; otherwise the low 31 bits of negative values are flipped): an integer maximum
// takes its partner lane's value straight from the DPP operand, where a floating-point one needs
// the value copied and quieted first.  All-reduce over the 16 lanes of a row, then over the four rows.
__device__ __forceinline__ int wave_allmax_key(int x) {
  x = max(x, dpp_i<0xB1>(x));    // quad_perm [1,0,3,2]
  x = max(x, dpp_i<0x4E>(x));    // quad_perm [2,3,0,1]
  x = max(x, dpp_i<0x141>(x));   // row_half_mirror
  x = max(x, dpp_i<0x140>(x));   // row_mirror
  return max(max(__builtin_amdgcn_readlane(x, 0), __builtin_amdgcn_readlane(x, 16)),
             max(__builtin_amdgcn_readlane(x, 32), __builtin_amdgcn_readlane(x, 48)));
}
__device__ __forceinline__ float wave_allmax(float v) {          // any finite values and -inf
  int x = __builtin_bit_cast(int, v);
  x ^= (x >> 31) & 0x7FFFFFFF;
  x = wave_allmax_key(x);
  x ^= (x >> 31) & 0x7FFFFFFF;
  return __builtin_bit_cast(float, x);
}
__device__ __forceinline__ float wave_allmax_nonneg(float v) {   // v >= 0 (+0 only)
  return __builtin_bit_cast(float, wave_allmax_key(__builtin_bit_cast(int, v)));
}
__device__ __forceinline__ float wave_allsum(float v) {
  v += dpp_f<0xB1>(v);
  v += dpp_f<0x4E>(v);
  v += dpp_f<0x141>(v);
  v += dpp_f<0x140>(v);
  return (lane_f(v, 0) + lane_f(v, 16)) + (lane_f(v, 32) + lane_f(v, 48));
}

// 2^e as a float for -126 <= e <= 127
__device__ __forceinline__ float pow2i(int e) {
  return __builtin_bit_cast(float, (uint32_t)(e + 127) << 23);
}

// BITS: code width.  NG: step groups per token row (group = 128 / NG).  R: query heads per kv head.  NW: wavefronts per workgroup (4 or 8); the tiles
// of one (sequence, kv head) are dealt round-robin to the NW waves of each of its n_split workgroups.
// TM: what to do about the fp16 tail (tokens not yet compressed).  0: there is none.  1: the launch
// has one workgroup per (sequence, kv head), which works the tail off while its first codes are on
// their way.  2: the launch has several workgroups per (sequence, kv head); the one of split 0 does
// the same and hands the tail's partial in with its own.  (A workgroup of its own for the tail was
// tried: on a full chip its few dependent loads take tens of microseconds behind the streams, and
// the workgroups queued behind it start that much later.)
// N3: three local tensors (format.i3 == 8).  Row a2*8 + e of the codes then belongs to the bond
// index e of the third tensor instead of a token: the tile's 128 row sums y are computed as
// before, the scores of the eight tokens of a run are s[a3] = sum_e T_3^K[e, a3] y[e], and the
// value rows are weighted with p'[e] = sum_a3 T_3^V[e, a3] p[a3] (signed, so these weights get a
// signed top limb like the query's).  The lanes that hold the eight rows of a run form a quad,
// so both products are quad broadcasts and fused multiply-adds.
// P2: a pair of kv heads of 64 channels each (j1 = 8), one query head per kv head, as one virtual
// head of 128 channels and two step groups (NG = 2, R = 2).  Virtual row r of the large tensors is row
// r % 8 of head r / 8, a virtual token row is the two heads' rows side by side, virtual query head hd
// is real head hd's query in its own 64 channels and zero in the other's, and the small tensors are
// the heads' 8 x 8 ones on the diagonal of a 16 x 16 one.  Scores, softmax and the epilogue then run
// unchanged: head hd's scores come from its own channels only, and its output sits in virtual
// channels [64 hd, 64 hd + 64) (the other half, the other head's values under this head's weights,
// is dropped).  Only addresses (each lane reads its own head's arrays), the masks that realise the
// zeros, and the mapping of the output differ.
template <int BITS, int NG, int R, int NW, int TM, bool N3, bool P2>
__global__ __launch_bounds__(64 * NW, (NW == 4 && BITS < 8) ? 2 : 1) void decode_mfma_kernel(DecodeArgs a) {
  static_assert(!P2 || (NG == 2 && R == 2 && !N3), "a pair of heads is two step groups and two query heads");
  typedef Codec<BITS> C;
  typedef typename C::chunk_t chunk_t;
  constexpr int CPH = 4 * NG;                 // B columns per head: column CPH*head + 4*group + limb
  constexpr int NC = CPH * R;
  static_assert(NC <= 16, "too many heads for sixteen B columns");
  constexpr int F = (R + 1) / 2;              // fold MFMAs (two heads each)
  constexpr int D = 128, J1 = 16, J2 = 8;
  // The epilogue multiplies o'[r][column] by the values' small tensor, sixteen columns at a time,
  // but one b2 fills only 3 R of them (one limb triple per head, once the two step groups' columns
  // have been merged): the columns of PK = 4 / R successive b2 are packed side by side first.
  // With four heads (R = 4) that packing would leave one b2 per set and 32 fp32 matrix instructions
  // per tile, which on this chip cost what ten vector instructions each cost (matrix and vector
  // instructions of one SIMD do not run side by side).  There the three limbs of a head are joined
  // first, as floats, by lane shifts (column 4*head + limb holds limb `limb`, most significant first),
  // and the joined columns of four successive b2 are packed side by side: 8 matrix instructions
  // per tile, and a quarter of the accumulators.
  constexpr bool JOIN = (R == 4 && NG == 1 && !N3 && !P2);
  constexpr int PK = JOIN ? 4 : 4 / R, NSET = J2 / PK;
  constexpr int RD = P2 ? 64 : D;             // channels of a real head (output, partials, cache rows)
  constexpr int RJ1 = P2 ? 8 : J1;            // rows of a real head's large tensors
  constexpr int ROWB = RD * BITS / 8;         // bytes of a key row in memory
  constexpr int VROWB = kTileTokens * BITS / 8;   // bytes of a value row (one r, one b2) in a tile
  constexpr int CHUNKB = sizeof(chunk_t);
  constexpr int SS = 132;                     // ints per column of the score staging (128 tokens + pad)
  constexpr int QS_BYTES = NC * 128, PS_BYTES = NC * 128, SS_BYTES = NC * SS * 4;
  constexpr int WAVE_LDS = QS_BYTES + PS_BYTES + SS_BYTES;
  static_assert(WAVE_LDS >= NC * D * 4 + 2 * R * 4, "merge area must fit the wave's LDS");
  __shared__ __attribute__((aligned(16))) unsigned char smem[NW * WAVE_LDS];
  // the fp16 tail's partial result (computed once per (sequence, kv head), by split 0, before the
  // first tile; its scratch borrows the waves' areas, which are not in use yet)
  typedef TailBlock<D, NW, R, P2> Tail;
  static_assert(sizeof(smem) >= Tail::kScratchFloats * sizeof(float), "tail scratch must fit the waves' LDS");
  __shared__ float s_tail[R * (D + 2)];
  __shared__ int s_last;
  __shared__ float s_wgt[4][kMaxSplits + 1];
  __shared__ float s_sum[4];

  const int tid = threadIdx.x, lane = tid & 63;
#ifdef DQ_TIMELINE
  // time line of this wave (instrumented build only): slot numbers in dq_decode.h
  unsigned long long* const tl_wave = a.timeline
      ? a.timeline + ((long)(blockIdx.y * gridDim.x + blockIdx.x) * NW + (tid >> 6)) * kTimelineSlots : nullptr;
#define DQ_STAMP(slot)                                                          \
  do {                                                                          \
    if (tl_wave && lane == 0) tl_wave[slot] = __builtin_amdgcn_s_memrealtime(); \
  } while (0)
#else
#define DQ_STAMP(slot) \
  do {                 \
  } while (0)
#endif
  DQ_STAMP(0);
#ifdef DQ_TIMELINE
  if (tl_wave && lane == 0) tl_wave[20] = NW;
#endif
  // the wave's number as a scalar: everything derived from it (its tiles, their addresses) is then
  // computed once per wave on the scalar unit instead of once per lane
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, g = lane >> 4;
  // More query heads per kv head than the sixteen B columns hold (R of them per workgroup) are
  // served in head groups: head_groups workgroups per (sequence, kv head, split), each streaming
  // the same codes for its own R heads.  The groups are the slow part of the grid's y index, so the
  // workgroups of one (sequence, kv head) are a multiple of eight apart in launch order (whenever
  // the number of units is one) and land on the same XCD: while they run side by side, the second
  // to ask for a line finds it in that XCD's L2.
  // (rows normally ride on the grid's y index, splits of a row next to each other in launch order;
  // more rows than a y extent takes ride on x)
  const int split = a.rows_on_x ? blockIdx.y : blockIdx.x;
  const int row = a.rows_on_x ? blockIdx.x : blockIdx.y;
  const int n_units = (a.rows_on_x ? gridDim.x : gridDim.y) / a.head_groups;
  const int hgrp = row / n_units;
  const int bh = unit_of_row(row % n_units, n_units, a.unit_map);
  const int H = a.cache.kv_heads, NB = a.cache.block_capacity;
  constexpr int HPU = P2 ? 2 : 1;              // kv heads per unit
  const int b = bh / (H / HPU), h = (bh % (H / HPU)) * HPU;
  const long bh0 = (long)b * H + h;            // the unit's (first) kv head among all (sequence, kv head) pairs
  const int tpb = a.fmt.block_tokens / kTileTokens;
  const long codes_per_block = (long)a.fmt.block_tokens * ROWB;
  constexpr int MG = P2 ? 1 : NG;              // step groups per row in memory
  const long scales_per_block = (long)a.fmt.block_tokens * MG;

  // The sequence length lives in device memory and takes a memory round trip to read.  Tiles are dealt round-robin over all waves of all splits of this (sequence, kv head), so a wave's
  // first tile does not depend on the sequence length and its loads can start before the length is
  // known; they are wasted only if the sequence is shorter than that tile.
  const int first_tile = split * NW + wave;
  const int tile_stride = a.n_split * NW;
  const bool spec_ok = first_tile * kTileTokens < a.max_seq_len;
  int S = 0;  // the sequence's real length, read after the speculative loads are on their way

  // ---- the last workgroup of this (sequence, kv head) to finish merges the partial results ----
  const long hq_first = (long)h * (a.q_heads / H) + (long)hgrp * R;   // this workgroup's first query head
  // the last group may hold fewer than R heads (3 = 3, 7 = 4 + 3 query heads per kv head): the columns
  // of the missing ones compute on a zero query and are never written out
  const int nh = P2 ? 2 : min(R, a.q_heads / H - hgrp * R);
  const long bhq0 = (long)b * a.q_heads + hq_first;
  int32_t* const ticket_counter = a.counters + (long)bh * a.head_groups + hgrp;
  const int n_contrib = a.n_split;   // workgroups that hand in partials
  auto ticket_and_merge = [&]() __attribute__((always_inline)) {
    // Ordering of the hand-over.  Producer: the partials above are device-scope (sc1) stores, which
    // write through the XCD's L2; every wave waits here until all of its own stores have been
    // acknowledged (the vector memory counter counts stores on this chip), and only after the
    // barrier that follows, i.e. after every wave of the workgroup has done so, does one thread take
    // a ticket, itself a device-scope read-modify-write performed at the memory side.  Consumer: the
    // workgroup that draws the last ticket knows that every other workgroup's increment, and so
    // every store ahead of it, has been performed; its loads of the partials are device-scope
    // loads (never served from this XCD's stale lines) issued after the second barrier, which the
    // compiler may not move them across.  No cache write-back or invalidation is involved.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (tid == 0) {
      const int ticket = __hip_atomic_fetch_add(ticket_counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_last = (ticket == n_contrib - 1);
      if (s_last) __hip_atomic_store(ticket_counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // clean for the next call
    }
    __syncthreads();
    if (!s_last) return;
    // Wave hd requests the maxima and sums of head hd's partials, one slot per lane, and every
    // thread the first eight slots of its output element, all in flight together; wave hd leaves
    // each slot's weight in LDS; then every thread adds up
    // its element over the slots, eight device-scope loads at a time (slots past the last one are
    // not read and weigh nothing).
    const int ns = a.n_slots;   // <= kMaxSplits + 1 (the tail's slot included)
    auto load_slots = [&](const float* col, int sp, float (&v)[8]) __attribute__((always_inline)) {
#pragma unroll
      for (int k = 0; k < 8; ++k)
        v[k] = (sp + k < ns) ? __hip_atomic_load(col + (sp + k) * (RD + 2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
    };
    float v_first[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float m0 = -INFINITY, l0 = 0.f, m1 = -INFINITY, l1 = 0.f;
    if (wave < nh) {
      const float* base = a.partials + (bhq0 + wave) * ns * (RD + 2);
      if (lane < ns) {
        m0 = __hip_atomic_load(base + lane * (RD + 2) + RD, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        l0 = __hip_atomic_load(base + lane * (RD + 2) + RD + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      if (lane + 64 < ns) {
        m1 = __hip_atomic_load(base + (lane + 64) * (RD + 2) + RD, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        l1 = __hip_atomic_load(base + (lane + 64) * (RD + 2) + RD + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    if (tid < nh * RD) load_slots(a.partials + (bhq0 + tid / RD) * ns * (RD + 2) + tid % RD, 0, v_first);
    if (wave < nh) {
      const float M = wave_allmax(fmaxf(m0, m1));
      const float w0 = (m0 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m0 - M);
      const float w1 = (m1 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m1 - M);
      if (lane < ns) s_wgt[wave][lane] = w0;
      if (lane + 64 < ns) s_wgt[wave][lane + 64] = w1;
      const float L = wave_allsum(l0 * w0 + l1 * w1);
      if (lane == 0) s_sum[wave] = L;
    }
    __syncthreads();
    for (int idx = tid; idx < nh * RD; idx += 64 * NW) {
      const int hd = idx / RD, c = idx % RD;
      const float* col = a.partials + (bhq0 + hd) * ns * (RD + 2) + c;
      float o = 0.f;
      for (int sp = 0; sp < ns; sp += 8) {
        float v[8];
        if (idx == tid && sp == 0) {
#pragma unroll
          for (int k = 0; k < 8; ++k) v[k] = v_first[k];
        } else {
          load_slots(col, sp, v);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const float wk = (sp + k < ns) ? s_wgt[hd][sp + k] : 0.f;
          o = (wk != 0.f) ? fmaf(v[k], wk, o) : o;   // an empty slot contributes nothing whatever it holds
        }
      }
      const float L = s_sum[hd];
      const float r = (L > 0.f) ? o / L : 0.f;
      a.out[(bhq0 + hd) * RD + c] = f2h_rne(r);
      if (a.out_f32) a.out_f32[(bhq0 + hd) * RD + c] = r;
    }
  };


  unsigned char* wl = smem + wave * WAVE_LDS;
  unsigned char* Qs = wl;                                        // [NC][8 row pairs][16 slots] bytes
  unsigned char* Ps = wl + QS_BYTES;                             // [NC][8 token groups][16 slots] bytes
  int* Ss = reinterpret_cast<int*>(wl + QS_BYTES + PS_BYTES);    // [NC][SS] ints
  const bool col_live = (n < NC) && (N3 || (n & 3) != 3);   // value side: three limbs per group of four columns (four with three local tensors)
  const bool col_live_k = n < NC;                      // key side: four
  // the epilogue's packed columns (see PK): column n holds head packed_head, slot packed_slot of its set
  const int packed_head = (R == 1) ? 0 : (R == 4) ? (n >> 2) : (NG == 1) ? ((n >> 2) & 1) : (n >> 3);
  const int packed_slot = JOIN ? (n & 3) : (R == 1) ? (n >> 2) : (R == 4) ? 0 : (NG == 1) ? (n >> 3) : ((n >> 2) & 1);

  // softmax layout: lane = 8*G16 + pi owns the two tokens of token group G16 whose weights sit in
  // B slots 2*pi and 2*pi + 1
  // (with three tensors and 2-bit codes the low lane bits are dealt the other way round, which
  // puts the eight rows of a run into one quad of lanes)
  const int G16 = lane >> 3, pi = (N3 && BITS == 2) ? (((lane & 3) << 1) | ((lane >> 2) & 1)) : (lane & 7);
  int tA, tB;
  if (BITS == 4) { tA = 16 * G16 + 8 * (pi >> 2) + ((0x5140 >> (4 * (pi & 3))) & 7); tB = tA + 2; }
  else if (BITS == 2) { tA = 16 * G16 + 8 * (pi & 1) + (pi >> 1); tB = tA + 4; }
  else { tA = 16 * G16 + 2 * pi; tB = tA + 1; }

  // loop-invariant B operands of the fold, q[k = b1][n' = (b2, head)].  The loads go out first (the
  // memory counter retires in issue order and q is needed before the first codes); the values are
  // packed further down, after the first tile's codes have been requested, so that the wait for q
  // does not sit in front of those requests.
  half4 bq[F];
  uint32_t q_raw[F][4];
  {
    const int b2 = n & 7;
#pragma unroll
    for (int f = 0; f < F; ++f) {
      const int hd = 2 * f + (n >> 3);
      // no branch here (columns past the last head read head nh - 1 and are zeroed when packed):
      // across a branch the compiler loses count of the loads in flight and waits for all of them
      // (a pair of heads: virtual row b1 = 4g + i of virtual head hd is row b1 % 8 of the real head;
      // the rows of the other head's half are zeroed when packed)
      const uint16_t* qp = a.q + (bhq0 + min(hd, nh - 1)) * RD;
#pragma unroll
      for (int i = 0; i < 4; ++i) q_raw[f][i] = qp[((4 * g + i) & (RJ1 - 1)) * J2 + b2];
    }
  }

  float m_run[R], l_run[R];
#pragma unroll
  for (int hd = 0; hd < R; ++hd) { m_run[hd] = -INFINITY; l_run[hd] = 0.f; }
  f32x4 acc[NSET];
#pragma unroll
  for (int st = 0; st < NSET; ++st) acc[st] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const float qk_scale = a.scale * kLog2e;
  constexpr int kMinusWord = (int)((uint32_t)((256 - C::kOffset) & 255) * 0x01010101u);  // four bytes of -offset
  const i32x4 a_minus = {kMinusWord, kMinusWord, kMinusWord, kMinusWord};
  const i32x4 izero = {0, 0, 0, 0};

  // ---- the code stream of one wave: 16 chunks per tile (keys j = 0..7 in slots 0..7, values
  // b2 = 0..7 in slots 8..15) flow through a 16-slot register ring; a slot is refilled in place
  // with the same chunk of the wave's next tile as soon as it has been unpacked, so one whole
  // tile per wave is in flight at all times.  The memory counter retires loads in issue order,
  // so everything is requested in the order it will be used: the next tile's small tensors and
  // steps first (needed before its first key chunk), then the refills.
  chunk_t ring[16];
  struct Side { u32x2 ksm, vsm; uint32_t dkA, dkB, dvA, dvB; };   // small tensors + the lane's steps
  Side cur = {{0, 0}, {0, 0}, 0, 0, 0, 0};
  // three tensors: the columns of T_3^K of the lane's two tokens and the rows of T_3^V of its two
  // rows, eight fp16 each (kept apart from Side so that the other instances carry nothing of it)
  struct Side3 { u32x4 k3A, k3B, v3A, v3B; };
  Side3 cur3 = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
  // a pair of heads: the second head's steps of the lane's two tokens (its step group 1)
  struct SideP { uint32_t dkA, dkB, dvA, dvB; };
  SideP curP = {0, 0, 0, 0};
  // the lane's part of a block-diagonal small tensor lies on the diagonal
  const bool small_live = !P2 || (g >> 1) == (n >> 3);

  auto tile_ptrs = [&](int tile, const unsigned char*& kc, const unsigned char*& vc, long& blkid, int& tib) {
    blkid = bh0 * NB + tile / tpb;
    tib = tile % tpb;
    if (P2) {
      // keys: a virtual row is the two heads' rows side by side, two chunks each; values: virtual
      // row r of a b2 is row r % 8 of head r / 8 (the second head's blocks lie NB blocks further on)
      kc = a.cache.k_codes + (blkid + (g >> 1) * NB) * codes_per_block + (long)tib * kTileTokens * ROWB + n * ROWB + CHUNKB * (g & 1);
      vc = a.cache.v_codes + (blkid + (n >> 3) * NB) * codes_per_block + (long)tib * kTileTokens * ROWB + (n & 7) * VROWB + CHUNKB * g;
    } else {
      kc = a.cache.k_codes + blkid * codes_per_block + (long)tib * kTileTokens * ROWB + n * ROWB + CHUNKB * g;
      vc = a.cache.v_codes + blkid * codes_per_block + (long)tib * kTileTokens * ROWB + n * VROWB + CHUNKB * g;
    }
  };
  auto load_steps = [&](const uint16_t* p, int t) -> uint32_t {   // the fp16 steps of token t as stored
    if (MG == 1) return p[t];
    return *reinterpret_cast<const uint32_t*>(p + 2 * t);
  };
  auto load_side = [&](Side& sd, long blkid, int tib) {
    if (P2) {
      // the lane's row of its own head's 8 x 8 small tensor (used only where small_live)
      const long sb = (blkid + (n >> 3) * NB) * (RJ1 * RJ1) + (n & 7) * RJ1 + 4 * (g & 1);
      sd.ksm = *reinterpret_cast<const u32x2*>(a.cache.k_small + sb);
      sd.vsm = *reinterpret_cast<const u32x2*>(a.cache.v_small + sb);
    } else {
      sd.ksm = *reinterpret_cast<const u32x2*>(a.cache.k_small + blkid * (J1 * J1) + n * J1 + 4 * g);
      sd.vsm = *reinterpret_cast<const u32x2*>(a.cache.v_small + blkid * (J1 * J1) + n * J1 + 4 * g);
    }
    const uint16_t* ksc = a.cache.k_scales + blkid * scales_per_block + tib * kTileTokens * MG;
    const uint16_t* vsc = a.cache.v_scales + blkid * scales_per_block + tib * kTileTokens * MG;
    sd.dkA = load_steps(ksc, tA); sd.dkB = load_steps(ksc, tB);
    sd.dvA = load_steps(vsc, tA); sd.dvB = load_steps(vsc, tB);
  };
  auto load_sideP = [&](SideP& sd, long blkid, int tib) {   // the same steps of the pair's second head
    const uint16_t* ksc = a.cache.k_scales + (blkid + NB) * scales_per_block + tib * kTileTokens;
    const uint16_t* vsc = a.cache.v_scales + (blkid + NB) * scales_per_block + tib * kTileTokens;
    sd.dkA = ksc[tA]; sd.dkB = ksc[tB];
    sd.dvA = vsc[tA]; sd.dvB = vsc[tB];
  };
  auto load_side3 = [&](Side3& sd, long blkid) {
    const uint16_t* k3 = a.cache.k_small3 + blkid * (kRun * kRun);   // [a3][e]
    const uint16_t* v3 = a.cache.v_small3 + blkid * (kRun * kRun);   // [e][a3]
    sd.k3A = *reinterpret_cast<const u32x4*>(k3 + (tA & 7) * kRun);
    sd.k3B = *reinterpret_cast<const u32x4*>(k3 + (tB & 7) * kRun);
    sd.v3A = *reinterpret_cast<const u32x4*>(v3 + (tA & 7) * kRun);
    sd.v3B = *reinterpret_cast<const u32x4*>(v3 + (tB & 7) * kRun);
  };
  auto issue_tile = [&](int tile) {
    const unsigned char *kc, *vc;
    long blkid;
    int tib;
    tile_ptrs(tile, kc, vc, blkid, tib);
    load_side(cur, blkid, tib);
    if (N3) load_side3(cur3, blkid);
    if (P2) load_sideP(curP, blkid, tib);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 8; ++j) ring[j] = __builtin_nontemporal_load(reinterpret_cast<const chunk_t*>(kc + j * (16 * ROWB)));
#pragma unroll
    for (int b2 = 0; b2 < 8; ++b2) ring[8 + b2] = __builtin_nontemporal_load(reinterpret_cast<const chunk_t*>(vc + b2 * (RJ1 * VROWB)));
  };
  // fp16 step of group grp: from the packed word, or (a pair of heads) from the second head's word
  auto step_of = [&](uint32_t packed, uint32_t second, int grp) -> float {
    if (P2) return h2f((uint16_t)(grp ? second : packed));
    return h2f((uint16_t)(grp ? (packed >> 16) : (packed & 0xFFFFu)));
  };

  // Three tensors: outA = sum over the run of coefA[row] * x[row] (and outB with coefB), where the
  // eight values x of a run sit in a quad of lanes, two per lane (xA, xB), and the coefficient
  // vectors hold one fp16 per row of the run.  Quad lane k holds the rows offA(k) and offB(k).
  auto quad_mix = [&](float xA, float xB, const u32x4& coefA, const u32x4& coefB, float& outA, float& outB)
                      __attribute__((always_inline)) {
    typedef _Float16 half8 __attribute__((ext_vector_type(8)));
    const half8 cA = __builtin_bit_cast(half8, coefA), cB = __builtin_bit_cast(half8, coefB);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int offA = (BITS == 4) ? ((0x5140 >> (4 * k)) & 7) : (BITS == 2) ? k : 2 * k;
      const int offB = (BITS == 4) ? offA + 2 : (BITS == 2) ? k + 4 : 2 * k + 1;
      float a_k, b_k;
      switch (k) {   // the DPP control must be a literal
        case 0: a_k = dpp_f<0x00>(xA); b_k = dpp_f<0x00>(xB); break;
        case 1: a_k = dpp_f<0x55>(xA); b_k = dpp_f<0x55>(xB); break;
        case 2: a_k = dpp_f<0xAA>(xA); b_k = dpp_f<0xAA>(xB); break;
        default: a_k = dpp_f<0xFF>(xA); b_k = dpp_f<0xFF>(xB); break;
      }
      outA = fmaf((float)cA[offA], a_k, outA);
      outA = fmaf((float)cA[offB], b_k, outA);
      outB = fmaf((float)cB[offA], a_k, outB);
      outB = fmaf((float)cB[offB], b_k, outB);
    }
  };

  // One tile.  HAS_NEXT: the wave has another tile after this one.
  auto compute_tile = [&](const int tile, auto has_next_tag) __attribute__((always_inline)) {
    constexpr bool HAS_NEXT = decltype(has_next_tag)::value;
    const int tok0 = tile * kTileTokens;
    const unsigned char *kc_next = nullptr, *vc_next = nullptr;
    long blkid_next = 0;
    int tib_next = 0;
    if (HAS_NEXT) tile_ptrs(tile + tile_stride, kc_next, vc_next, blkid_next, tib_next);
    Side nxt = cur;
    if (HAS_NEXT) load_side(nxt, blkid_next, tib_next);
    Side3 nxt3;
    if (N3) {
      nxt3 = cur3;
      if (HAS_NEXT) load_side3(nxt3, blkid_next);
    }
    SideP nxtP;
    if (P2) {
      nxtP = curP;
      if (HAS_NEXT) load_sideP(nxtP, blkid_next, tib_next);
    }
    __builtin_amdgcn_sched_barrier(0);
    const bool okA = (tok0 + tA) < S, okB = (tok0 + tB) < S;
    // three tensors: a row counts as soon as its run of eight holds a valid token
    const bool rowA = N3 ? (tok0 + (tA & ~7)) < S : okA, rowB = N3 ? (tok0 + (tB & ~7)) < S : okB;
    float dvA[NG], dvB[NG], dkA[NG], dkB[NG];
#pragma unroll
    for (int gr = 0; gr < NG; ++gr) {
      dvA[gr] = rowA ? step_of(cur.dvA, curP.dvA, gr) : 0.f;
      dvB[gr] = rowB ? step_of(cur.dvB, curP.dvB, gr) : 0.f;
      dkA[gr] = step_of(cur.dkA, curP.dkA, gr);
      dkB[gr] = step_of(cur.dkB, curP.dkB, gr);
    }
    const half4 vsm_h = __builtin_bit_cast(half4, small_live ? cur.vsm : u32x2{0u, 0u});

    // ---- 1. fold T_S^K into q; limbs of q' relative to 2^e >= max |q'| ----
    float q_unscale;
    float q_unscale_second = 0.f;   // a pair of heads: each head's query gets a scale of its own
    {
      const half4 aK = __builtin_bit_cast(half4, small_live ? cur.ksm : u32x2{0u, 0u});
      f32x4 fd[F];
      float amax = 0.f;
#pragma unroll
      for (int f = 0; f < F; ++f) {
        fd[f] = __builtin_amdgcn_mfma_f32_16x16x16f16(aK, bq[f], (f32x4){0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        // a pair of heads: rows r = 4g + i of the other head's half are zero by construction; they
        // are set to zero outright so that nothing the other head holds (a NaN, say) gets across
        if (P2 && !small_live) fd[f] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i) amax = fmaxf(amax, fabsf(fd[f][i]));
      }
      auto exponent_of = [&](float m) -> int {
        int e = 0;
        if (m > 0.f && m < INFINITY) e = __builtin_amdgcn_frexp_expf(m);  // m = f * 2^e, f in [0.5, 1)
        return max(min(e, 100), -100);
      };
      int e;
      if (P2) {
        // the lane's column belongs to head n / 8: one maximum per head
        const int e_first = exponent_of(wave_allmax_nonneg((n >> 3) ? 0.f : amax) * qk_scale);
        const int e_second = exponent_of(wave_allmax_nonneg((n >> 3) ? amax : 0.f) * qk_scale);
        e = (n >> 3) ? e_second : e_first;
        q_unscale = pow2i(e_first - (kQueryBits - 1));
        q_unscale_second = pow2i(e_second - (kQueryBits - 1));
      } else {
        e = exponent_of(wave_allmax_nonneg(amax) * qk_scale);
        q_unscale = pow2i(e - (kQueryBits - 1));
      }
      const float qn = qk_scale * pow2i(kQueryBits - 1 - e);   // |q' * qn| < 2^27
      // the fold's D layout: lane (n' = b2 + 8*head, g) holds rows r = 4g + i.  Channel (r, b2) is
      // code number (r & 1)*8 + b2 of the 16 codes that row pair r >> 1 contributes to one MFMA.
#pragma unroll
      for (int f = 0; f < F; ++f) {
        const int hd = 2 * f + (n >> 3);
        if (hd < R) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int vi = (int)__builtin_rintf(fd[f][i] * qn);
            const int r = 4 * g + i;
            const int grp = (NG == 2) ? (r >> 3) : 0;
            const int pos = (r >> 1) * 16 + C::slot((r & 1) * 8 + (n & 7));
            unsigned char* dst = Qs + (CPH * hd + 4 * grp) * 128 + pos;
            dst[0] = (unsigned char)(vi >> (3 * kLimbBits));
            dst[128] = (unsigned char)((vi >> (2 * kLimbBits)) & 127);
            dst[256] = (unsigned char)((vi >> kLimbBits) & 127);
            dst[384] = (unsigned char)(vi & 127);
          }
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
    i32x4 bqs[2];
#pragma unroll
    for (int w = 0; w < 2; ++w) {
      i32x4 t = izero;
      if (col_live_k) t = *reinterpret_cast<const i32x4*>(Qs + n * 128 + (2 * g + w) * 16);
      bqs[w] = t;
    }

    // ---- 2. scores: S[t][col] = sum_c (u[t, c] - offset) limb[col][c] ----
    // (the offset's share, the same for every token, is the accumulators' starting value)
    {
      i32x4 cinitk = izero;
      if (C::kOffset != 0) {
        cinitk = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_minus, bqs[0], izero, 0, 0, 0);
        cinitk = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_minus, bqs[1], cinitk, 0, 0, 0);
      }
      i32x4 s_prev = izero;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const i32x4 a0 = C::half(ring[j], 0), a1 = C::half(ring[j], 1);
        __builtin_amdgcn_sched_barrier(0);   // the slot is dead from here on: refill it in place
        if (HAS_NEXT) ring[j] = __builtin_nontemporal_load(reinterpret_cast<const chunk_t*>(kc_next + j * (16 * ROWB)));
        __builtin_amdgcn_sched_barrier(0);
        i32x4 s = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, bqs[0], cinitk, 0, 0, 0);
        s = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, bqs[1], s, 0, 0, 0);
        // the previous chunk's scores are stored while this chunk's MFMAs run
        if (j > 0 && col_live_k) *reinterpret_cast<i32x4*>(Ss + n * SS + 16 * (j - 1) + 4 * g) = s_prev;
        s_prev = s;
      }
      if (col_live_k) *reinterpret_cast<i32x4*>(Ss + n * SS + 16 * 7 + 4 * g) = s_prev;
    }
    __builtin_amdgcn_wave_barrier();

    // ---- 3. online softmax, tokens tA and tB per lane ----
    float v_unscale, vs = 0.f;
    float vs_second = 0.f;   // a pair of heads: the second head's steps get a scale of their own
    if (!N3) {
      float dvm = fmaxf(dvA[0], dvB[0]);
      if (NG == 2 && !P2) dvm = fmaxf(dvm, fmaxf(dvA[NG - 1], dvB[NG - 1]));
      const float dvmax = wave_allmax_nonneg(dvm);
      int e = 0;
      if (dvmax > 0.f && dvmax < INFINITY) e = __builtin_amdgcn_frexp_expf(dvmax);
      vs = pow2i(kMantBits - e);   // p * step * vs < 2^21
      v_unscale = pow2i(e - kMantBits);
      if (P2) {
        const float dvmax2 = wave_allmax_nonneg(fmaxf(dvA[NG - 1], dvB[NG - 1]));
        int e2 = 0;
        if (dvmax2 > 0.f && dvmax2 < INFINITY) e2 = __builtin_amdgcn_frexp_expf(dvmax2);
        vs_second = pow2i(kMantBits - e2);
        // the epilogue's rows b1 = n of the second head (n >= 8) undo the second head's scale
        if (n >> 3) v_unscale = pow2i(e2 - kMantBits);
      }
    }
    float alpha[R];
    float wA[R][NG], wB[R][NG];   // three tensors: the weights, kept until their common scale is known
    float wmax = 0.f;
#pragma unroll
    for (int hd = 0; hd < R; ++hd) {
      float sA = 0.f, sB = 0.f;
#pragma unroll
      for (int gr = 0; gr < NG; ++gr) {
        if (P2 && gr != hd) continue;   // a head of a pair has its channels in its own step group only
        const int* s0 = Ss + (CPH * hd + 4 * gr) * SS;
        const int* s1 = s0 + SS;
        const int* s2 = s1 + SS;
        const int* s3 = s2 + SS;
        // limb pairs are joined as integers (|S| < 2^17 per limb: 128 channels x 8 x 127), then as floats
        sA += ((float)(s0[tA] * 128 + s1[tA]) * 16384.f + (float)(s2[tA] * 128 + s3[tA])) * dkA[gr];
        sB += ((float)(s0[tB] * 128 + s1[tB]) * 16384.f + (float)(s2[tB] * 128 + s3[tB])) * dkB[gr];
      }
      if (N3) {   // rows -> tokens with T_3^K
        const float yA = sA, yB = sB;
        sA = 0.f; sB = 0.f;
        quad_mix(yA, yB, cur3.k3A, cur3.k3B, sA, sB);
      }
      const float unscale = (P2 && hd) ? q_unscale_second : q_unscale;
      sA = okA ? sA * unscale : -INFINITY;
      sB = okB ? sB * unscale : -INFINITY;
      // the running maximum moves in a sequence's first tiles and rarely afterwards: the wave-wide
      // reduction runs only when some lane holds a score above it
      const float mt_lane = fmaxf(sA, sB);
      float m_new = m_run[hd];                           // finite after the first tile (it has a valid token)
      alpha[hd] = 1.f;
      if (__any(mt_lane > m_new)) {
        m_new = wave_allmax(mt_lane);
        alpha[hd] = __builtin_amdgcn_exp2f(m_run[hd] - m_new);
      }
      const float pA = __builtin_amdgcn_exp2f(sA - m_new);
      const float pB = __builtin_amdgcn_exp2f(sB - m_new);
      l_run[hd] = l_run[hd] * alpha[hd] + (pA + pB);
      m_run[hd] = m_new;
      if (N3) {   // tokens -> rows with T_3^V; the weights are signed
        float qA = 0.f, qB = 0.f;
        quad_mix(pA, pB, cur3.v3A, cur3.v3B, qA, qB);
#pragma unroll
        for (int gr = 0; gr < NG; ++gr) {
          wA[hd][gr] = rowA ? qA * dvA[gr] : 0.f;
          wB[hd][gr] = rowB ? qB * dvB[gr] : 0.f;
          wmax = fmaxf(wmax, fmaxf(fabsf(wA[hd][gr]), fabsf(wB[hd][gr])));
        }
      } else {
#pragma unroll
        for (int gr = 0; gr < NG; ++gr) {
          // a pair of heads: only the head's own rows are kept, so only their column gets weights
          // (the other one stays zero from the start)
          if (P2 && gr != hd) continue;
          const float vsg = (P2 && gr) ? vs_second : vs;
          const float wa = okA ? pA * (dvA[gr] * vsg) : 0.f;
          const float wb = okB ? pB * (dvB[gr] * vsg) : 0.f;
          const uint32_t iA = min((uint32_t)(wa + 0.5f), (1u << kMantBits) - 1u);
          const uint32_t iB = min((uint32_t)(wb + 0.5f), (1u << kMantBits) - 1u);
          unsigned char* dst = Ps + (CPH * hd + 4 * gr) * 128 + G16 * 16 + 2 * pi;
          *reinterpret_cast<uint16_t*>(dst) = (uint16_t)((iA >> 14) | ((iB >> 14) << 8));
          *reinterpret_cast<uint16_t*>(dst + 128) = (uint16_t)(((iA >> 7) & 127u) | (((iB >> 7) & 127u) << 8));
          *reinterpret_cast<uint16_t*>(dst + 256) = (uint16_t)((iA & 127u) | ((iB & 127u) << 8));
        }
      }
    }
    if (N3) {
      // limbs relative to the largest weight of the tile: |w * vs| < 2^27, top limb signed
      wmax = wave_allmax_nonneg(wmax);
      int e = 0;
      if (wmax > 0.f && wmax < INFINITY) e = __builtin_amdgcn_frexp_expf(wmax);
      e = max(min(e, 100), -100);
      vs = pow2i(kSignedWeightBits - 1 - e);
      v_unscale = pow2i(e - (kSignedWeightBits - 1));
#pragma unroll
      for (int hd = 0; hd < R; ++hd) {
#pragma unroll
        for (int gr = 0; gr < NG; ++gr) {
          const int iA = (int)__builtin_rintf(wA[hd][gr] * vs), iB = (int)__builtin_rintf(wB[hd][gr] * vs);
          unsigned char* dst = Ps + (CPH * hd + 4 * gr) * 128 + G16 * 16 + 2 * pi;
          *reinterpret_cast<uint16_t*>(dst) = (uint16_t)(((iA >> 21) & 255) | (((iB >> 21) & 255) << 8));
          *reinterpret_cast<uint16_t*>(dst + 128) = (uint16_t)(((iA >> 14) & 127) | (((iB >> 14) & 127) << 8));
          *reinterpret_cast<uint16_t*>(dst + 256) = (uint16_t)(((iA >> 7) & 127) | (((iB >> 7) & 127) << 8));
          *reinterpret_cast<uint16_t*>(dst + 384) = (uint16_t)((iA & 127) | ((iB & 127) << 8));
        }
      }
    }
    __builtin_amdgcn_wave_barrier();

    // ---- 4 + 5. o' = sum_t u limb per b2, then the small-tensor epilogue ----
    i32x4 bp[2];
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      i32x4 t = izero;
      if (col_live) t = *reinterpret_cast<const i32x4*>(Ps + n * 128 + (2 * g + v) * 16);
      bp[v] = t;
    }
    float alpha_col = 1.f;
#pragma unroll
    for (int hd = 0; hd < R; ++hd) alpha_col = (packed_head == hd) ? alpha[hd] : alpha_col;
    float aT[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) aT[i] = (float)vsm_h[i] * v_unscale;
    i32x4 cinitv = izero;
    if (C::kOffset != 0) {
      cinitv = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_minus, bp[0], izero, 0, 0, 0);
      cinitv = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_minus, bp[1], cinitv, 0, 0, 0);
    }
    if (__any(alpha_col != 1.f)) {   // the running maximum moved: rare after the first tiles
#pragma unroll
      for (int st = 0; st < NSET; ++st) acc[st] *= alpha_col;
    }
    // o' of one b2 arrives with column 4*(NG*head + group) + limb.  pack() puts it into the
    // set's B operand: with two step groups a column's weights carry the step of one group only,
    // so rows r = 4g + i < 8 are taken from the first group's column and rows >= 8 from the second
    // group's (four lanes further on), which leaves one limb triple per head; then the triple
    // moves to the bank of four columns that slot k = b2 % PK owns.
    auto pack = [&](i32x4& pk, i32x4 o, auto k_tag) __attribute__((always_inline)) {
      constexpr int K = decltype(k_tag)::value % PK;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int v = o[i];
        if (NG == 2) v = __builtin_amdgcn_update_dpp(v, v, 0x104 /* row_shl:4 */, 0xC, 0x5, false);
        if (K == 0) {
          pk[i] = v;
        } else {
          // live banks after the merge: R = 1: {0};  R = 2: {0, 1} (one group), {0, 2} (two groups)
          constexpr int kShift = (R == 2 && NG == 1) ? 8 * K : 4 * K;
          constexpr int kBanks = ((R == 1) ? 0x1 : (NG == 1) ? 0x3 : 0x5) << (kShift / 4);
          pk[i] = __builtin_amdgcn_update_dpp(pk[i], v, 0x110 + kShift /* row_shr */, 0xF, kBanks, false);
        }
      }
    };
    // JOIN: the limbs of o' joined as floats.  In the lane of column 4*head + k the three limbs of
    // that head sit k, k - 1 and k - 2 lanes below; every lane computes the combination with the
    // same shifts and the lanes of slot k = b2 % 4 keep it.  The joined value (|o'| < 2^32) takes one
    // fp32 rounding, of the size of the accumulation's own.
    auto pack_joined = [&](i32x4& pk, i32x4 o, auto k_tag) __attribute__((always_inline)) {
      constexpr int K = decltype(k_tag)::value % 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float f = (float)o[i];
        const int fb = __builtin_bit_cast(int, f);
        // (shift by zero lanes: the value itself)
        const float l0 = K == 0 ? f : __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, fb, 0x110 + K /* row_shr:K */, 0xF, 0xF, true));
        const float l1 = K == 1 ? f : K == 0 ? __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, fb, 0x101 /* row_shl:1 */, 0xF, 0xF, true))
                                             : __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, fb, 0x110 + (K - 1), 0xF, 0xF, true));
        const float l2 = K == 2 ? f : K == 3 ? __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, fb, 0x111 /* row_shr:1 */, 0xF, 0xF, true))
                                             : __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, fb, 0x100 + (2 - K) /* row_shl */, 0xF, 0xF, true));
        const float joined = fmaf(l0, 16384.f, fmaf(l1, 128.f, l2));
        pk[i] = ((n & 3) == K) ? __builtin_bit_cast(int, joined) : pk[i];
      }
    };
    auto epilogue = [&](int st, const i32x4& pk) __attribute__((always_inline)) {
      f32x4 c = acc[st];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int word = pk[i];   // (a copy: the bit cast below wants an object, not an element of a vector)
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(aT[i], JOIN ? __builtin_bit_cast(float, word) : (float)word, c, 0, 0, 0);
      }
      acc[st] = c;
    };
    i32x4 pk_cur = izero, pk_done = izero;
#pragma unroll
    for (int b2 = 0; b2 < J2; ++b2) {
      const i32x4 a0 = C::half(ring[8 + b2], 0), a1 = C::half(ring[8 + b2], 1);
      __builtin_amdgcn_sched_barrier(0);
      if (HAS_NEXT) ring[8 + b2] = __builtin_nontemporal_load(reinterpret_cast<const chunk_t*>(vc_next + b2 * (RJ1 * VROWB)));
      __builtin_amdgcn_sched_barrier(0);
      i32x4 o = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, bp[0], cinitv, 0, 0, 0);
      o = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, bp[1], o, 0, 0, 0);
      // the previous set's epilogue runs while this b2's integer MFMAs do
      if (b2 > 0 && b2 % PK == 0) epilogue(b2 / PK - 1, pk_done);
      if constexpr (JOIN) {
        if (b2 % 4 == 0) pack_joined(pk_cur, o, std::integral_constant<int, 0>{});
        else if (b2 % 4 == 1) pack_joined(pk_cur, o, std::integral_constant<int, 1>{});
        else if (b2 % 4 == 2) pack_joined(pk_cur, o, std::integral_constant<int, 2>{});
        else pack_joined(pk_cur, o, std::integral_constant<int, 3>{});
      } else if (b2 % PK == 0) pack(pk_cur, o, std::integral_constant<int, 0>{});
      else if (b2 % PK == 1) pack(pk_cur, o, std::integral_constant<int, 1>{});
      else if (b2 % PK == 2) pack(pk_cur, o, std::integral_constant<int, 2>{});
      else pack(pk_cur, o, std::integral_constant<int, 3>{});
      if (b2 % PK == PK - 1) pk_done = pk_cur;
    }
    epilogue(NSET - 1, pk_done);
    cur = nxt;
    if (N3) cur3 = nxt3;
    if (P2) curP = nxtP;
    __builtin_amdgcn_wave_barrier();
  };

  // The first requests go out in one straight line of code, without a branch: across a branch the
  // compiler loses count of the loads in flight and makes every later wait a wait for all of them.
  // So a wave whose first tile lies past max_seq_len reads tile 0 instead (in bounds: the cache
  // holds at least one block) and throws it away, and with TM == 1 every row of the tail below its
  // capacity is requested whatever the tail's length.  The tail's rows go first: they are worked
  // off while the codes are on their way.
  Tail tb;
  const bool do_tail = (TM == 1) || (TM == 2 && split == 0);   // TM == 2: a branch, and coarser waits
  if (do_tail) tb.issue_keys(a, b, h, hq_first, nh);
  issue_tile(spec_ok ? first_tile : 0);
  // Both lengths are requested only now (a scalar load that is still out holds up every wait on
  // scalar data, the addresses of the loads above among them) and before the asm statements below
  // (after them the compiler no longer treats memory as unchanged and would fetch these with vector
  // loads, whose wait covers the requests above).
  const int seq_len_raw = a.seq_lens[b];
  const int tail_len_raw = do_tail ? a.tail.tail_lens[b] : 0;
#pragma unroll
  for (int f = 0; f < F; ++f) {
    const bool head_live = (2 * f + (n >> 3)) < nh && (!P2 || (g >> 1) == (n >> 3));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      asm volatile("" : "+v"(q_raw[f][i]));   // nothing derived from q may move above the requests
      bq[f][i] = __builtin_bit_cast(_Float16, (uint16_t)(head_live ? q_raw[f][i] : 0u));
    }
  }
  if (do_tail) tb.finish(tail_len_raw, nh, reinterpret_cast<float*>(smem), s_tail);

  if (NG == 2) {
    // A channel contributes nothing to the other group's columns: those bytes of the query limbs
    // are the same in every tile and are zeroed once (the fold writes only its own group's).
    static_assert(QS_BYTES % 16 == 0, "");
    for (int o = lane * 16; o < QS_BYTES; o += 64 * 16) *reinterpret_cast<i32x4*>(Qs + o) = izero;
    if (P2) {   // the weight columns of the other head's step group are never written: zero for good
      static_assert(PS_BYTES % 16 == 0, "");
      for (int o = lane * 16; o < PS_BYTES; o += 64 * 16) *reinterpret_cast<i32x4*>(Ps + o) = izero;
    }
    __builtin_amdgcn_wave_barrier();
  }
  S = min(max(seq_len_raw, 0), a.max_seq_len);
  const int tiles_total = (S + kTileTokens - 1) / kTileTokens;
  DQ_STAMP(1);
  {
    int tile = first_tile;
    [[maybe_unused]] int nth = 0;
    if (tile < tiles_total) {
      if (!spec_ok) issue_tile(tile);   // cannot happen while seq_len <= max_seq_len; kept for safety
      for (; tile + tile_stride < tiles_total; tile += tile_stride) {
        DQ_STAMP(2 + min(nth++, 15));
        compute_tile(tile, std::true_type{});
      }
      DQ_STAMP(2 + min(nth++, 15));
      compute_tile(tile, std::false_type{});
    }
  }
  DQ_STAMP(18);

  // ---- merge the waves of the workgroup ----
  float* Macc = reinterpret_cast<float*>(wl);            // [NC][128] per wave (reuses the wave's LDS)
  float* Mml = Macc + NC * D;                            // [R] m, [R] l
#pragma unroll
  for (int hd = 0; hd < R; ++hd) l_run[hd] = wave_allsum(l_run[hd]);
  if (JOIN) {                 // [head][0][channel b1 * 8 + b2]: the limbs are joined already
#pragma unroll
    for (int st = 0; st < NSET; ++st) {
#pragma unroll
      for (int i = 0; i < 4; ++i) Macc[4 * packed_head * D + (4 * g + i) * J2 + st * PK + packed_slot] = acc[st][i];
    }
  } else if (N3 || (n & 3) != 3) {   // [head][limb][channel b1 * 8 + b2]
#pragma unroll
    for (int st = 0; st < NSET; ++st) {
#pragma unroll
      for (int i = 0; i < 4; ++i) Macc[(4 * packed_head + (n & 3)) * D + (4 * g + i) * J2 + st * PK + packed_slot] = acc[st][i];
    }
  }
  if (lane == 0) {
#pragma unroll
    for (int hd = 0; hd < R; ++hd) { Mml[hd] = m_run[hd]; Mml[R + hd] = l_run[hd]; }
  }
  __syncthreads();
  for (int idx = tid; idx < nh * RD; idx += 64 * NW) {
    // c: the real head's channel; cv: where it sits among the 128 channels the waves worked on
    const int hd = idx / RD, c = idx % RD, cv = P2 ? c + RD * hd : c;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) M = fmaxf(M, reinterpret_cast<const float*>(smem + w * WAVE_LDS)[NC * D + hd]);
    float o = 0.f, L = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float* base = reinterpret_cast<const float*>(smem + w * WAVE_LDS);
      const float mw = base[NC * D + hd];
      const float wgt = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - M);
      const float* col = base + 4 * hd * D + cv;
      const float v = JOIN ? col[0]
                      : N3 ? ((col[0] * 128.f + col[D]) * 128.f + col[2 * D]) * 128.f + col[3 * D]
                           : col[0] * 16384.f + col[D] * 128.f + col[2 * D];
      o = fmaf(v, wgt, o);
      L = fmaf(base[NC * D + R + hd], wgt, L);
    }
    if (a.n_split == 1) {   // this workgroup saw the whole sequence: finish here
      if (TM == 1) {  // fold in the fp16 tail's partial
        const float* tp = s_tail + hd * (D + 2);
        const float mt = tp[D];
        const float Mn = fmaxf(M, mt);
        const float w0 = (M == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(M - Mn);
        const float w1 = (mt == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mt - Mn);
        o = o * w0 + tp[cv] * w1;
        L = L * w0 + tp[D + 1] * w1;
      }
      const float r = (L > 0.f) ? o / L : 0.f;
      a.out[(bhq0 + hd) * RD + c] = f2h_rne(r);
      if (a.out_f32) a.out_f32[(bhq0 + hd) * RD + c] = r;
    } else {
      // device-scope stores: they go through to memory, past the per-XCD L2, so that a workgroup
      // on another XCD can read them without any cache write-back or invalidation
      float* part = a.partials + ((bhq0 + hd) * a.n_slots + split) * (RD + 2);
      __hip_atomic_store(part + c, o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (c == 0) {
        __hip_atomic_store(part + RD, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // M in log2 units
        __hip_atomic_store(part + RD + 1, L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      if (TM == 2 && split == 0) {   // the tail's partial travels with split 0's, in the slot after the splits
        float* tpart = a.partials + ((bhq0 + hd) * a.n_slots + a.n_split) * (RD + 2);
        const float* tp = s_tail + hd * (D + 2);
        __hip_atomic_store(tpart + c, tp[cv], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (c == 0) {
          __hip_atomic_store(tpart + RD, tp[D], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(tpart + RD + 1, tp[D + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
  }
  if (a.n_split == 1) {
    DQ_STAMP(19);
    return;
  }

  ticket_and_merge();
  DQ_STAMP(19);
}
#undef DQ_STAMP
template <int BITS, int NG, int R, int TM, bool N3, bool P2>
inline void launch_tm(const DecodeArgs& a, hipStream_t st) {
  const int units = a.cache.batch * a.cache.kv_heads / (P2 ? 2 : 1);
  const dim3 grid = a.rows_on_x ? dim3(units * a.head_groups, a.n_split) : dim3(a.n_split, units * a.head_groups);
  // the events, when given, receive the kernel's own begin and end timestamps
  // (8-bit codes: a wave's ring of chunks is twice as large and an 8-wave workgroup runs out of
  // registers, so that width always takes 4 waves)
  if constexpr (BITS < 8) {
    if (a.nw == 8) {
      hipExtLaunchKernelGGL((decode_mfma_kernel<BITS, NG, R, 8, TM, N3, P2>), grid, dim3(512), 0, st, a.ev_start, a.ev_stop, 0, a);
      return;
    }
  }
  hipExtLaunchKernelGGL((decode_mfma_kernel<BITS, NG, R, 4, TM, N3, P2>), grid, dim3(256), 0, st, a.ev_start, a.ev_stop, 0, a);
}

template <int BITS, int NG, int R, bool N3, bool P2 = false>
inline void launch_n3(const DecodeArgs& a, hipStream_t st) {
  if (!a.tail.k_tail) launch_tm<BITS, NG, R, 0, N3, P2>(a, st);
  else if (a.n_split == 1) launch_tm<BITS, NG, R, 1, N3, P2>(a, st);
  else launch_tm<BITS, NG, R, 2, N3, P2>(a, st);
}

template <int BITS, int NG, int R>
inline void launch_r(const DecodeArgs& a, hipStream_t st) {
  if (a.fmt.i3 == kRun) launch_n3<BITS, NG, R, true>(a, st);
  else launch_n3<BITS, NG, R, false>(a, st);
}

template <int BITS>
int32_t launch_bits(const DecodeArgs& a, hipStream_t st) {
  if (a.pair_heads) {   // two kv heads of 64 channels per workgroup
    launch_n3<BITS, 2, 2, false, true>(a, st);
    return DQ_OK;
  }
  const int rep = a.heads_per_group;   // query heads per workgroup (the last group may hold fewer)
  if (a.fmt.group == 128) {
    switch (rep) {
      case 1: launch_r<BITS, 1, 1>(a, st); break;
      case 2: launch_r<BITS, 1, 2>(a, st); break;
      case 4: launch_r<BITS, 1, 4>(a, st); break;
      default: return DQ_EINVAL;
    }
  } else {
    switch (rep) {
      case 1: launch_r<BITS, 2, 1>(a, st); break;
      case 2: launch_r<BITS, 2, 2>(a, st); break;
      default: return DQ_EINVAL;
    }
  }
  return DQ_OK;
}


}  // namespace dq
