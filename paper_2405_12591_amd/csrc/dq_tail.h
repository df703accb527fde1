// The fp16 tail of a sequence (tokens appended since the last compressed block, Section 3.2 of
// arXiv 2405.12591) as one more partial result of the decode step: plain fp32 attention of the
// query heads of one kv head over at most kMaxTailRows rows, computed by one workgroup.
//
// A row of D halves is read by D/8 lanes, 16 bytes each, so a wave covers 4 (D = 128) or 8 (D = 64)
// whole rows per load; the query heads of the group share every row that is read.  The work comes in
// two halves so that a caller can put other loads in flight between them:
//   issue_keys()  starts the loads of q and of the first batch of key and value rows (no
//                 dependent address: rows below the capacity are readable whatever the length);
//   finish()      scores, softmax over the rows, weighted sum of the value rows; leaves
//                 out[head][0..D) (unnormalised), out[head][D] = max score in log2 units
//                 (-inf for an empty tail) and out[head][D + 1] = sum of weights in `result`.
#pragma once

#include "dq_decode.h"

namespace dq {

typedef _Float16 tail_h8 __attribute__((ext_vector_type(8)));
typedef uint32_t tail_u4 __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ float tail_dpp(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// D: head dimension.  NWV: waves in the workgroup (all of them must call both functions).
// HEADS: query heads handled together (every row read serves all of them).
// PAIR: D = 128 stands for two neighbouring kv heads of 64 channels, each with its own query head
// (HEADS = 2): a row is the two heads' rows side by side (the lanes of each half read their own
// head's array), query head hd is zero outside its own half, and so result[hd] is head hd's
// partial in channels [64 hd, 64 hd + 64); the other half of it means nothing.
template <int D, int NWV, int HEADS, bool PAIR = false>
struct TailBlock {
  static_assert(!PAIR || (D == 128 && HEADS == 2), "a pair is two heads of 64 channels");
  static constexpr int RD = PAIR ? D / 2 : D;   // halves per row in memory
  static constexpr int LPR = D / 8;      // lanes per row
  static constexpr int RPI = 64 / LPR;   // rows per wave-wide load
  static constexpr int HB = HEADS;
  // Row loads a lane keeps in flight, all requested before the tail's length is known: 128 rows per
  // workgroup either way (rows past the capacity re-read the last row, so a deeper batch on eight
  // waves only added loads: +1.5 us per launch on the long-context shape against +0.4 us now).
  static constexpr int BATCH = (NWV >= 8) ? 4 : 8;
  static constexpr int ROWS_PER_BATCH = BATCH * RPI * NWV;
  // floats of LDS scratch finish() needs, and of the result it leaves
  static constexpr int kScratchFloats = HB * kMaxTailRows + NWV * HB * D + 2 * HB * NWV;
  static constexpr int kResultFloats = HB * (D + 2);

  tail_u4 kreg[BATCH], vreg[BATCH], qraw[HB];
  float qreg[HB][8];
  float qk;
  const uint16_t* kt;
  const uint16_t* vt;
  int lane, wave, chunk, rsub, cap;

  __device__ __forceinline__ int batch_row(int batch, int it) const {
    return batch * ROWS_PER_BATCH + RPI * (wave + NWV * it) + rsub;
  }

  // heads [hq0, hq0 + nh) of sequence b are the query heads of kv head h (nh <= HB)
  __device__ __forceinline__ void issue_keys(const DecodeArgs& a, int b, int h, long hq0, int nh) {
    lane = threadIdx.x & 63; wave = threadIdx.x >> 6;
    chunk = lane % LPR; rsub = lane / LPR;
    cap = a.tail.capacity;
    const int H = a.cache.kv_heads;
    // the lane's 8 halves of a row: kt + row * RD
    const int own = PAIR ? chunk / (LPR / 2) : 0;          // which head of the pair the lane reads
    const int part = PAIR ? chunk % (LPR / 2) : chunk;
    kt = a.tail.k_tail + ((long)b * H + h + own) * cap * RD + 8 * part;
    vt = a.tail.v_tail + ((long)b * H + h + own) * cap * RD + 8 * part;
    qk = a.scale * 1.4426950408889634f;
#pragma unroll
    for (int hd = 0; hd < HB; ++hd)
      qraw[hd] = *reinterpret_cast<const tail_u4*>(a.q + ((long)b * a.q_heads + hq0 + min(hd, nh - 1)) * RD + 8 * part);
    // Rows below the capacity are readable whatever the tail's length, which is not known yet; rows
    // past the capacity read the last row instead.  No branches: the caller may have other loads in
    // flight whose count the compiler has to keep.
#pragma unroll
    for (int it = 0; it < BATCH; ++it)
      kreg[it] = *reinterpret_cast<const tail_u4*>(kt + (long)min(batch_row(0, it), cap - 1) * RD);
#pragma unroll
    for (int it = 0; it < BATCH; ++it)
      vreg[it] = *reinterpret_cast<const tail_u4*>(vt + (long)min(batch_row(0, it), cap - 1) * RD);
  }

  __device__ __forceinline__ void score_rows(const tail_u4 (&rows)[BATCH], int batch, int n_tail, float* sc) {
#pragma unroll
    for (int it = 0; it < BATCH; ++it) {
      const int row = batch_row(batch, it);
      const tail_h8 kv = __builtin_bit_cast(tail_h8, rows[it]);
      float part[HB];
#pragma unroll
      for (int hd = 0; hd < HB; ++hd) part[hd] = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float kf = (float)kv[i];
#pragma unroll
        for (int hd = 0; hd < HB; ++hd) part[hd] = fmaf(kf, qreg[hd][i], part[hd]);
      }
#pragma unroll
      for (int hd = 0; hd < HB; ++hd) {
        float v = part[hd];
        // a pair: the lanes on the other head's half of the row add an outright zero (their query is
        // zero, but zero times whatever that head's row holds need not be)
        if (PAIR && chunk / (LPR / 2) != hd) v = 0.f;
        v += tail_dpp<0xB1>(v);                    // lane ^ 1
        v += tail_dpp<0x4E>(v);                    // lane ^ 2
        v += tail_dpp<0x141>(v);                   // 7 - lane within 8
        if (LPR == 16) v += tail_dpp<0x140>(v);    // 15 - lane within 16
        if (chunk == 0 && row < n_tail) sc[hd * kMaxTailRows + row] = v;
      }
    }
  }

  // tail_len: the caller's read of tail_lens[b] (requested early, so that it has arrived by now)
  __device__ __forceinline__ void finish(int tail_len, int nh, float* scratch, float* result) {
    float* sc = scratch;                       // [HB][kMaxTailRows] scores, then weights
    float* red = scratch + HB * kMaxTailRows;  // [NWV][HB][D]
    float* stat = red + NWV * HB * D;          // [2][HB][NWV]
    const int tid = threadIdx.x;
    const int n_tail = min(max(tail_len, 0), cap);
#pragma unroll
    for (int hd = 0; hd < HB; ++hd) {
      // nothing derived from q may move above loads the caller issued after issue_keys()
      asm volatile("" : "+v"(qraw[hd].x), "+v"(qraw[hd].y), "+v"(qraw[hd].z), "+v"(qraw[hd].w));
      const tail_h8 qv = __builtin_bit_cast(tail_h8, qraw[hd]);
#pragma unroll
      for (int i = 0; i < 8; ++i) qreg[hd][i] = (hd < nh && (!PAIR || chunk / (LPR / 2) == hd)) ? (float)qv[i] * qk : 0.f;
    }
    const int n_batches = (n_tail + ROWS_PER_BATCH - 1) / ROWS_PER_BATCH;
    // ---- scores ----
    if (n_batches > 0) score_rows(kreg, 0, n_tail, sc);
    for (int batch = 1; batch < n_batches; ++batch) {
      tail_u4 rows[BATCH];
#pragma unroll
      for (int it = 0; it < BATCH; ++it) {
        const int row = batch_row(batch, it);
        rows[it] = tail_u4{0u, 0u, 0u, 0u};
        if (row < n_tail) rows[it] = *reinterpret_cast<const tail_u4*>(kt + (long)row * RD);
      }
      score_rows(rows, batch, n_tail, sc);
    }
    __syncthreads();
    // ---- softmax over the rows: thread t owns rows t, t + 64 NWV, ... ----
    float m[HB];
#pragma unroll
    for (int hd = 0; hd < HB; ++hd) {
      float v = -INFINITY;
      for (int t = tid; t < n_tail; t += 64 * NWV) v = fmaxf(v, sc[hd * kMaxTailRows + t]);
      for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
      if (lane == 0) stat[hd * NWV + wave] = v;
    }
    __syncthreads();
#pragma unroll
    for (int hd = 0; hd < HB; ++hd) {
      float mm = -INFINITY;
#pragma unroll
      for (int w = 0; w < NWV; ++w) mm = fmaxf(mm, stat[hd * NWV + w]);
      m[hd] = mm;
      float v = 0.f;
      for (int t = tid; t < n_tail; t += 64 * NWV) {
        const float p = __builtin_amdgcn_exp2f(sc[hd * kMaxTailRows + t] - mm);
        sc[hd * kMaxTailRows + t] = p;
        v += p;
      }
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
      if (lane == 0) stat[(HB + hd) * NWV + wave] = v;
    }
    __syncthreads();
    // ---- weighted sum of the value rows ----
    float acc[HB][8];
#pragma unroll
    for (int hd = 0; hd < HB; ++hd)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[hd][i] = 0.f;
    for (int batch = 0; batch < n_batches; ++batch) {
      tail_u4 rows[BATCH];
#pragma unroll
      for (int it = 0; it < BATCH; ++it) {
        const int row = batch_row(batch, it);
        // batch 0 was requested by issue_keys() for every row below the capacity: rows past the
        // tail's length hold whatever the caller left there and are dropped here
        rows[it] = (row < n_tail) ? vreg[it] : tail_u4{0u, 0u, 0u, 0u};
        if (batch > 0 && row < n_tail) rows[it] = *reinterpret_cast<const tail_u4*>(vt + (long)row * RD);
      }
#pragma unroll
      for (int it = 0; it < BATCH; ++it) {
        const int row = batch_row(batch, it);
        const tail_h8 vv = __builtin_bit_cast(tail_h8, rows[it]);
        float w[HB];
#pragma unroll
        for (int hd = 0; hd < HB; ++hd) w[hd] = (row < n_tail) ? sc[hd * kMaxTailRows + row] : 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float vf = (float)vv[i];
#pragma unroll
          for (int hd = 0; hd < HB; ++hd) acc[hd][i] = fmaf(w[hd], vf, acc[hd][i]);
        }
      }
    }
    // lanes with the same chunk (different rows) add up, then the waves
#pragma unroll
    for (int hd = 0; hd < HB; ++hd) {
      if (hd < nh) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          float v = acc[hd][i];
          for (int o = LPR; o < 64; o <<= 1) v += __shfl_xor(v, o);
          if (rsub == 0) red[(wave * HB + hd) * D + 8 * chunk + i] = v;
        }
      }
    }
    __syncthreads();
    for (int idx = tid; idx < nh * D; idx += 64 * NWV) {
      const int hd = idx / D, c = idx % D;
      float o = 0.f;
#pragma unroll
      for (int w = 0; w < NWV; ++w) o += red[(w * HB + hd) * D + c];
      result[hd * (D + 2) + c] = o;
      if (c == 0) {
        float l = 0.f;
#pragma unroll
        for (int w = 0; w < NWV; ++w) l += stat[(HB + hd) * NWV + w];
        result[hd * (D + 2) + D] = (n_tail > 0) ? m[hd] : -INFINITY;
        result[hd * (D + 2) + D + 1] = l;
      }
    }
    __syncthreads();
  }
};

}  // namespace dq
