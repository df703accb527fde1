// Shared host/device helpers of libdecoquant (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "decoquant.h"

namespace dq {

constexpr int kTileTokens = 128;   // tokens per value-code tile and per decode work tile
constexpr int kMaxSplits = 64;     // upper bound on split-sequence partials per (b, head)
constexpr int kWsHeaderBytes = 256;
constexpr int kMaxCompressUnits = 1 << 22;   // blocks (keys and values counted apart) one compression call takes
constexpr int kMaxHeadGroups = 16; // matrix-core decode: groups of query heads per kv head
constexpr int kMaxGridY = 65535;   // largest y extent of a launch; more rows than that ride on the x index
constexpr int kMaxDecodeRows = 1 << 24;   // (sequence, query head) pairs one decode call takes (index arithmetic stays in 32 bits)
constexpr int kMaxTailRows = 1024; // rows of the fp16 tail a decode call takes per sequence and kv head
constexpr int kRun = 8;            // side of the third local tensor: tokens per run it mixes

// Record a failed HIP runtime call for dq_last_hip_error().
void set_last_hip_error(hipError_t e);

#define DQ_HIP_CHECK(expr)                         \
  do {                                             \
    hipError_t _e = (expr);                        \
    if (_e != hipSuccess) {                        \
      ::dq::set_last_hip_error(_e);                \
      return DQ_EHIP;                              \
    }                                              \
  } while (0)

inline bool format_ok(const dq_format* f) {
  if (!f) return false;
  if (f->bits != 2 && f->bits != 4 && f->bits != 8) return false;
  if (f->head_dim != 64 && f->head_dim != 128) return false;
  if (f->j1 != 8 && f->j1 != 16 && f->j1 != 32) return false;
  if (f->j2 <= 0 || f->j1 * f->j2 != f->head_dim) return false;
  if (f->group <= 0 || f->head_dim % f->group) return false;
  const int seg = f->head_dim / 2;
  if (!(f->group == f->head_dim || (f->group <= seg && seg % f->group == 0))) return false;
  if ((f->group * f->bits) % 32) return false;  // a group covers whole 32-bit words
  if (f->block_tokens <= 0 || f->block_tokens % kTileTokens) return false;
  if (f->i3 != 1 && f->i3 != kRun) return false;
  if (f->levels != 0 && f->levels != 1) return false;
  if (f->i1 != 1 && f->i1 != 2 && f->i1 != 4) return false;
  if (f->i1 > 1 && (f->i3 != 1 || f->i1 * f->j1 > 32)) return false;
  return true;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- cache geometry (element strides, in units of the array's element type) ----
struct Geometry {
  int bits, G, d, j1, j2, Tb;
  int row_bytes;        // d*bits/8
  int groups;           // d/G
  int tiles_per_block;  // Tb/128
  int vrow_bytes;       // 128*bits/8: bytes of one (b2, r) value row inside a tile
  long codes_per_block; // bytes of k_codes (== v_codes) per block
  long scales_per_block;
  long small_per_block;
  int NB, H;
};

__host__ __device__ inline Geometry make_geometry(const dq_format& f, int kv_heads, int block_capacity) {
  Geometry g;
  g.bits = f.bits; g.G = f.group; g.d = f.head_dim; g.j1 = f.j1; g.j2 = f.j2; g.Tb = f.block_tokens;
  g.row_bytes = f.head_dim * f.bits / 8;
  g.groups = f.head_dim / f.group;
  g.tiles_per_block = f.block_tokens / kTileTokens;
  g.vrow_bytes = kTileTokens * f.bits / 8;
  g.codes_per_block = (long)f.block_tokens * g.row_bytes;
  g.scales_per_block = (long)f.block_tokens * g.groups;
  g.small_per_block = (long)(f.i1 * f.j1) * (f.i1 * f.j1);
  g.NB = block_capacity; g.H = kv_heads;
  return g;
}

// ---- fp16 bit helpers (device) ----
__device__ inline float h2f(uint16_t h) {
  return (float)__builtin_bit_cast(_Float16, h);
}
__device__ inline uint16_t f2h_rne(float x) {
  return __builtin_bit_cast(uint16_t, (_Float16)x);
}

// fp64 -> fp16 bits with a single round-to-nearest-even; saturating variant clamps to +-65504.
__device__ inline uint16_t f64_to_f16_rne(double x, bool saturate, bool* saturated) {
  const uint64_t bits = __builtin_bit_cast(uint64_t, x);
  const uint16_t sign = (uint16_t)((bits >> 48) & 0x8000u);
  const double ax = __builtin_fabs(x);
  if (!(ax == ax)) return (uint16_t)(sign | 0x7E00u);
  if (ax >= 65520.0) {  // rounds to infinity
    if (saturated) *saturated = true;
    return (uint16_t)(sign | (saturate ? 0x7BFFu : 0x7C00u));
  }
  if (ax < 6.103515625e-05) {  // below 2^-14: subnormal grid of 2^-24
    const double r = __builtin_rint(ax * 16777216.0);
    return (uint16_t)(sign | (uint16_t)r);
  }
  const int e = (int)((bits >> 52) & 0x7FF) - 1023;  // floor(log2(ax)), -14 <= e <= 15
  // 2^(10-e) as a double, exact scaling so that one fp16 ulp becomes 1.0
  const double scale = __builtin_bit_cast(double, (uint64_t)(1023 + 10 - e) << 52);
  const double r = __builtin_rint(ax * scale);  // in [1024, 2048]
  const uint32_t h = ((uint32_t)(e + 15) << 10) + ((uint32_t)r - 1024u);
  return (uint16_t)(sign | h);
}

}  // namespace dq
