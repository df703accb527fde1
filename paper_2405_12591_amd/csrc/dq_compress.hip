// Compression of K/V blocks into DecoQuant form (Section 3.1 of arXiv 2405.12591):
//   step 1  two-site MPO split of the regrouped block, M = T_S * T_L            (Eq. 2, Eq. 3)
//   step 2  per-group round-to-nearest quantization of T_L, T_S kept in fp16   (Eq. 1)
// Two kernels: `decompose_kernel` (Gram matrix, Jacobi eigen-solver, projection; one wave per block) writes the
// small tensor into the cache and the fp32 large tensor into the workspace;
// `quantize_tiles_kernel` turns fp32 rows into packed codes and fp16 steps.
#include "dq_common.h"

namespace dq {

// What one dq_compress_kv call works on: t_new rows per (sequence, kv head), cut into n_blocks
// blocks of T_b rows (the last one may be short); block j of sequence b goes to slot blk_idx[b] + j.
struct CompressJob {
  const uint16_t* k_new;     // [B, H, t_new, d] fp16 bits
  const uint16_t* v_new;
  int t_new;
  int n_blocks;              // ceil(t_new / T_b)
  const int32_t* blk_idx;    // [B]
  const int32_t* n_valid;    // [B] or null
  int keep_large;            // the one-kernel three-tensor build also leaves its fp32 rows in the workspace
};

// Work unit `unit` = (((b * H + h) * n_blocks) + j) * 2 + which.  slot < 0: nothing to do (sequence
// skipped, slot past the cache's capacity, or a block none of whose rows is valid).
struct UnitRef {
  int which, b, slot, nv;    // nv: valid rows of this block (the rest count as zero)
  long bh;                   // b * H + h
  const uint16_t* X;         // the block's first row
};
__device__ __forceinline__ UnitRef unit_ref(const Geometry& g, const CompressJob& job, int unit) {
  UnitRef u;
  u.which = unit & 1;
  const int ub = unit >> 1;
  const int j = ub % job.n_blocks;
  u.bh = ub / job.n_blocks;
  u.b = (int)(u.bh / g.H);
  const int first = job.blk_idx[u.b];
  int rows = job.t_new;
  if (job.n_valid) rows = min(max(job.n_valid[u.b], 0), job.t_new);
  u.nv = min(max(rows - j * g.Tb, 0), g.Tb);
  u.slot = (first < 0 || first + j >= g.NB || u.nv == 0) ? -1 : first + j;
  u.X = (u.which ? job.v_new : job.k_new) + (u.bh * job.t_new + (long)j * g.Tb) * g.d;
  return u;
}

// ------------------------------------------------------------------------------------------
// Quantize + pack one tile of 128 token rows (Eq. 1 per group).  256 threads.
// ------------------------------------------------------------------------------------------

// Step of a group: fp16(amax / qmax), the exact quotient rounded once (nearest, ties to even).
// The quotient is first rounded to odd in fp32 (13 more bits than fp16), which makes the second
// rounding to fp16 land where a single rounding of the exact quotient would.
template <int QMAX>
__device__ __forceinline__ uint16_t group_step_bits(float amax) {
  if (QMAX == 1) return f2h_rne(amax);
  const float q = amax / (float)QMAX;                  // correctly rounded fp32 division
  const float e = fmaf(-(float)QMAX, q, amax);         // sign of (exact quotient - q); 0 iff q is exact
  uint32_t bits = __builtin_bit_cast(uint32_t, q);
  if (e > 0.f) bits |= 1u;                             // exact lies above q: odd end of [q, next]
  else if (e < 0.f) bits -= (bits & 1u) ? 0u : 1u;     // exact lies below q: odd end of [prev, q]
  return f2h_rne(__builtin_bit_cast(float, bits));
}

// Code of one element: nearest integer of the exact x / step, ties to even, clamped.
// `q` = x * (1/step) from the fp32 reciprocal estimate is within 4e-5 of the exact quotient
// (|q| <= 128, three roundings of 2^-23), so rint(q) is the answer unless q sits that close to a
// half-integer.  Only then the exact path runs: the residual x - c*step is exact in fp64 (24-bit x,
// 7-bit c, 11-bit step) and settles the candidate, ties included.
constexpr float kNearTie = 0.5f - 0x1p-12f;

// Value of another lane by a fixed data-parallel-primitive pattern (no LDS round trip).
template <int CTRL>
__device__ __forceinline__ float lane_exchange(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}

__device__ __forceinline__ int settle_code(float x, float c0, float step, double half_step) {
  const double r = fma(-(double)c0, (double)step, (double)x);
  int c = (int)c0;
  const double ar = fabs(r);
  const bool move = (ar > half_step) | ((ar == half_step) & ((c & 1) != 0));   // false when r is NaN (step = inf)
  c += move ? (r > 0.0 ? 1 : -1) : 0;
  return c;
}

// The stored fields (code + bias, one byte each) of four elements that share a step; the same
// arithmetic as in quantize_tile: the reciprocal estimate decides unless the quotient sits within
// 2^-12 of a half-integer, then the exact residual does.
template <int BITS, bool FULL>
__device__ __forceinline__ uint32_t fields_of_four(float x0, float x1, float x2, float x3, float step, float inv) {
  constexpr int QMAX = (1 << (BITS - 1)) - 1;
  constexpr int QMIN = FULL ? -QMAX - 1 : -QMAX;
  constexpr int BIAS = 1 << (BITS - 1);
  const float xs[4] = {x0, x1, x2, x3};
  uint32_t fields = 0;
  bool near = false;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float q = xs[e] * inv;
    const float cf = __builtin_rintf(q);
    near |= fabsf(q - cf) > kNearTie;
    fields |= (uint32_t)(min(max((int)cf, QMIN), QMAX) + BIAS) << (8 * e);
  }
  if (near) {   // rare
    const double hs = 0.5 * (double)step;
    fields = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int c = settle_code(xs[e], __builtin_rintf(xs[e] * inv), step, hs);
      fields |= (uint32_t)(min(max(c, QMIN), QMAX) + BIAS) << (8 * e);
    }
  }
  return fields;
}

// Second half of the quantizer: the tile's stored fields, one byte per element in lds_u[128][D],
// leave as packed codes in key layout (rows of D elements) or value layout ([b2][r][128 tokens]).
// All NT threads of the workgroup call it, after a barrier that follows the last field's store;
// it ends with a barrier (lds_u may be reused).  The value layout needs D * (128 * BITS / 32 + 1)
// words of staging behind the fields.
// Parts of a tile whose value rows are collected before they are stored: enough for 32 bytes.
__host__ __device__ constexpr int pack_parts(int bits, int qt) {
  const int want = bits == 8 ? 64 : 32;   // bytes per store and row
  return (qt * bits / 8 >= want || qt >= kTileTokens) ? 1 : (want * 8 / (qt * bits) < kTileTokens / qt ? want * 8 / (qt * bits) : kTileTokens / qt);
}

// QT < 128: lds_u holds QT rows, the rows [part * QT, (part + 1) * QT) of the tile that begins at
// codes_out (staging D * (pack_parts(BITS, QT) * QT * BITS / 32 + 1) words).
template <int BITS, int D, int NT, int QT = kTileTokens>
__device__ __forceinline__ void pack_fields(uint8_t* __restrict__ lds_u, int j1, int j2, int value_layout,
                                            uint8_t* __restrict__ codes_out, int part = 0) {
  constexpr int d = D;
  const int tid = threadIdx.x;
  constexpr int PER_WORD = 32 / BITS;
  constexpr int total_words = QT * d / PER_WORD;
  uint32_t* out32 = reinterpret_cast<uint32_t*>(codes_out);
  if (!value_layout) {
    // key layout: rows of d elements, element index contiguous
    out32 += part * total_words;
    for (int w = tid; w < total_words; w += NT) {
      const uint32_t* f = reinterpret_cast<const uint32_t*>(lds_u + w * PER_WORD);
      uint32_t word = 0;
#pragma unroll
      for (int k4 = 0; k4 < PER_WORD / 4; ++k4) {
        const uint32_t x = f[k4];
#pragma unroll
        for (int k = 0; k < 4; ++k) word |= ((x >> (8 * k)) & 0xFFu) << ((4 * k4 + k) * BITS);
      }
      out32[w] = word;
    }
  } else {
    // value layout: [b2][r][128 tokens], tokens contiguous.  Consecutive lanes take consecutive
    // columns (conflict-free byte reads), the words are transposed through a padded LDS buffer and
    // leave in output order.
    constexpr int WPR = QT / PER_WORD;            // words per (b2, r) row held here
    constexpr int WPR_TILE = kTileTokens / PER_WORD;   // ... and in the tile
    // A row's words of AP successive parts are collected in the staging area (it lies behind the
    // fields and survives from part to part) and leave together, so that no store is shorter
    // than 32 bytes: shorter pieces of a row cost the memory system a whole request each.
    constexpr int AP = pack_parts(BITS, QT);
    constexpr int WST = AP * WPR;                 // words per row in the staging area
    uint32_t* stage = reinterpret_cast<uint32_t*>(lds_u + QT * d);
    const int sub = part % AP;
    for (int idx = tid; idx < total_words; idx += NT) {
      const int col = idx % d, wi = idx / d;
      const int b2 = col % j2, r = col / j2;
      uint32_t word = 0;
#pragma unroll
      for (int k = 0; k < PER_WORD; ++k)
        word |= (uint32_t)lds_u[(wi * PER_WORD + k) * d + col] << (k * BITS);
      stage[(b2 * j1 + r) * (WST + 1) + sub * WPR + wi] = word;
    }
    __syncthreads();
    if (sub == AP - 1) {
      const int first = (part - sub) * WPR;       // the collected words' place in the tile's row
      for (int w = tid; w < AP * total_words; w += NT)
        out32[(w / WST) * WPR_TILE + first + w % WST] = stage[(w / WST) * (WST + 1) + w % WST];
    }
  }
  __syncthreads();
}

// FULL: the non-default level set (format.levels == 1): codes in [-QMAX - 1, QMAX], and the step is
// the larger of max(x) / QMAX and max(-x) / (QMAX + 1), each rounded once to fp16 (rounding is
// monotonic, so that is the rounded larger quotient; the second divisor is a power of two).
template <int BITS, int D, bool FULL>
__device__ __forceinline__ void quantize_tile(const float* __restrict__ src,  // [128, D] fp32
                              int G, int j1, int j2, int value_layout,
                              uint8_t* __restrict__ codes_out,    // tile's code bytes
                              uint16_t* __restrict__ scales_out,  // [128, D/G]
                              uint8_t* __restrict__ lds_u) {      // [128 * D] stored fields (+ value staging)
  constexpr int QMAX = (1 << (BITS - 1)) - 1;
  constexpr int QMIN = FULL ? -QMAX - 1 : -QMAX;
  constexpr int BIAS = 1 << (BITS - 1);
  constexpr int d = D;
  constexpr int LPR = D / 4;                 // lanes per row, 4 elements each: 32 or 16
  constexpr int ROWS_PER_PASS = 256 / LPR;
  constexpr int PASSES = kTileTokens / ROWS_PER_PASS;
  const int tid = threadIdx.x;
  const int li = tid & (LPR - 1), rp = tid / LPR;
  const int gl = G >> 2;                     // lanes per group, a power of two
  const int groups = d / G;

  // Straight-line over the passes, stage by stage, so that the 8 or 16 independent rows a thread
  // handles overlap their latencies (loads, cross-lane steps, the division) instead of queueing.
  float4 v[PASSES];                          // the whole tile in flight before the first use
#pragma unroll
  for (int ps = 0; ps < PASSES; ++ps)
    v[ps] = *reinterpret_cast<const float4*>(src + (long)(ps * ROWS_PER_PASS + rp) * d + 4 * li);
  // amax: max |x| of the group (FULL: max x, at least 0); amin (FULL only): max -x, at least 0
  float amax[PASSES], amin[PASSES];
#pragma unroll
  for (int ps = 0; ps < PASSES; ++ps) {
    if (FULL) {
      amax[ps] = fmaxf(fmaxf(fmaxf(v[ps].x, v[ps].y), fmaxf(v[ps].z, v[ps].w)), 0.f);
      amin[ps] = fmaxf(fmaxf(fmaxf(-v[ps].x, -v[ps].y), fmaxf(-v[ps].z, -v[ps].w)), 0.f);
    } else {
      amax[ps] = fmaxf(fmaxf(fabsf(v[ps].x), fabsf(v[ps].y)), fmaxf(fabsf(v[ps].z), fabsf(v[ps].w)));
      amin[ps] = 0.f;
    }
  }
  // group maximum over gl lanes: lane exchanges inside a row of 16 lanes, then across the two rows
  auto group_max = [&](float (&m)[PASSES]) __attribute__((always_inline)) {
    if (gl > 1) {
#pragma unroll
      for (int ps = 0; ps < PASSES; ++ps) m[ps] = fmaxf(m[ps], lane_exchange<0xB1>(m[ps]));    // i ^ 1
    }
    if (gl > 2) {
#pragma unroll
      for (int ps = 0; ps < PASSES; ++ps) m[ps] = fmaxf(m[ps], lane_exchange<0x4E>(m[ps]));    // i ^ 2
    }
    if (gl > 4) {
#pragma unroll
      for (int ps = 0; ps < PASSES; ++ps) m[ps] = fmaxf(m[ps], lane_exchange<0x141>(m[ps]));   // 7 - i in 8
    }
    if (gl > 8) {
#pragma unroll
      for (int ps = 0; ps < PASSES; ++ps) m[ps] = fmaxf(m[ps], lane_exchange<0x140>(m[ps]));   // 15 - i in 16
    }
    if (LPR > 16 && gl > 16) {
#pragma unroll
      for (int ps = 0; ps < PASSES; ++ps) m[ps] = fmaxf(m[ps], __shfl_xor(m[ps], 16));
    }
  };
  group_max(amax);
  if (FULL) group_max(amin);
  float step[PASSES], inv[PASSES];
#pragma unroll
  for (int ps = 0; ps < PASSES; ++ps) {
    uint16_t sbits = group_step_bits<QMAX>(amax[ps]);
    if (FULL) {
      // both are bit patterns of non-negative fp16 values (or +inf), which order like integers
      const uint16_t down = f2h_rne(amin[ps] * (1.0f / (float)(QMAX + 1)));   // exact: a power of two
      sbits = sbits > down ? sbits : down;
    }
    step[ps] = h2f(sbits);
    inv[ps] = step[ps] > 0.f ? __builtin_amdgcn_rcpf(step[ps]) : 0.f;   // step 0 (and inf): every code 0
    if ((li & (gl - 1)) == 0) scales_out[(ps * ROWS_PER_PASS + rp) * groups + li / gl] = sbits;
  }
  uint32_t near_mask = 0;
#pragma unroll
  for (int ps = 0; ps < PASSES; ++ps) {
    const float xs[4] = {v[ps].x, v[ps].y, v[ps].z, v[ps].w};
    uint32_t fields = 0;
    bool near = false;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float q = xs[e] * inv[ps];
      const float cf = __builtin_rintf(q);
      near |= fabsf(q - cf) > kNearTie;
      fields |= (uint32_t)(min(max((int)cf, QMIN), QMAX) + BIAS) << (8 * e);
    }
    near_mask |= (near ? 1u : 0u) << ps;
    *reinterpret_cast<uint32_t*>(lds_u + (ps * ROWS_PER_PASS + rp) * d + 4 * li) = fields;
  }
  if (near_mask) {   // rare: some quotient sits within 2^-12 of a half-integer
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
      if ((near_mask >> ps) & 1u) {
        const float xs[4] = {v[ps].x, v[ps].y, v[ps].z, v[ps].w};
        const double hs = 0.5 * (double)step[ps];
        uint32_t fields = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int c = settle_code(xs[e], __builtin_rintf(xs[e] * inv[ps]), step[ps], hs);
          fields |= (uint32_t)(min(max(c, QMIN), QMAX) + BIAS) << (8 * e);
        }
        *reinterpret_cast<uint32_t*>(lds_u + (ps * ROWS_PER_PASS + rp) * d + 4 * li) = fields;
      }
    }
  }
  __syncthreads();
  pack_fields<BITS, D, 256>(lds_u, j1, j2, value_layout, codes_out);
}

// LDS bytes quantize_tile needs: one byte per element plus the padded transpose buffer.
__host__ __device__ inline size_t quantize_lds_bytes(int d, int bits) {
  return (size_t)kTileTokens * d + (size_t)d * (kTileTokens * bits / 32 + 1) * sizeof(uint32_t);
}

// Stand-alone entry: contiguous input rows, contiguous outputs (dq_quantize_pack).
template <int BITS, int D, bool FULL>
__global__ __launch_bounds__(256) void quantize_pack_kernel(const float* __restrict__ t_large, int G, int j1,
                                                            int j2, int value_layout,
                                                            uint8_t* __restrict__ codes,
                                                            uint16_t* __restrict__ scales) {
  extern __shared__ uint8_t lds_u[];
  const long tile = blockIdx.x;
  const long tile_code_bytes = (long)kTileTokens * D * BITS / 8;
  quantize_tile<BITS, D, FULL>(t_large + tile * kTileTokens * D, G, j1, j2, value_layout,
                         codes + tile * tile_code_bytes, scales + tile * kTileTokens * (D / G), lds_u);
}

// The per-block status words of the decomposition become the call's two status words (flags OR-ed,
// sweeps at their maximum).  One workgroup of 256 threads.
__device__ __forceinline__ void fold_status(const int32_t* __restrict__ unit_status, int n_units,
                                            int32_t* __restrict__ status) {
  __shared__ int red[2];
  if (threadIdx.x < 2) red[threadIdx.x] = 0;
  __syncthreads();
  int flags = 0, sweeps = 0;
  for (int u = threadIdx.x; u < n_units; u += 256) {
    const int w = unit_status[u];
    flags |= w & 0xFF;
    sweeps = max(sweeps, w >> 8);
  }
  atomicOr(&red[0], flags);
  atomicMax(&red[1], sweeps);
  __syncthreads();
  if (threadIdx.x < 2) status[threadIdx.x] = red[threadIdx.x];
}

// Compress path: tile `blockIdx.x % tiles_per_block` of work unit `blockIdx.x / tiles_per_block`.
template <int BITS, int D, bool FULL>
__global__ __launch_bounds__(256) void quantize_tiles_kernel(const float* __restrict__ large_ws,
                                                             dq_format fmt, dq_cache cache,
                                                             CompressJob job,
                                                             const int32_t* __restrict__ unit_status,
                                                             int n_units, int32_t* __restrict__ status) {
  extern __shared__ uint8_t lds_u[];
  const Geometry g = make_geometry(fmt, cache.kv_heads, cache.block_capacity);
  if (blockIdx.x == 0) fold_status(unit_status, n_units, status);
  const int tile = blockIdx.x % g.tiles_per_block;
  const int unit = blockIdx.x / g.tiles_per_block;
  const UnitRef ur = unit_ref(g, job, unit);
  const int which = ur.which, slot = ur.slot;
  if (slot < 0) return;
  const long blk = ur.bh * g.NB + slot;
  const float* src = large_ws + ((long)unit * g.Tb + (long)tile * kTileTokens) * D;
  uint8_t* codes = (which ? cache.v_codes : cache.k_codes) + blk * g.codes_per_block +
                   (long)tile * kTileTokens * g.row_bytes;
  uint16_t* scales = (which ? cache.v_scales : cache.k_scales) + blk * g.scales_per_block +
                     (long)tile * kTileTokens * g.groups;
  quantize_tile<BITS, D, FULL>(src, g.G, g.j1, g.j2, which, codes, scales, lds_u);
}

// ------------------------------------------------------------------------------------------
// Decomposition: Gram matrix in fp64, parallel cyclic Jacobi, projection.  One wavefront per
// (sequence, kv head, K|V) block, so all synchronisation is inside one wave.
// ------------------------------------------------------------------------------------------
constexpr int kGramTile = 8;  // tokens staged in LDS per Gram step

// Reciprocal and reciprocal square root in fp64 from the hardware estimates plus Newton steps
// (relative error about 1e-16).  The Jacobi rotations sit on a serial path of a few lanes, where the
// compiler's IEEE-exact division and square root sequences cost several times more.
__device__ __forceinline__ double fast_rcp(double x) {
  double r = __builtin_amdgcn_rcp(x);
  r = r * (2.0 - x * r);
  r = r * (2.0 - x * r);
  return r;
}
__device__ __forceinline__ double fast_rsqrt(double x) {
  double y = __builtin_amdgcn_rsq(x);
  y = y * (1.5 - 0.5 * x * y * y);
  y = y * (1.5 - 0.5 * x * y * y);
  return y;
}

// n: side of the small tensor (i1 * j1); i1 rows are staged per token position
__host__ __device__ inline size_t decompose_lds_bytes(int n, int d, int i1) {
  const size_t mat = (size_t)n * (n + 1);
  return (5 * mat + 5 * (size_t)n) * sizeof(double) + 3 * (size_t)n * sizeof(int) +
         (size_t)kGramTile * d * i1 * sizeof(float) + 64;
}

// I1 > 1: a token factor on the small tensor (Eq. 2 with n = 2, i_1 = I1).  The regrouped matrix has
// rows (a1, b1) and columns (a2, b2), M[(a1, b1), (a2, b2)] = X[a1*i2 + a2, b1*j2 + b2]; everything
// below runs on its side I1*J1 instead of J1, and row a2*I1 + rho of the large tensor holds the
// elements T_L[rho*J1 + r', (a2, b2)].
template <int J1, int DD, int I1 = 1>
__global__ __launch_bounds__(64) void decompose_kernel(dq_format fmt, dq_cache cache, CompressJob job,
                                                       float* __restrict__ large_ws,
                                                       int32_t* __restrict__ unit_status) {
  const Geometry g = make_geometry(fmt, cache.kv_heads, cache.block_capacity);
  const int unit = blockIdx.x;
  const UnitRef ur = unit_ref(g, job, unit);
  const int which = ur.which, slot = ur.slot, nv = ur.nv;
  const long bh = ur.bh;
  if (slot < 0) {
    if (threadIdx.x == 0) unit_status[unit] = 0;
    return;
  }
  const int tid = threadIdx.x;
  constexpr int cj1 = J1, d = DD, j2 = DD / J1;   // compile-time shapes: loops unroll, no divisions
  constexpr int j1 = I1 * J1;            // side of the regrouped matrix's row index (a1, b1)
  constexpr int ld = j1 + 1;             // padded leading dimension of the small matrices
  constexpr int nent = j1 * j1;
  const int i2 = g.Tb / I1;              // positions a2 per block
  const uint16_t* X = ur.X;  // [nv, d] fp16 bits

  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  double* A0 = reinterpret_cast<double*>(lds_raw);   // Gram matrix, double buffered
  double* A1 = A0 + j1 * ld;
  double* V0 = A1 + j1 * ld;                         // accumulated rotations, double buffered
  double* V1 = V0 + j1 * ld;
  double* W = V1 + j1 * ld;                          // W[r][b1] = U[b1][order r] / sigma_r
  double* rc = W + j1 * ld;                          // rotation (c, s) per index (both partners)
  double* rs = rc + j1;
  double* lam = rs + j1;
  double* sigma = lam + j1;
  double* offarr = sigma + j1;                       // per rotating lane: largest relative off-diagonal
  int* partner = reinterpret_cast<int*>(offarr + j1);
  int* is_p = partner + j1;                          // 1 if the index is the first member of its pair
  int* order = is_p + j1;
  float* xs = reinterpret_cast<float*>(order + j1 + (j1 & 1));   // [I1][kGramTile][d]

  // ---- Gram matrix: Gm[p][q] = sum_{a2, b2} M[p, (a2, b2)] M[q, (a2, b2)], p = (a1, b1) ----
  // lane (pb, qb) of an 8 x 8 grid owns a (j1/8) x (j1/8) block of entries
  constexpr int BS = j1 / 8;
  const int pb = (tid >> 3) * BS, qb = (tid & 7) * BS;
  double acc[BS][BS];
#pragma unroll
  for (int i = 0; i < BS; ++i)
#pragma unroll
    for (int j = 0; j < BS; ++j) acc[i][j] = 0.0;
  // row p = (a1, b1) of M takes channel b1*j2 + b2 of token group a1's staged row
  int off_p[BS], off_q[BS];
#pragma unroll
  for (int i = 0; i < BS; ++i) {
    off_p[i] = ((pb + i) / cj1) * kGramTile * d + ((pb + i) % cj1) * j2;
    off_q[i] = ((qb + i) / cj1) * kGramTile * d + ((qb + i) % cj1) * j2;
  }
  // (positions past the last valid row of the first token group hold zeros in every group)
  const int np = min(i2, nv);
  for (int t0 = 0; t0 < np; t0 += kGramTile) {
    const int nt = min(kGramTile, np - t0);
    for (int i = tid; i < I1 * nt * d; i += 64) {
      const int a1 = i / (nt * d), rest = i % (nt * d);
      const int row = a1 * i2 + t0 + rest / d;
      xs[a1 * kGramTile * d + rest] = row < nv ? h2f(X[(long)row * d + rest % d]) : 0.f;
    }
    __syncthreads();
    for (int t = 0; t < nt; ++t) {
      const float* xr = xs + t * d;
#pragma unroll
      for (int b2 = 0; b2 < j2; ++b2) {
        double xp[BS], xq[BS];
#pragma unroll
        for (int i = 0; i < BS; ++i) {
          xp[i] = (double)xr[off_p[i] + b2];
          xq[i] = (double)xr[off_q[i] + b2];
        }
        // every product of two fp16 values is exact in fp64; only the sum rounds
#pragma unroll
        for (int i = 0; i < BS; ++i)
#pragma unroll
          for (int j = 0; j < BS; ++j) acc[i][j] = fma(xp[i], xq[j], acc[i][j]);
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < BS; ++i)
#pragma unroll
    for (int j = 0; j < BS; ++j) A0[(pb + i) * ld + qb + j] = acc[i][j];
  for (int idx = tid; idx < nent; idx += 64) V0[(idx / j1) * ld + idx % j1] = (idx / j1 == idx % j1) ? 1.0 : 0.0;
  __syncthreads();

  // ---- parallel cyclic Jacobi: j1-1 rounds of j1/2 disjoint rotations per sweep ----
  double* Ac = A0; double* An = A1; double* Vc = V0; double* Vn = V1;
  const int nm1 = j1 - 1;
  int sweeps = 0;
  for (int sweep = 0; sweep < 16; ++sweep) {
    ++sweeps;
    if (tid < j1) offarr[tid] = 0.0;
    __syncthreads();
    for (int round = 0; round < nm1; ++round) {
      if (tid < j1 / 2) {
        int p, q;
        if (tid == 0) { p = nm1; q = round; }
        else { p = (round + tid) % nm1; q = (round - tid + nm1) % nm1; }
        if (p > q) { const int t = p; p = q; q = t; }
        const double app = Ac[p * ld + p], aqq = Ac[q * ld + q], apq = Ac[p * ld + q];
        double c = 1.0, s = 0.0;
        // skip off-diagonals that are already negligible against the diagonal (also keeps tau finite)
        if (fabs(apq) > 1e-300 && fabs(apq) > 1e-40 * (fabs(app) + fabs(aqq))) {
          const double tau = (aqq - app) * 0.5 * fast_rcp(apq);
          const double w = 1.0 + tau * tau;                       // sqrt(w) = w * rsqrt(w)
          const double t = (tau >= 0.0 ? 1.0 : -1.0) * fast_rcp(fabs(tau) + w * fast_rsqrt(w));
          c = fast_rsqrt(1.0 + t * t);
          s = t * c;
          const double rel2 = apq * apq * fast_rcp(fabs(app * aqq) + 1e-300);   // squared relative size
          if (rel2 > offarr[tid]) offarr[tid] = rel2;
        }
        rc[p] = c; rs[p] = s; rc[q] = c; rs[q] = s;
        partner[p] = q; partner[q] = p;
        is_p[p] = 1; is_p[q] = 0;
      }
      __syncthreads();
      // J has J[p][p] = c, J[p][q] = s, J[q][p] = -s, J[q][q] = c for each pair.
      // A' = J^T A J ; V' = V J.  Entry (i, j) needs A at {i, pi} x {j, pj}.
      for (int idx = tid; idx < nent; idx += 64) {
        const int i = idx / j1, j = idx % j1;
        const int pi = partner[i], pj = partner[j];
        // column j of J: J[j][j] = c_j, J[pj][j] = (is_p[j] ? -s : +s)
        const double cj = rc[j], sj = is_p[j] ? -rs[j] : rs[j];
        const double ci = rc[i], si = is_p[i] ? -rs[i] : rs[i];
        const double aj_i = Ac[i * ld + j] * cj + Ac[i * ld + pj] * sj;     // (A J)[i][j]
        const double aj_pi = Ac[pi * ld + j] * cj + Ac[pi * ld + pj] * sj;  // (A J)[pi][j]
        An[i * ld + j] = ci * aj_i + si * aj_pi;                            // (J^T (A J))[i][j]
        Vn[i * ld + j] = Vc[i * ld + j] * cj + Vc[i * ld + pj] * sj;
      }
      __syncthreads();
      double* t = Ac; Ac = An; An = t;
      t = Vc; Vc = Vn; Vn = t;
    }
    double om = 0.0;
    for (int i = 0; i < j1 / 2; ++i) om = fmax(om, offarr[i]);
    __syncthreads();
    if (om < 1e-24) break;   // every rotated off-diagonal was below 1e-12 of its diagonal pair
  }

  // ---- singular values, ordering, small tensor ----
  if (tid < j1) lam[tid] = Ac[tid * ld + tid];
  __syncthreads();
  if (tid < j1) {
    int rank = 0;
    const double me = lam[tid];
    for (int s = 0; s < j1; ++s) rank += (lam[s] > me) || (lam[s] == me && s < tid);
    order[rank] = tid;
  }
  __syncthreads();
  if (tid < j1) {
    const double lmax = fmax(lam[order[0]], 0.0);
    const double l = lam[order[tid]];
    sigma[tid] = (l > 1e-12 * lmax && l > 0.0) ? sqrt(l) : 0.0;
  }
  __syncthreads();
  {
    const long blk = (long)bh * g.NB + slot;
    uint16_t* small = (which ? cache.v_small : cache.k_small) + blk * g.small_per_block;
    bool sat = false;
    for (int idx = tid; idx < nent; idx += 64) {
      // neighbouring lanes write neighbouring entries of the stored array (keys are stored transposed)
      const int b1 = which ? idx / j1 : idx % j1, r = which ? idx % j1 : idx / j1;
      const double u = Vc[b1 * ld + order[r]];
      const double sg = sigma[r];
      W[r * ld + b1] = sg > 0.0 ? u / sg : 0.0;
      const uint16_t hb = f64_to_f16_rne(u * sg, true, &sat);
      if (which) small[b1 * j1 + r] = hb;   // values: natural [b1][r]
      else small[r * j1 + b1] = hb;         // keys: transposed [r][b1]
    }
    // this block's status word: bit 0 = T_S saturated, bits 8.. = Jacobi sweeps used
    const bool any_sat = __any(sat);
    if (tid == 0) unit_status[unit] = (any_sat ? 1 : 0) | (sweeps << 8);
  }
  __syncthreads();

  // ---- projection: T_L[r, (a2, b2)] = sum_p W[r][p] M[p, (a2, b2)], fp64 -> fp32, to row
  // a2*I1 + r / J1, element (r % J1)*j2 + b2 ----
  float* out = large_ws + (long)unit * g.Tb * d;
  for (int item = tid; item < i2 * j2; item += 64) {
    const int t = item / j2, b2 = item % j2;
    if (t < nv) {
      double xv[j1];
#pragma unroll
      for (int p = 0; p < j1; ++p) {
        const int row = (p / cj1) * i2 + t;
        xv[p] = row < nv ? (double)h2f(X[(long)row * d + (p % cj1) * j2 + b2]) : 0.0;
      }
      for (int r = 0; r < j1; ++r) {
        double a = 0.0;
#pragma unroll
        for (int p = 0; p < j1; ++p) a = fma(W[r * ld + p], xv[p], a);
        out[((long)t * I1 + r / cj1) * d + (r % cj1) * j2 + b2] = (float)a;
      }
    } else {
      for (int r = 0; r < j1; ++r) out[((long)t * I1 + r / cj1) * d + (r % cj1) * j2 + b2] = 0.f;
    }
  }
}

// ------------------------------------------------------------------------------------------
// Fast decomposition for the common shape d = 128, j1 = 16, j2 = 8: one wave per block, the two
// dense contractions (Gram matrix, projection) on the fp64 matrix cores, the Jacobi solver with the
// 16 x 16 matrices cut into 64 blocks of 2 x 2, one per lane.
//
// v_mfma_f64_16x16x4_f64 operand layout (one double per lane for A and B, four for D):
//   A[m][k]: lane l -> m = l % 16, k = l / 16;  B[k][n]: lane l -> n = l % 16, k = l / 16;
//   D[m][n]: lane l, register i -> n = l % 16, m = l / 16 + 4 i.
// ------------------------------------------------------------------------------------------
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// Rotation (c, s) that annihilates entry (p, q) of a symmetric matrix; `big` reports whether that
// entry was still above kSettled relative to its diagonal pair.  The angle comes from the hardware
// estimates alone (relative error near 1e-7: the entry shrinks by that factor instead of
// vanishing, which does not slow the quadratic convergence); c is refined to full precision so
// that c^2 + s^2 = 1 and the accumulated rotations stay orthogonal.
constexpr double kSettled2 = 1e-9;   // (3e-5)^2: one more sweep squares 3e-5 to about 1e-9

__device__ __forceinline__ void jacobi_rotation(double app, double aqq, double apq, double floor_abs,
                                                double& c, double& s, bool& big) {
  // Entries at the rounding level of the whole matrix (floor_abs = 1e-17 * trace) or negligible
  // against their own diagonal pair are skipped: rotating them changes nothing that is kept, and
  // between two numerically zero eigenvalues they would never settle.  Written without branches.
  const bool live = fabs(apq) > floor_abs && fabs(apq) > 1e-40 * (fabs(app) + fabs(aqq));
  const double tau = (aqq - app) * 0.5 * __builtin_amdgcn_rcp(apq);
  const double root = __builtin_amdgcn_sqrt(fma(tau, tau, 1.0));
  const double t = copysign(__builtin_amdgcn_rcp(fabs(tau) + root), tau);
  const double cc = fast_rsqrt(fma(t, t, 1.0));
  c = live ? cc : 1.0;
  s = live ? t * cc : 0.0;
  big = live && apq * apq > kSettled2 * fabs(app * aqq);
}

// Pair `k` (0..7) of round `round` (0..14) of the round-robin schedule over 16 indices.
__device__ __forceinline__ void pair16(int round, int k, int& p, int& q) {
  if (k == 0) { p = 15; q = round; return; }
  p = round + k; if (p >= 15) p -= 15;
  q = round - k; if (q < 0) q += 15;
}

// NWV waves per block: the two contractions are split over the waves by token, the eigen-solver
// runs in one of them.  The host picks NWV so that the launch has about one wave per SIMD.
// PAIR: heads of 64 channels with j1 = 8.  The same block (keys or values, same sequence and block
// position) of two neighbouring kv heads is worked as one block of 128 channels: the two 8 x T_b*8
// regrouped matrices on top of each other.  The 16 x 16 Gram matrix then holds the heads' own 8 x 8
// Gram matrices on its diagonal; the blocks off the diagonal (products across heads) are set to
// zero, after which every rotation between the two halves is the identity and the iteration solves
// the two 8 x 8 problems side by side (the rotations, their order and the stopping rule are those of
// the 16 x 16 case).  Ordering, small tensors, projection and outputs are per head.
// QB, FULL: QB != 0 quantizes the large tensor here, straight from the projection's registers, to
// QB-bit codes (FULL: all 2^QB of them) and writes codes and steps into the cache; the fp32 rows do
// not go to the workspace then and no quantizer launch follows (d = 128, one or two step groups per
// row).  QB == 0 leaves the fp32 rows in the workspace for quantize_tiles_kernel.
// Then the kernel also ends the call: the last workgroup to finish (a ticket counter in the third
// word of the workspace header, zero between calls) folds the blocks' status words into the call's
// two; status words travel as device-scope stores and loads, as the counter does, so no cache
// write-back or invalidation is needed between the XCDs.
// LEAN: the build for calls of thousands of blocks (a prompt), which are bound by throughput, not by
// one block's latency: one wave per block, several blocks resident per SIMD so that one block's
// eigen-solver (a chain of dependent instructions) overlaps the other blocks' contractions.  For
// that the wave keeps fewer registers (loads in smaller batches, the solver's rounds not unrolled) and
// less LDS (the quantizer works on 64 rows at a time in the space the solver's matrices leave).  The
// arithmetic, and so every bit written, is that of the other builds.
// N3 (lean build with the quantizer, d = 128): three local tensors (Eq. 2 with n = 3, factor shapes
// 1 * (T_b/8) * 8 by j1 * j2 * 1) in the same kernel.  The first cut's right factor R is never
// stored: a first pass over the rows forms it 16 tokens at a time (rounded to fp32, the precision
// the three-kernel path keeps it in) and adds it to the 8 x 8 Gram matrix of the second cut,
// A^T A with A[(r, a2, b2), a3]; the same wave solves that 8 x 8 problem and writes T_3; a second
// pass forms R again, this time with the tokens down the rows of the matrix-core result, which is
// the operand layout that lets a second matrix product contract over the eight tokens of a run
// (T_2 = A V' diag(1/sigma')), and hands the rows of T_2 to the quantizer in the registers it
// expects them in.  job.keep_large: the fp32 rows of T_2 also go to the workspace.
template <int NWV, bool PAIR, int QB = 0, bool FULL = false, bool LEAN = false, bool N3 = false>
__global__ __launch_bounds__(64 * NWV, LEAN ? ((PAIR || N3) ? 3 : 4) : 1) void decompose16_kernel(dq_format fmt, dq_cache cache, CompressJob job,
                                                               float* __restrict__ large_ws,
                                                               int32_t* __restrict__ unit_status,
                                                               int32_t* __restrict__ call_status) {
  __shared__ int s_last_block;
  auto end_call = [&]() __attribute__((always_inline)) {   // QB != 0 only; every workgroup, once, at its end
    // every wave waits for its own device-scope stores (the status words) to be acknowledged; after
    // the barrier all of the workgroup's have been, and only then is the ticket taken
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (threadIdx.x == 0) {
      const int ticket = __hip_atomic_fetch_add(call_status + 2, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_last_block = (ticket == (int)gridDim.x - 1);
      if (s_last_block) __hip_atomic_store(call_status + 2, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!s_last_block || threadIdx.x >= 64) return;
    int flags = 0, sweeps = 0;
    const int n_units = (PAIR ? 2 : 1) * (int)gridDim.x;
    for (int u = threadIdx.x; u < n_units; u += 64) {
      const int w = __hip_atomic_load(unit_status + u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      flags |= w & 0xFF;
      sweeps = max(sweeps, w >> 8);
    }
    for (int o = 32; o > 0; o >>= 1) {
      flags |= __shfl_xor(flags, o);
      sweeps = max(sweeps, __shfl_xor(sweeps, o));
    }
    if (threadIdx.x == 0) { call_status[0] = flags; call_status[1] = sweeps; }
  };
  const Geometry g = make_geometry(fmt, cache.kv_heads, cache.block_capacity);
  // the work unit (of the pair's first head); the second head's unit lies `unit_gap` further on
  int unit = blockIdx.x;
  const int unit_gap = 2 * job.n_blocks;
  if (PAIR) {
    const int pb = blockIdx.x >> 1, j = pb % job.n_blocks, hp = pb / job.n_blocks;   // hp = b * (H/2) + head pair
    const int half_h = g.H >> 1;
    unit = (((hp / half_h) * g.H + 2 * (hp % half_h)) * job.n_blocks + j) * 2 + (blockIdx.x & 1);
  }
  const UnitRef ur = unit_ref(g, job, unit);
  const int which = ur.which, slot = ur.slot, nv = ur.nv;
  const long bh = ur.bh;
  if (slot < 0) {
    if (threadIdx.x == 0) {
      if (QB != 0) {
        __hip_atomic_store(unit_status + unit, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (PAIR) __hip_atomic_store(unit_status + unit + unit_gap, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      } else {
        unit_status[unit] = 0;
        if (PAIR) unit_status[unit + unit_gap] = 0;
      }
    }
    if constexpr (QB != 0) end_call();
    return;
  }
  const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int solver = blockIdx.x % NWV;   // the wave that runs the eigen-solver (spread over the SIMDs)
  constexpr int j1 = 16, ld = 17;
  constexpr int d = PAIR ? 64 : 128;     // halves per row in memory
  const uint16_t* X = ur.X;  // [nv, d] fp16 bits
  const long head_gap = (long)job.t_new * d;   // PAIR: from a row of the first head to the same row of the second

  static_assert(!LEAN || NWV == 1, "the lean build is one wave per block");
  static_assert(!N3 || (LEAN && !PAIR && QB != 0), "three tensors: lean build with the quantizer, d = 128");
  constexpr int kMat = j1 * ld;                              // doubles per 16 x 16 matrix (padded rows)
  constexpr int kMatBytes = (3 + (NWV > 1 ? NWV - 1 : 1)) * kMat * (int)sizeof(double);
  // fused quantizer: one byte per element of QT token rows, then the value layout's staging
  // (a pair: one such area per head, of 64 channels each)
  constexpr int QT = LEAN ? 32 : kTileTokens;                // rows quantized and packed at a time
  constexpr int kHeadArea = QT * d + d * (pack_parts(QB ? QB : 8, QT) * QT * (QB ? QB : 8) / 32 + 1) * 4;
  constexpr int kFieldBytes = QB ? (PAIR ? 2 : 1) * kHeadArea : 16;
  // the lean build's fields take the place of the matrices, which are dead by then (one wave: its
  // LDS operations execute in program order)
  constexpr int kPoolBytes = LEAN ? (kMatBytes > kFieldBytes ? kMatBytes : kFieldBytes) : kMatBytes + kFieldBytes;
  __shared__ __attribute__((aligned(16))) unsigned char pool[kPoolBytes];
  double* const A = reinterpret_cast<double*>(pool);
  double* const V = A + kMat;
  double* const W = V + kMat;
  double* const P = W + kMat;                                // Gram partials of the other waves
  uint8_t* const lds_u = LEAN ? pool : pool + kMatBytes;
  __shared__ double lam[j1], sigma[j1];
  __shared__ int order[j1];

  // ---- Gram matrix G[p][q] = sum_{t, b2} X[t, p*8+b2] X[t, q*8+b2] ----
  // A and B operand of one MFMA are the same register: lane (b1 = l%16, k = l/16) holds
  // X[t0 + k][b1*8 + b2] for the 4 tokens of a group and one b2.  A lane loads the 8 b2 of its
  // (token, b1) as one 16-byte chunk; 16 lanes cover a 256-byte row.  Wave wv takes every NWV-th
  // group of 4 tokens.
  {
    const int b1 = l & 15, tk = l >> 4;
    constexpr int NG = 32 / NWV;   // groups per wave in a chunk of 128 tokens
    f64x4 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = f64x4{0.0, 0.0, 0.0, 0.0};
    constexpr int GC = LEAN ? 8 : NG;   // groups requested together (the same order of products either way)
    for (int t0 = 0; t0 < nv; t0 += 128) {
#pragma unroll 1
      for (int u0 = 0; u0 < NG; u0 += GC) {
        u32x4 x[GC];
#pragma unroll
        for (int u = 0; u < GC; ++u) {
          const int t = t0 + 4 * ((u0 + u) * NWV + wv) + tk;
          x[u] = u32x4{0u, 0u, 0u, 0u};
          if (t < nv)
            x[u] = *reinterpret_cast<const u32x4*>(PAIR ? X + (b1 >> 3) * head_gap + (long)t * d + (b1 & 7) * 8
                                                        : X + (long)t * d + b1 * 8);
        }
#pragma unroll
        for (int u = 0; u < GC; ++u) {
          const f16x8 h = __builtin_bit_cast(f16x8, x[u]);
#pragma unroll
          for (int b2 = 0; b2 < 8; ++b2) {
            const double a = (double)(float)h[b2];
            acc[b2 & 3] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, a, acc[b2 & 3], 0, 0, 0);
          }
        }
      }
    }
    double* dst = wv == 0 ? A : P + (wv - 1) * j1 * ld;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (l >> 4) + 4 * i, col = l & 15;
      const double sum = (acc[0][i] + acc[1][i]) + (acc[2][i] + acc[3][i]);
      dst[row * ld + col] = (PAIR && (row >> 3) != (col >> 3)) ? 0.0 : sum;   // no products across heads
    }
    for (int idx = threadIdx.x; idx < j1 * j1; idx += 64 * NWV)
      V[(idx >> 4) * ld + (idx & 15)] = ((idx >> 4) == (idx & 15)) ? 1.0 : 0.0;
  }
  __syncthreads();
  if (NWV > 1) {
    for (int idx = threadIdx.x; idx < j1 * j1; idx += 64 * NWV) {
      const int e = (idx >> 4) * ld + (idx & 15);
      double sum = A[e];
#pragma unroll
      for (int k = 0; k < NWV - 1; ++k) sum += P[k * j1 * ld + e];   // fixed order: reproducible
      A[e] = sum;
    }
    __syncthreads();
  }

  if (wv == solver) {
    // ---- parallel cyclic Jacobi: 15 rounds of 8 disjoint rotations per sweep ----
    // Lane (I, J) owns the 2 x 2 block rows(pair I) x columns(pair J) of the matrix and rows
    // {2I, 2I+1} x columns(pair J) of the accumulated rotations; it derives the rotation of pair I
    // from that pair's three entries and takes the one of pair J from lane (J, I).
    const int I = l >> 3, J = l & 7;
    // (a pair: each head's entries are measured against its own trace)
    double trace_lo = 0.0, trace_hi = 0.0;
#pragma unroll
    for (int i = 0; i < j1 / 2; ++i) { trace_lo += A[i * ld + i]; trace_hi += A[(i + 8) * ld + i + 8]; }
    const double floor_lo = fmax((PAIR ? trace_lo : trace_lo + trace_hi) * 1e-17, 1e-300);
    const double floor_hi = PAIR ? fmax(trace_hi * 1e-17, 1e-300) : floor_lo;
    int sweeps = 0;
    for (int sweep = 0; sweep < 16; ++sweep) {
      ++sweeps;
      bool unsettled = false;
      auto one_round = [&](const int round) __attribute__((always_inline)) {
        int p, q, u, v;
        pair16(round, I, p, q);
        pair16(round, J, u, v);
        const double app = A[p * ld + p], aqq = A[q * ld + q], apq = A[p * ld + q];
        const double b00 = A[p * ld + u], b01 = A[p * ld + v], b10 = A[q * ld + u], b11 = A[q * ld + v];
        const int r0 = 2 * I * ld, r1 = r0 + ld;
        const double v00 = V[r0 + u], v01 = V[r0 + v], v10 = V[r1 + u], v11 = V[r1 + v];
        // the rotation of the row pair is computed here; that of the column pair J is the row-pair
        // rotation of the transposed lane (J, I)
        double cI, sI;
        bool big;
        jacobi_rotation(app, aqq, apq, (PAIR && (p >> 3)) ? floor_hi : floor_lo, cI, sI, big);
        const double cJ = __shfl(cI, 8 * J + I), sJ = __shfl(sI, 8 * J + I);
        unsettled |= big;
        // Jm has Jm[p][p] = c, Jm[p][q] = s, Jm[q][p] = -s, Jm[q][q] = c;  A' = Jm^T A Jm,  V' = V Jm
        const double x00 = b00 * cJ - b01 * sJ, x01 = b00 * sJ + b01 * cJ;
        const double x10 = b10 * cJ - b11 * sJ, x11 = b10 * sJ + b11 * cJ;
        A[p * ld + u] = cI * x00 - sI * x10;
        A[p * ld + v] = cI * x01 - sI * x11;
        A[q * ld + u] = sI * x00 + cI * x10;
        A[q * ld + v] = sI * x01 + cI * x11;
        V[r0 + u] = v00 * cJ - v01 * sJ;
        V[r0 + v] = v00 * sJ + v01 * cJ;
        V[r1 + u] = v10 * cJ - v11 * sJ;
        V[r1 + v] = v10 * sJ + v11 * cJ;
        // One wave: its LDS operations execute in program order, so the next round's reads see these
        // writes without waiting for them; the compiler only has to keep the order.
        __builtin_amdgcn_wave_barrier();
      };
      if constexpr (LEAN) {
        // (the round number stays a run-time value: fifteen rounds' worth of addresses would cost
        // the registers that let several blocks share a SIMD)
#pragma unroll 1
        for (int round = 0; round < 15; ++round) one_round(round);
      } else {
        // unrolled: the LDS addresses of a round depend only on the lane and are computed once
#pragma unroll
        for (int round = 0; round < 15; ++round) one_round(round);
      }
      // every entry rotated in this sweep was below 3e-5 of its diagonal pair, so the sweep (one
      // more quadratic step) has left them near 1e-9, two orders under the fp32 rounding of T_L
      if (!__any(unsettled)) break;
    }

    // ---- singular values, ordering, small tensor ----
    if (l < j1) lam[l] = A[l * ld + l];
    __builtin_amdgcn_wave_barrier();
    if (l < j1) {
      // (a pair: every head's eigenvalues are ranked among themselves and stay in its half)
      int rank = 0;
      const double me = lam[l];
      for (int s = 0; s < j1; ++s)
        rank += (!PAIR || (s >> 3) == (l >> 3)) && ((lam[s] > me) || (lam[s] == me && s < l));
      order[(PAIR ? (l & 8) : 0) + rank] = l;
    }
    __builtin_amdgcn_wave_barrier();
    if (l < j1) {
      const double lmax = fmax(lam[order[PAIR ? (l & 8) : 0]], 0.0);
      const double lv = lam[order[l]];
      sigma[l] = (lv > 1e-12 * lmax && lv > 0.0) ? sqrt(lv) : 0.0;
    }
    __builtin_amdgcn_wave_barrier();
    const long blk = (long)bh * g.NB + slot;
    uint16_t* small = (which ? cache.v_small : cache.k_small) + blk * g.small_per_block;
    bool sat = false;
    for (int idx = l; idx < j1 * j1; idx += 64) {
      // neighbouring lanes write neighbouring entries of the stored array (keys are stored transposed)
      const int b1 = which ? idx >> 4 : idx & 15, r = which ? idx & 15 : idx >> 4;
      const double uv = V[b1 * ld + order[r]];
      const double sg = sigma[r];
      W[r * ld + b1] = sg > 0.0 ? uv / sg : 0.0;
      if (PAIR) {
        // the heads' 8 x 8 small tensors are the diagonal blocks (the second head's blocks lie NB
        // blocks further on in the cache); the entries off the diagonal are zero and go nowhere
        if ((b1 >> 3) == (r >> 3)) {
          const uint16_t hb = f64_to_f16_rne(uv * sg, true, &sat);
          uint16_t* sm = small + (long)(b1 >> 3) * g.NB * g.small_per_block;
          if (which) sm[(b1 & 7) * 8 + (r & 7)] = hb;
          else sm[(r & 7) * 8 + (b1 & 7)] = hb;
        }
      } else {
        const uint16_t hb = f64_to_f16_rne(uv * sg, true, &sat);
        if (which) small[b1 * j1 + r] = hb;   // values: natural [b1][r]
        else small[r * j1 + b1] = hb;         // keys: transposed [r][b1]
      }
    }
    // this block's status word: bit 0 = T_S saturated, bits 8.. = Jacobi sweeps used
    const bool any_sat = __any(sat);
    if (l == 0) {
      const int word = (any_sat ? 1 : 0) | (sweeps << 8);
      // (a pair: one word for both heads)
      if (QB != 0) {
        __hip_atomic_store(unit_status + unit, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (PAIR) __hip_atomic_store(unit_status + unit + unit_gap, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      } else {
        unit_status[unit] = word;
        if (PAIR) unit_status[unit + unit_gap] = word;
      }
    }
  }
  __syncthreads();

  // ---- projection: K'[t, r*8+b2] = sum_b1 W[r][b1] X[t, b1*8+b2], fp64 -> fp32 ----
  // One MFMA chain per b2: rows r, columns 16 tokens, contraction over b1 in 4 steps of 4.
  // Wave wv takes every NWV-th group of 16 tokens.
  {
    constexpr int NT = QT / 16 / NWV;   // token groups per wave in a chunk of QT tokens
    constexpr int TB = LEAN ? 1 : NT;   // groups whose rows are requested together
    double wreg[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) wreg[s] = W[(l & 15) * ld + 4 * s + (l >> 4)];
    if (LEAN) __builtin_amdgcn_wave_barrier();   // W is read; the fields may take the matrices' place
    double w3reg[4] = {0.0, 0.0, 0.0, 0.0};
    if constexpr (N3) {
      // ---- second cut: Gram matrix of A[(r, a2, b2), a3] from the right factor, 16 tokens at a time ----
      constexpr int N = kRun, LD3 = N + 1;
      double* const Dm = reinterpret_cast<double*>(pool);        // 16 x 16 token products, padded rows
      double* A0 = Dm + kMat;
      double* A1 = A0 + N * LD3;
      double* V0 = A1 + N * LD3;
      double* V1 = V0 + N * LD3;
      double* const W3 = V1 + N * LD3;                           // [e][a3] = V'[a3, e] / sigma'_e
      double* const rc = W3 + N * N;
      double* const rs = rc + N;
      double* const lam3 = rs + N;
      double* const sigma3 = lam3 + N;
      int* const partner = reinterpret_cast<int*>(sigma3 + N);
      int* const is_p = partner + N;
      int* const order3 = is_p + N;
      static_assert((kMat + 4 * N * LD3 + N * N + 4 * N) * (int)sizeof(double) + 3 * N * (int)sizeof(int) <= kPoolBytes,
                    "the second cut's matrices fit the pool");
      f64x4 g3[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) g3[i] = f64x4{0.0, 0.0, 0.0, 0.0};
#pragma unroll 1
      for (int t0 = 0; t0 < nv; t0 += 16) {
        const int t = t0 + (l & 15);
        u32x4 x[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          x[s] = u32x4{0u, 0u, 0u, 0u};
          if (t < nv) x[s] = *reinterpret_cast<const u32x4*>(X + (long)t * d + (4 * s + (l >> 4)) * 8);
        }
        f64x4 acc[8];
#pragma unroll
        for (int b2 = 0; b2 < 8; ++b2) acc[b2] = f64x4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const f16x8 h = __builtin_bit_cast(f16x8, x[s]);
#pragma unroll
          for (int b2 = 0; b2 < 8; ++b2)
            acc[b2] = __builtin_amdgcn_mfma_f64_16x16x4f64(wreg[s], (double)(float)h[b2], acc[b2], 0, 0, 0);
        }
        // lane (token l % 16, k = l / 16) holds R[r = k + 4 i][token][b2]: both operands of a product
        // of the 16 tokens with themselves over four r; the runs' own 8 x 8 blocks are kept below
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int b2 = 0; b2 < 8; ++b2) {
            const double v = (double)(float)acc[b2][i];
            g3[b2 & 3] = __builtin_amdgcn_mfma_f64_16x16x4f64(v, v, g3[b2 & 3], 0, 0, 0);
          }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
        Dm[((l >> 4) + 4 * i) * ld + (l & 15)] = (g3[0][i] + g3[1][i]) + (g3[2][i] + g3[3][i]);
      __builtin_amdgcn_wave_barrier();
      {
        const int p = l >> 3, q = l & 7;
        A0[p * LD3 + q] = Dm[p * ld + q] + Dm[(p + 8) * ld + q + 8];
        V0[p * LD3 + q] = (p == q) ? 1.0 : 0.0;
      }
      __builtin_amdgcn_wave_barrier();
      double trace3 = 0.0;
#pragma unroll
      for (int i = 0; i < N; ++i) trace3 += A0[i * LD3 + i];
      const double floor3 = 1e-17 * trace3;
      // parallel cyclic Jacobi: 7 rounds of 4 disjoint rotations per sweep (the iteration of the
      // three-kernel path's second cut, in this one wave)
      double* Ac = A0; double* An = A1; double* Vc = V0; double* Vn = V1;
      constexpr int NM1 = N - 1;
      for (int sweep = 0; sweep < 16; ++sweep) {
        bool any_big = false;
#pragma unroll 1
        for (int round = 0; round < NM1; ++round) {
          bool big = false;
          if (l < N / 2) {
            int p, q;
            if (l == 0) { p = NM1; q = round; }
            else { p = (round + l) % NM1; q = (round - l + NM1) % NM1; }
            if (p > q) { const int tmp = p; p = q; q = tmp; }
            double c, sn;
            jacobi_rotation(Ac[p * LD3 + p], Ac[q * LD3 + q], Ac[p * LD3 + q], floor3, c, sn, big);
            rc[p] = c; rs[p] = sn; rc[q] = c; rs[q] = sn;
            partner[p] = q; partner[q] = p;
            is_p[p] = 1; is_p[q] = 0;
          }
          any_big = any_big || __any(big);
          __builtin_amdgcn_wave_barrier();
          {
            const int i = l >> 3, j = l & 7;
            const int pi = partner[i], pj = partner[j];
            const double cj = rc[j], sj = is_p[j] ? -rs[j] : rs[j];
            const double ci = rc[i], si = is_p[i] ? -rs[i] : rs[i];
            const double aj_i = Ac[i * LD3 + j] * cj + Ac[i * LD3 + pj] * sj;
            const double aj_pi = Ac[pi * LD3 + j] * cj + Ac[pi * LD3 + pj] * sj;
            An[i * LD3 + j] = ci * aj_i + si * aj_pi;
            Vn[i * LD3 + j] = Vc[i * LD3 + j] * cj + Vc[i * LD3 + pj] * sj;
          }
          __builtin_amdgcn_wave_barrier();
          double* tp = Ac; Ac = An; An = tp;
          tp = Vc; Vc = Vn; Vn = tp;
        }
        if (!any_big) break;
      }
      if (l < N) lam3[l] = Ac[l * LD3 + l];
      __builtin_amdgcn_wave_barrier();
      if (l < N) {
        int rank = 0;
        const double me = lam3[l];
        for (int s2 = 0; s2 < N; ++s2) rank += (lam3[s2] > me) || (lam3[s2] == me && s2 < l);
        order3[rank] = l;
      }
      __builtin_amdgcn_wave_barrier();
      if (l < N) {
        const double lmax = fmax(lam3[order3[0]], 0.0);
        const double lv = lam3[order3[l]];
        sigma3[l] = (lv > 1e-12 * lmax && lv > 0.0) ? sqrt(lv) : 0.0;
      }
      __builtin_amdgcn_wave_barrier();
      {
        const int e = l >> 3, a3 = l & 7;
        const double v = Vc[a3 * LD3 + order3[e]];
        const double sg = sigma3[e];
        W3[e * N + a3] = sg > 0.0 ? v / sg : 0.0;
        const long b3 = ((long)bh * g.NB + slot) * (N * N);
        const uint16_t hb = f64_to_f16_rne(v * sg, true, nullptr);   // |T_3| <= sqrt(j1): far inside fp16
        if (which) cache.v_small3[b3 + e * N + a3] = hb;   // values: natural [e][a3]
        else cache.k_small3[b3 + a3 * N + e] = hb;         // keys: transposed [a3][e]
      }
      __builtin_amdgcn_wave_barrier();
      // the token mix as the right-hand operand of a product over four tokens (k = l / 16, token
      // k + 4 i of the group): column n = l % 16 is row e = n % 8 of run n / 8; a token of the other
      // run contributes nothing
#pragma unroll
      for (int i = 0; i < 4; ++i)
        w3reg[i] = ((i >> 1) == ((l & 15) >> 3)) ? W3[(l & 7) * N + (((l >> 4) + 4 * i) & 7)] : 0.0;
      __builtin_amdgcn_wave_barrier();   // W3 is read; the fields may take the pool
    }
    float* out = large_ws + (long)unit * g.Tb * d;
    const long out_gap = (long)unit_gap * g.Tb * d;   // PAIR: to the second head's rows in the workspace
    for (int t0 = 0; t0 < g.Tb; t0 += QT) {
#pragma unroll 1
     for (int tg0 = 0; tg0 < NT; tg0 += TB) {
      u32x4 x[TB][4];
#pragma unroll
      for (int tgi = 0; tgi < TB; ++tgi) {
        const int t = t0 + 16 * ((tg0 + tgi) * NWV + wv) + (l & 15);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          x[tgi][s] = u32x4{0u, 0u, 0u, 0u};
          // b1 = 4 s + l / 16 (a pair: row b1 % 8 of head b1 / 8 = s / 2)
          if (t < nv)
            x[tgi][s] = *reinterpret_cast<const u32x4*>(PAIR ? X + (s >> 1) * head_gap + (long)t * d + ((4 * s + (l >> 4)) & 7) * 8
                                                             : X + (long)t * d + (4 * s + (l >> 4)) * 8);
        }
      }
#pragma unroll
      for (int tgi = 0; tgi < TB; ++tgi) {
        const int tg = tg0 + tgi;
        const int t = t0 + 16 * (tg * NWV + wv) + (l & 15);
        f64x4 acc[8];
#pragma unroll
        for (int b2 = 0; b2 < 8; ++b2) acc[b2] = f64x4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const f16x8 h = __builtin_bit_cast(f16x8, x[tgi][s]);
#pragma unroll
          for (int b2 = 0; b2 < 8; ++b2) {
            // (three tensors: operands swapped, so that the result has the 16 tokens down its rows)
            if (N3) acc[b2] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)(float)h[b2], wreg[s], acc[b2], 0, 0, 0);
            else acc[b2] = __builtin_amdgcn_mfma_f64_16x16x4f64(wreg[s], (double)(float)h[b2], acc[b2], 0, 0, 0);
          }
        }
        if constexpr (N3) {
          // lane (r = l % 16, k = l / 16) holds R[r][token k + 4 i][b2], rounded to fp32 as in the first
          // pass: left operand of the product over the tokens; the result has rows r = l / 16 + 4 i and
          // columns (run, e), which is where the quantizer below expects a row of the large tensor
#pragma unroll
          for (int b2 = 0; b2 < 8; ++b2) {
            f64x4 o = f64x4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int i = 0; i < 4; ++i)
              o = __builtin_amdgcn_mfma_f64_16x16x4f64((double)(float)acc[b2][i], w3reg[i], o, 0, 0, 0);
            acc[b2] = o;
          }
        }
        if constexpr (QB == 0) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            // row r = l / 16 + 4 i of the large tensor (a pair: row r % 8 of head r / 8 = i / 2)
            float* dst = PAIR ? out + (i >> 1) * out_gap + (long)t * d + (((l >> 4) + 4 * i) & 7) * 8
                              : out + (long)t * d + ((l >> 4) + 4 * i) * 8;
            *reinterpret_cast<float4*>(dst) = make_float4((float)acc[0][i], (float)acc[1][i], (float)acc[2][i], (float)acc[3][i]);
            *reinterpret_cast<float4*>(dst + 4) = make_float4((float)acc[4][i], (float)acc[5][i], (float)acc[6][i], (float)acc[7][i]);
          }
        } else {
          // ---- Eq. 1 on the token's row, from the registers: the lane holds rows r = l / 16 + 4 i
          // (i = 0..3) of token t, eight b2 each; the token's other rows sit in the lanes 16, 32 and
          // 48 further on.  Step groups: the whole row, or rows r < 8 (i < 2) and r >= 8.
          constexpr int QMAX = (1 << (QB - 1)) - 1;
          float f[4][8];
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int b2 = 0; b2 < 8; ++b2) f[i][b2] = (float)acc[b2][i];
          if (N3 && job.keep_large) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              float* dst = out + (long)t * d + ((l >> 4) + 4 * i) * 8;
              *reinterpret_cast<float4*>(dst) = make_float4(f[i][0], f[i][1], f[i][2], f[i][3]);
              *reinterpret_cast<float4*>(dst + 4) = make_float4(f[i][4], f[i][5], f[i][6], f[i][7]);
            }
          }
          float up[2] = {0.f, 0.f}, dn[2] = {0.f, 0.f};   // max |x| (FULL: max x and max -x) per group
#pragma unroll
          for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int b2 = 0; b2 < 8; ++b2) {
              if (FULL) {
                up[i >> 1] = fmaxf(up[i >> 1], f[i][b2]);
                dn[i >> 1] = fmaxf(dn[i >> 1], -f[i][b2]);
              } else {
                up[i >> 1] = fmaxf(up[i >> 1], fabsf(f[i][b2]));
              }
            }
          }
          if (!PAIR && g.groups == 1) {   // (a pair: group i / 2 is head i / 2's row, its only group)
            up[0] = up[1] = fmaxf(up[0], up[1]);
            dn[0] = dn[1] = fmaxf(dn[0], dn[1]);
          }
          uint16_t sb[2];
          float step[2], inv[2];
#pragma unroll
          for (int gi = 0; gi < 2; ++gi) {
            up[gi] = fmaxf(up[gi], __shfl_xor(up[gi], 16));
            up[gi] = fmaxf(up[gi], __shfl_xor(up[gi], 32));
            sb[gi] = group_step_bits<QMAX>(up[gi]);
            if (FULL) {
              dn[gi] = fmaxf(dn[gi], __shfl_xor(dn[gi], 16));
              dn[gi] = fmaxf(dn[gi], __shfl_xor(dn[gi], 32));
              const uint16_t down = f2h_rne(dn[gi] * (1.0f / (float)(QMAX + 1)));
              sb[gi] = sb[gi] > down ? sb[gi] : down;
            }
            step[gi] = h2f(sb[gi]);
            inv[gi] = step[gi] > 0.f ? __builtin_amdgcn_rcpf(step[gi]) : 0.f;
          }
          const int tl = 16 * (tg * NWV + wv) + (l & 15);   // the token's row among the QT rows in LDS
          if ((l >> 4) == 0) {
            uint16_t* sc = (which ? cache.v_scales : cache.k_scales) + ((long)bh * g.NB + slot) * g.scales_per_block +
                           (long)(t0 + tl) * g.groups;
            sc[0] = sb[0];
            if (PAIR) sc[(long)g.NB * g.scales_per_block] = sb[1];   // the second head's block, NB blocks further on
            else if (g.groups == 2) sc[1] = sb[1];
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            uint2 w;
            w.x = fields_of_four<QB, FULL>(f[i][0], f[i][1], f[i][2], f[i][3], step[i >> 1], inv[i >> 1]);
            w.y = fields_of_four<QB, FULL>(f[i][4], f[i][5], f[i][6], f[i][7], step[i >> 1], inv[i >> 1]);
            uint8_t* dst = PAIR ? lds_u + (i >> 1) * kHeadArea + tl * d + (((l >> 4) + 4 * i) & 7) * 8
                                : lds_u + tl * d + ((l >> 4) + 4 * i) * 8;
            *reinterpret_cast<uint2*>(dst) = w;
          }
        }
      }
     }
      if constexpr (QB != 0) {
        // every wave has left the fields of its tokens: pack these rows of the tile and send them off
        __syncthreads();
        uint8_t* codes = (which ? cache.v_codes : cache.k_codes) + ((long)bh * g.NB + slot) * g.codes_per_block +
                         (long)(t0 & ~(kTileTokens - 1)) * g.row_bytes;
        const int part = (t0 & (kTileTokens - 1)) / QT;
        if (PAIR) {
          pack_fields<QB, d, 64 * NWV, QT>(lds_u, 8, 8, which, codes, part);
          pack_fields<QB, d, 64 * NWV, QT>(lds_u + kHeadArea, 8, 8, which, codes + (long)g.NB * g.codes_per_block, part);
        } else {
          pack_fields<QB, d, 64 * NWV, QT>(lds_u, 16, 8, which, codes, part);
        }
      }
    }
  }
  if constexpr (QB != 0) end_call();
}

// ------------------------------------------------------------------------------------------
// Second cut of the three-tensor form (Eq. 2 with n = 3; factor shapes 1 * (T_b/8) * 8 by
// j1 * j2 * 1).  The first cut left its right factor R[(a2, a3), c'] (orthonormal over r) as fp32
// rows in the workspace.  Regrouped as A[(a2, c'), a3] it is cut again,
//   A = T_2 diag(sigma') V'^T,   T_3[e, a3] = sigma'_e V'[a3, e],   T_2 = A V' diag(1/sigma'),
// through the 8 x 8 Gram matrix A^T A (fp64; the fp32 inputs make every product exact), the same
// Jacobi iteration as the first cut, and a projection that overwrites the eight rows of every run
// a2 in place: row a2*8 + e becomes T_2[., a2, ., e].  One workgroup of four waves per block.
// ------------------------------------------------------------------------------------------
template <int DD>
__global__ __launch_bounds__(256) void split3_kernel(dq_format fmt, dq_cache cache, CompressJob job,
                                                     float* __restrict__ large_ws) {
  constexpr int N = kRun, LD = N + 1;
  const Geometry g = make_geometry(fmt, cache.kv_heads, cache.block_capacity);
  const int unit = blockIdx.x;
  const UnitRef ur = unit_ref(g, job, unit);
  const int which = ur.which, slot = ur.slot;
  const long bh = ur.bh;
  if (slot < 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float* blk = large_ws + (long)unit * g.Tb * DD;
  const int runs = g.Tb / N;

  __shared__ double gpart[4][16 * 16];
  __shared__ double A0[N * LD], A1[N * LD], V0[N * LD], V1[N * LD], W3[N * N];
  __shared__ double rc[N], rs[N], lam[N], sigma[N];
  __shared__ int partner[N], is_p[N], order[N];

  // ---- Gram matrix on the fp64 matrix cores: a 16 x 16 product of two runs side by side, whose
  // two diagonal 8 x 8 blocks are the runs' contributions.  Lane (n, k): row a2 = 2*pair + n/8,
  // token a3 = n % 8, elements c' = 16*S + 4*k + j for the j-th of four successive products.
  {
    const int n = lane & 15, k = lane >> 4;
    f64x4 acc = {0.0, 0.0, 0.0, 0.0};
    for (int pair = wave; pair < runs / 2; pair += 4) {
      const float* row = blk + (long)((2 * pair + (n >> 3)) * N + (n & 7)) * DD + 4 * k;
      float4 v[DD / 16];
#pragma unroll
      for (int S = 0; S < DD / 16; ++S) v[S] = *reinterpret_cast<const float4*>(row + 16 * S);
#pragma unroll
      for (int S = 0; S < DD / 16; ++S) {
        const double x0 = v[S].x, x1 = v[S].y, x2 = v[S].z, x3 = v[S].w;
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(x0, x0, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(x1, x1, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(x2, x2, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(x3, x3, acc, 0, 0, 0);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) gpart[wave][(k + 4 * i) * 16 + n] = acc[i];
  }
  __syncthreads();
  if (tid < N * N) {
    const int p = tid >> 3, q = tid & 7;
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < 4; ++w) s += gpart[w][p * 16 + q] + gpart[w][(p + 8) * 16 + q + 8];   // fixed order
    A0[p * LD + q] = s;
    V0[p * LD + q] = (p == q) ? 1.0 : 0.0;
  }
  __syncthreads();
  // ---- wave 0 alone: Jacobi, ordering, T_3.  A wave's LDS operations execute in order, so
  // inside it a compiler barrier (no hardware one) separates the steps. ----
  if (wave == 0) {
    double trace = 0.0;
#pragma unroll
    for (int i = 0; i < N; ++i) trace += A0[i * LD + i];
    const double floor_abs = 1e-17 * trace;
    // parallel cyclic Jacobi: 7 rounds of 4 disjoint rotations per sweep
    double* Ac = A0; double* An = A1; double* Vc = V0; double* Vn = V1;
    constexpr int NM1 = N - 1;
    for (int sweep = 0; sweep < 16; ++sweep) {
      bool any_big = false;
      for (int round = 0; round < NM1; ++round) {
        bool big = false;
        if (lane < N / 2) {
          int p, q;
          if (lane == 0) { p = NM1; q = round; }
          else { p = (round + lane) % NM1; q = (round - lane + NM1) % NM1; }
          if (p > q) { const int t = p; p = q; q = t; }
          double c, sn;
          jacobi_rotation(Ac[p * LD + p], Ac[q * LD + q], Ac[p * LD + q], floor_abs, c, sn, big);
          rc[p] = c; rs[p] = sn; rc[q] = c; rs[q] = sn;
          partner[p] = q; partner[q] = p;
          is_p[p] = 1; is_p[q] = 0;
        }
        any_big = any_big || __any(big);
        __builtin_amdgcn_wave_barrier();
        // J[p][p] = c, J[p][q] = s, J[q][p] = -s, J[q][q] = c per pair;  A' = J^T A J,  V' = V J
        {
          const int i = lane >> 3, j = lane & 7;
          const int pi = partner[i], pj = partner[j];
          const double cj = rc[j], sj = is_p[j] ? -rs[j] : rs[j];
          const double ci = rc[i], si = is_p[i] ? -rs[i] : rs[i];
          const double aj_i = Ac[i * LD + j] * cj + Ac[i * LD + pj] * sj;
          const double aj_pi = Ac[pi * LD + j] * cj + Ac[pi * LD + pj] * sj;
          An[i * LD + j] = ci * aj_i + si * aj_pi;
          Vn[i * LD + j] = Vc[i * LD + j] * cj + Vc[i * LD + pj] * sj;
        }
        __builtin_amdgcn_wave_barrier();
        double* t = Ac; Ac = An; An = t;
        t = Vc; Vc = Vn; Vn = t;
      }
      if (!any_big) break;   // no rotated entry was above 3e-5 of its diagonal pair: this sweep finished them
    }

    // singular values in descending order, T_3, and W3[e][a3] = V'[a3, e] / sigma'_e
    if (lane < N) lam[lane] = Ac[lane * LD + lane];
    __builtin_amdgcn_wave_barrier();
    if (lane < N) {
      int rank = 0;
      const double me = lam[lane];
      for (int s2 = 0; s2 < N; ++s2) rank += (lam[s2] > me) || (lam[s2] == me && s2 < lane);
      order[rank] = lane;
    }
    __builtin_amdgcn_wave_barrier();
    if (lane < N) {
      const double lmax = fmax(lam[order[0]], 0.0);
      const double l = lam[order[lane]];
      sigma[lane] = (l > 1e-12 * lmax && l > 0.0) ? sqrt(l) : 0.0;
    }
    __builtin_amdgcn_wave_barrier();
    {
      const int e = lane >> 3, a3 = lane & 7;
      const double v = Vc[a3 * LD + order[e]];
      const double sg = sigma[e];
      W3[e * N + a3] = sg > 0.0 ? v / sg : 0.0;
      const long b3 = ((long)bh * g.NB + slot) * (N * N);
      const uint16_t hb = f64_to_f16_rne(v * sg, true, nullptr);   // |T_3| <= sqrt(j1): far inside fp16
      if (which) cache.v_small3[b3 + e * N + a3] = hb;   // values: natural [e][a3]
      else cache.k_small3[b3 + a3 * N + e] = hb;         // keys: transposed [a3][e]
    }
  }
  __syncthreads();

  // ---- projection in place: a thread owns one (a2, c') column of eight rows ----
  for (int idx = tid; idx < runs * DD; idx += 256) {
    const int a2 = idx / DD, c = idx % DD;
    float* col = blk + (long)a2 * N * DD + c;
    double x[N];
#pragma unroll
    for (int a3 = 0; a3 < N; ++a3) x[a3] = (double)col[a3 * DD];
#pragma unroll
    for (int e = 0; e < N; ++e) {
      double y = 0.0;
#pragma unroll
      for (int a3 = 0; a3 < N; ++a3) y = fma(W3[e * N + a3], x[a3], y);
      col[e * DD] = (float)y;
    }
  }
}

}  // namespace dq

// ------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------
using namespace dq;

static size_t compress_workspace_bytes(const dq_format* fmt, int batch, int kv_heads, int n_blocks) {
  // header (status words), the fp32 large tensors, one status word per block
  const size_t units = (size_t)batch * kv_heads * 2 * n_blocks;
  return (size_t)kWsHeaderBytes + units * fmt->block_tokens * fmt->head_dim * sizeof(float) +
         align_up(units * sizeof(int32_t), 256);
}

extern "C" size_t dq_compress_workspace_bytes(const dq_format* fmt, int32_t batch, int32_t kv_heads) {
  if (!format_ok(fmt) || batch <= 0 || kv_heads <= 0) return 0;
  return compress_workspace_bytes(fmt, batch, kv_heads, 1);
}

extern "C" size_t dq_compress_blocks_workspace_bytes(const dq_format* fmt, int32_t batch, int32_t kv_heads,
                                                     int32_t t_new) {
  if (!format_ok(fmt) || batch <= 0 || kv_heads <= 0 || t_new < 1) return 0;
  const int n_blocks = (t_new + fmt->block_tokens - 1) / fmt->block_tokens;
  if ((long)batch * kv_heads * 2 * n_blocks > (long)kMaxCompressUnits) return 0;
  return compress_workspace_bytes(fmt, batch, kv_heads, n_blocks);
}

extern "C" int32_t dq_quantize_pack(const dq_format* fmt, const float* t_large, int64_t n_rows,
                                    int32_t value_layout, uint8_t* codes, uint16_t* scales,
                                    void* hip_stream) {
  if (!format_ok(fmt) || !t_large || !codes || !scales) return DQ_EINVAL;
  if (n_rows < 0 || n_rows % kTileTokens) return DQ_EINVAL;
  if (n_rows == 0) return DQ_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  const int tiles = (int)(n_rows / kTileTokens);
  const size_t lds = quantize_lds_bytes(fmt->head_dim, fmt->bits);
  const int d = fmt->head_dim, G = fmt->group, j1 = fmt->j1, j2 = fmt->j2;
#define DQ_LAUNCH_QPACK(B_, D_)                                                                                  \
  do {                                                                                                           \
    if (fmt->levels)                                                                                             \
      hipLaunchKernelGGL((quantize_pack_kernel<B_, D_, true>), dim3(tiles), dim3(256), lds, st, t_large, G, j1,  \
                         j2, value_layout, codes, scales);                                                       \
    else                                                                                                         \
      hipLaunchKernelGGL((quantize_pack_kernel<B_, D_, false>), dim3(tiles), dim3(256), lds, st, t_large, G, j1, \
                         j2, value_layout, codes, scales);                                                       \
  } while (0)
  if (d == 128) {
    if (fmt->bits == 2) DQ_LAUNCH_QPACK(2, 128);
    else if (fmt->bits == 4) DQ_LAUNCH_QPACK(4, 128);
    else DQ_LAUNCH_QPACK(8, 128);
  } else {
    if (fmt->bits == 2) DQ_LAUNCH_QPACK(2, 64);
    else if (fmt->bits == 4) DQ_LAUNCH_QPACK(4, 64);
    else DQ_LAUNCH_QPACK(8, 64);
  }
#undef DQ_LAUNCH_QPACK
  DQ_HIP_CHECK(hipGetLastError());
  return DQ_OK;
}

static int32_t compress_impl(const dq_format* fmt, dq_cache* cache, const uint16_t* k_new,
                             const uint16_t* v_new, int32_t t_new, int n_blocks, const int32_t* blk_idx,
                             const int32_t* n_valid, void* workspace, size_t workspace_bytes, uint32_t flags,
                             void* hip_stream) {
  if (!cache->k_codes || !cache->k_scales || !cache->k_small || !cache->v_codes || !cache->v_scales ||
      !cache->v_small)
    return DQ_EINVAL;
  if (fmt->i3 != 1 && (!cache->k_small3 || !cache->v_small3)) return DQ_EINVAL;
  if (cache->batch <= 0 || cache->kv_heads <= 0 || cache->block_capacity <= 0) return DQ_EINVAL;
  if ((long)cache->batch * cache->kv_heads * 2 * n_blocks > (long)kMaxCompressUnits) return DQ_EINVAL;
  const size_t need = compress_workspace_bytes(fmt, cache->batch, cache->kv_heads, n_blocks);
  if (workspace_bytes < need) return DQ_ENOSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  int32_t* status = reinterpret_cast<int32_t*>(workspace);
  float* large_ws = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + kWsHeaderBytes);
  const int units = cache->batch * cache->kv_heads * 2 * n_blocks;
  int32_t* unit_status = reinterpret_cast<int32_t*>(large_ws + (size_t)units * fmt->block_tokens * fmt->head_dim);
  const CompressJob job = {k_new, v_new, t_new, n_blocks, blk_idx, n_valid, (flags & DQ_COMPRESS_NO_LARGE) ? 0 : 1};
  const size_t dlds = decompose_lds_bytes(fmt->i1 * fmt->j1, fmt->head_dim, fmt->i1);
#define DQ_LAUNCH_DECOMPOSE(J, DD_)                                                                      \
  hipLaunchKernelGGL((decompose_kernel<J, DD_>), dim3(units), dim3(64), dlds, st, *fmt, *cache, job, large_ws, \
                     unit_status)
#define DQ_LAUNCH_DECOMPOSE_I1(J, DD_, I_)                                                               \
  hipLaunchKernelGGL((decompose_kernel<J, DD_, I_>), dim3(units), dim3(64), dlds, st, *fmt, *cache, job, \
                     large_ws, unit_status)
  const bool force_general = (flags & DQ_COMPRESS_PLAIN) != 0;
  const int want_waves = (int)((flags >> 8) & 0xFu);   // 0: the library's choice
  // heads of 64 channels with j1 = 8 go through the same kernel two at a time
  const bool pair_heads = fmt->head_dim == 64 && fmt->j1 == 8 && (cache->kv_heads & 1) == 0 && fmt->i1 == 1;
  // Where the caller does not need the fp32 large tensors the decomposition kernel quantizes them
  // itself, which saves their trip through memory (four times the bytes the method needs) and the
  // quantizer's launch.  Calls of a few hundred blocks are bound by the latency of one block's chain
  // and give a block several waves; calls of more than 1024 blocks are bound by throughput and take
  // the lean build (one wave per block, three blocks per SIMD).
  const bool fused = (flags & DQ_COMPRESS_NO_LARGE) && fmt->i3 == 1 && fmt->i1 == 1 && !force_general &&
                     ((fmt->head_dim == 128 && fmt->j1 == 16 && (fmt->group == 128 || fmt->group == 64)) ||
                      (pair_heads && fmt->group == 64));
  // Three local tensors (d = 128, j1 = 16): the lean build makes both cuts and quantizes in one
  // launch, and leaves the fp32 rows of T_2 in the workspace if the caller wants them.  It is one wave
  // per block, so a call of a few hundred blocks, which is bound by the latency of one block's
  // chain, keeps the three launches (first cut with several waves per block, second cut,
  // quantizer); larger calls, and a forced wave count of one, take the one-kernel build.
  const bool fused3 = fmt->i3 == kRun && fmt->i1 == 1 && !force_general && fmt->head_dim == 128 && fmt->j1 == 16 &&
                      (fmt->group == 128 || fmt->group == 64) && (want_waves == 1 || (want_waves == 0 && units > 512));
  if (fused3) {
#define DQ_LAUNCH_FUSED3(B_)                                                                                     \
  do {                                                                                                           \
    if (fmt->levels)                                                                                             \
      hipLaunchKernelGGL((decompose16_kernel<1, false, B_, true, true, true>), dim3(units), dim3(64), 0, st, *fmt, \
                         *cache, job, large_ws, unit_status, status);                                            \
    else                                                                                                         \
      hipLaunchKernelGGL((decompose16_kernel<1, false, B_, false, true, true>), dim3(units), dim3(64), 0, st,    \
                         *fmt, *cache, job, large_ws, unit_status, status);                                      \
  } while (0)
    if (fmt->bits == 2) DQ_LAUNCH_FUSED3(2);
    else if (fmt->bits == 4) DQ_LAUNCH_FUSED3(4);
    else DQ_LAUNCH_FUSED3(8);
#undef DQ_LAUNCH_FUSED3
    DQ_HIP_CHECK(hipGetLastError());
    return DQ_OK;
  }
  if (fused) {
#define DQ_LAUNCH_FUSED(N_, B_)                                                                                 \
  do {                                                                                                          \
    if (pair_heads && fmt->levels)                                                                              \
      hipLaunchKernelGGL((decompose16_kernel<N_, true, B_, true>), dim3(units / 2), dim3(64 * N_), 0, st, *fmt, \
                         *cache, job, large_ws, unit_status, status);                                           \
    else if (pair_heads)                                                                                        \
      hipLaunchKernelGGL((decompose16_kernel<N_, true, B_, false>), dim3(units / 2), dim3(64 * N_), 0, st,      \
                         *fmt, *cache, job, large_ws, unit_status, status);                                     \
    else if (fmt->levels)                                                                                       \
      hipLaunchKernelGGL((decompose16_kernel<N_, false, B_, true>), dim3(units), dim3(64 * N_), 0, st, *fmt,    \
                         *cache, job, large_ws, unit_status, status);                                           \
    else                                                                                                        \
      hipLaunchKernelGGL((decompose16_kernel<N_, false, B_, false>), dim3(units), dim3(64 * N_), 0, st, *fmt,   \
                         *cache, job, large_ws, unit_status, status);                                           \
  } while (0)
#define DQ_LAUNCH_FUSED_LEAN(B_)                                                                                \
  do {                                                                                                          \
    if (pair_heads && fmt->levels)                                                                              \
      hipLaunchKernelGGL((decompose16_kernel<1, true, B_, true, true>), dim3(units / 2), dim3(64), 0, st, *fmt, \
                         *cache, job, large_ws, unit_status, status);                                           \
    else if (pair_heads)                                                                                        \
      hipLaunchKernelGGL((decompose16_kernel<1, true, B_, false, true>), dim3(units / 2), dim3(64), 0, st,      \
                         *fmt, *cache, job, large_ws, unit_status, status);                                     \
    else if (fmt->levels)                                                                                       \
      hipLaunchKernelGGL((decompose16_kernel<1, false, B_, true, true>), dim3(units), dim3(64), 0, st, *fmt,    \
                         *cache, job, large_ws, unit_status, status);                                           \
    else                                                                                                        \
      hipLaunchKernelGGL((decompose16_kernel<1, false, B_, false, true>), dim3(units), dim3(64), 0, st, *fmt,   \
                         *cache, job, large_ws, unit_status, status);                                           \
  } while (0)
    const int fused_groups = pair_heads ? units / 2 : units;
    int fused_waves = fused_groups <= 256 ? 4 : fused_groups <= 512 ? 2 : fused_groups <= 1024 ? 1 : 0;   // 0: the lean build
    if (want_waves) fused_waves = want_waves;
    if (fused_waves == 0) {
      if (fmt->bits == 2) DQ_LAUNCH_FUSED_LEAN(2);
      else if (fmt->bits == 4) DQ_LAUNCH_FUSED_LEAN(4);
      else DQ_LAUNCH_FUSED_LEAN(8);
    } else if (fused_waves == 4) {
      if (fmt->bits == 2) DQ_LAUNCH_FUSED(4, 2);
      else if (fmt->bits == 4) DQ_LAUNCH_FUSED(4, 4);
      else DQ_LAUNCH_FUSED(4, 8);
    } else if (fused_waves == 2) {
      if (fmt->bits == 2) DQ_LAUNCH_FUSED(2, 2);
      else if (fmt->bits == 4) DQ_LAUNCH_FUSED(2, 4);
      else DQ_LAUNCH_FUSED(2, 8);
    } else {
      if (fmt->bits == 2) DQ_LAUNCH_FUSED(1, 2);
      else if (fmt->bits == 4) DQ_LAUNCH_FUSED(1, 4);
      else DQ_LAUNCH_FUSED(1, 8);
    }
#undef DQ_LAUNCH_FUSED
#undef DQ_LAUNCH_FUSED_LEAN
    DQ_HIP_CHECK(hipGetLastError());
    return DQ_OK;
  }
  if (fmt->i1 > 1) {   // a token factor on the small tensor: the plain kernel on the side i1 * j1
    const int dd = fmt->head_dim, jj = fmt->j1;
    if (fmt->i1 == 2) {
      if (dd == 128 && jj == 16) DQ_LAUNCH_DECOMPOSE_I1(16, 128, 2);
      else if (dd == 128 && jj == 8) DQ_LAUNCH_DECOMPOSE_I1(8, 128, 2);
      else if (dd == 64 && jj == 16) DQ_LAUNCH_DECOMPOSE_I1(16, 64, 2);
      else if (dd == 64 && jj == 8) DQ_LAUNCH_DECOMPOSE_I1(8, 64, 2);
      else return DQ_EINVAL;
    } else {
      if (dd == 128 && jj == 8) DQ_LAUNCH_DECOMPOSE_I1(8, 128, 4);
      else if (dd == 64 && jj == 8) DQ_LAUNCH_DECOMPOSE_I1(8, 64, 4);
      else return DQ_EINVAL;
    }
  } else if (((fmt->head_dim == 128 && fmt->j1 == 16) || pair_heads) && !force_general) {
    // At most one workgroup per compute unit (256 on the chip) gets more waves per block: the
    // eigen-solver wave is issue-bound and slows down when two of them share a SIMD.
#define DQ_LAUNCH_D16(N_)                                                                                     \
  do {                                                                                                        \
    if (pair_heads)                                                                                           \
      hipLaunchKernelGGL((decompose16_kernel<N_, true>), dim3(units / 2), dim3(64 * N_), 0, st, *fmt, *cache, \
                         job, large_ws, unit_status, (int32_t*)nullptr);                                      \
    else                                                                                                      \
      hipLaunchKernelGGL((decompose16_kernel<N_, false>), dim3(units), dim3(64 * N_), 0, st, *fmt, *cache,    \
                         job, large_ws, unit_status, (int32_t*)nullptr);                                      \
  } while (0)
    const int groups16 = pair_heads ? units / 2 : units;
    int nwv = groups16 <= 256 ? 4 : groups16 <= 512 ? 2 : groups16 <= 1024 ? 1 : 0;   // 0: the lean build
    if (want_waves) nwv = want_waves;
    if (nwv == 0) {
      if (pair_heads)
        hipLaunchKernelGGL((decompose16_kernel<1, true, 0, false, true>), dim3(units / 2), dim3(64), 0, st, *fmt, *cache,
                           job, large_ws, unit_status, (int32_t*)nullptr);
      else
        hipLaunchKernelGGL((decompose16_kernel<1, false, 0, false, true>), dim3(units), dim3(64), 0, st, *fmt, *cache,
                           job, large_ws, unit_status, (int32_t*)nullptr);
    } else if (nwv >= 4) DQ_LAUNCH_D16(4);
    else if (nwv >= 2) DQ_LAUNCH_D16(2);
    else DQ_LAUNCH_D16(1);
#undef DQ_LAUNCH_D16
  } else if (fmt->head_dim == 128) {
    if (fmt->j1 == 8) DQ_LAUNCH_DECOMPOSE(8, 128);
    else if (fmt->j1 == 16) DQ_LAUNCH_DECOMPOSE(16, 128);
    else DQ_LAUNCH_DECOMPOSE(32, 128);
  } else {
    if (fmt->j1 == 8) DQ_LAUNCH_DECOMPOSE(8, 64);
    else if (fmt->j1 == 16) DQ_LAUNCH_DECOMPOSE(16, 64);
    else DQ_LAUNCH_DECOMPOSE(32, 64);
  }
#undef DQ_LAUNCH_DECOMPOSE
#undef DQ_LAUNCH_DECOMPOSE_I1
  DQ_HIP_CHECK(hipGetLastError());
  if (fmt->i3 == kRun) {   // three local tensors: cut the right factor again before it is quantized
    if (fmt->head_dim == 128)
      hipLaunchKernelGGL((split3_kernel<128>), dim3(units), dim3(256), 0, st, *fmt, *cache, job, large_ws);
    else
      hipLaunchKernelGGL((split3_kernel<64>), dim3(units), dim3(256), 0, st, *fmt, *cache, job, large_ws);
    DQ_HIP_CHECK(hipGetLastError());
  }
  const int tiles = units * (fmt->block_tokens / kTileTokens);
  const size_t lds = quantize_lds_bytes(fmt->head_dim, fmt->bits);
#define DQ_LAUNCH_QTILES(B_, D_)                                                                              \
  do {                                                                                                        \
    if (fmt->levels)                                                                                          \
      hipLaunchKernelGGL((quantize_tiles_kernel<B_, D_, true>), dim3(tiles), dim3(256), lds, st, large_ws,    \
                         *fmt, *cache, job, unit_status, units, status);                                      \
    else                                                                                                      \
      hipLaunchKernelGGL((quantize_tiles_kernel<B_, D_, false>), dim3(tiles), dim3(256), lds, st, large_ws,   \
                         *fmt, *cache, job, unit_status, units, status);                                      \
  } while (0)
  if (fmt->head_dim == 128) {
    if (fmt->bits == 2) DQ_LAUNCH_QTILES(2, 128);
    else if (fmt->bits == 4) DQ_LAUNCH_QTILES(4, 128);
    else DQ_LAUNCH_QTILES(8, 128);
  } else {
    if (fmt->bits == 2) DQ_LAUNCH_QTILES(2, 64);
    else if (fmt->bits == 4) DQ_LAUNCH_QTILES(4, 64);
    else DQ_LAUNCH_QTILES(8, 64);
  }
#undef DQ_LAUNCH_QTILES
  DQ_HIP_CHECK(hipGetLastError());
  return DQ_OK;
}

extern "C" int32_t dq_compress_kv(const dq_format* fmt, dq_cache* cache, const uint16_t* k_new,
                                  const uint16_t* v_new, int32_t t_new, const int32_t* blk_idx,
                                  const int32_t* n_valid, void* workspace, size_t workspace_bytes,
                                  void* hip_stream) {
  if (!format_ok(fmt) || !cache || !k_new || !v_new || !blk_idx || !workspace) return DQ_EINVAL;
  if (t_new < 1 || t_new > fmt->block_tokens) return DQ_EINVAL;
  return compress_impl(fmt, cache, k_new, v_new, t_new, 1, blk_idx, n_valid, workspace, workspace_bytes,
                       DQ_COMPRESS_KEEP_LARGE, hip_stream);
}

extern "C" int32_t dq_compress_kv_blocks(const dq_format* fmt, dq_cache* cache, const uint16_t* k_new,
                                         const uint16_t* v_new, int32_t t_new, const int32_t* blk_idx,
                                         const int32_t* n_valid, void* workspace, size_t workspace_bytes,
                                         void* hip_stream) {
  if (!format_ok(fmt) || !cache || !k_new || !v_new || !blk_idx || !workspace) return DQ_EINVAL;
  if (t_new < 1) return DQ_EINVAL;
  const int n_blocks = (t_new + fmt->block_tokens - 1) / fmt->block_tokens;
  if (n_blocks > cache->block_capacity) return DQ_EINVAL;
  return compress_impl(fmt, cache, k_new, v_new, t_new, n_blocks, blk_idx, n_valid, workspace,
                       workspace_bytes, DQ_COMPRESS_KEEP_LARGE, hip_stream);
}

extern "C" int32_t dq_compress_kv_ex(const dq_format* fmt, dq_cache* cache, const uint16_t* k_new,
                                     const uint16_t* v_new, int32_t t_new, const int32_t* blk_idx,
                                     const int32_t* n_valid, void* workspace, size_t workspace_bytes,
                                     uint32_t flags, void* hip_stream) {
  if (!format_ok(fmt) || !cache || !k_new || !v_new || !blk_idx || !workspace) return DQ_EINVAL;
  if (t_new < 1 || (flags & ~(DQ_COMPRESS_NO_LARGE | DQ_COMPRESS_PLAIN | DQ_COMPRESS_WAVES(0xF)))) return DQ_EINVAL;
  {
    const uint32_t wv = (flags >> 8) & 0xFu;
    if (wv != 0 && wv != 1 && wv != 2 && wv != 4) return DQ_EINVAL;
  }
  const int n_blocks = (t_new + fmt->block_tokens - 1) / fmt->block_tokens;
  if (n_blocks > cache->block_capacity) return DQ_EINVAL;
  return compress_impl(fmt, cache, k_new, v_new, t_new, n_blocks, blk_idx, n_valid, workspace,
                       workspace_bytes, flags, hip_stream);
}
