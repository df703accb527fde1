// Reference-grade decode attention over the compressed cache: plain fp32 HIP, any supported
// format, one workgroup per (sequence, query head, sequence split).  It states the fused
// computation of Section 3.2 (arXiv 2405.12591) in its simplest form:
//   q'[r, b2]  = scale * sum_b1 T_S^K[b1, r] q[b1, b2]            (small tensor folded into q)
//   s_t        = sum_g step^K[t, g] * sum_{c' in g} code^K[t, c'] q'[c']
//   o'[c']     = sum_t p_t step^V[t, g(c')] code^V[t, c']          (per 128-token tile)
//   acc[b1,b2] = alpha * acc[b1, b2] + sum_r T_S^V[b1, r] o'[r, b2]
// followed by a log-sum-exp merge of the splits.  With three local tensors (format.i3 == 8) row
// a2*8 + e of the codes belongs to the bond index e, not to a token: the scores of the eight tokens
// of a run are s[a2*8 + a3] = sum_e T_3^K[e, a3] y[a2*8 + e] (y: the row sums above), and the values
// are weighted with p'[a2*8 + e] = sum_a3 T_3^V[e, a3] p[a2*8 + a3].
#include <hip/hip_ext.h>

#include "dq_decode.h"
#include "dq_tail.h"

namespace dq {

template <int BITS>
__device__ inline float dot_codes(const uint32_t* __restrict__ words, const float* __restrict__ qf, int n) {
  // sum over n consecutive elements (n * BITS multiple of 32) of code * qf
  constexpr int PER = 32 / BITS;
  constexpr int MASK = (1 << BITS) - 1;
  constexpr int BIAS = 1 << (BITS - 1);
  float s = 0.f;
  for (int w = 0; w < n / PER; ++w) {
    const uint32_t x = words[w];
#pragma unroll
    for (int k = 0; k < PER; ++k) s = fmaf((float)((int)((x >> (k * BITS)) & MASK) - BIAS), qf[w * PER + k], s);
  }
  return s;
}

template <int BITS>
__global__ __launch_bounds__(256) void decode_generic_kernel(DecodeArgs a) {
  const Geometry g = make_geometry(a.fmt, a.cache.kv_heads, a.cache.block_capacity);
  const int d = g.d, j1 = g.j1, j2 = g.j2, G = g.G;
  const int split = a.rows_on_x ? blockIdx.y : blockIdx.x;
  const int bhq = a.rows_on_x ? blockIdx.x : blockIdx.y;
  const int b = bhq / a.q_heads, hq = bhq % a.q_heads;
  const int rep = a.q_heads / g.H;
  const int h = hq / rep;
  const int tid = threadIdx.x;
  const int S = min(max(a.seq_lens[b], 0), a.max_seq_len);
  const int tiles_total = (S + kTileTokens - 1) / kTileTokens;
  const int max_tiles = (a.max_seq_len + kTileTokens - 1) / kTileTokens;
  const int tps = (max_tiles + a.n_split - 1) / a.n_split;
  const int tile_begin = split * tps;
  const int tile_end = min(tile_begin + tps, tiles_total);

  __shared__ float qs[128];        // the query as fp32
  __shared__ float qf[128];        // folded query q'
  __shared__ float sc[kTileTokens];
  __shared__ float red[8];
  __shared__ float opart[4][128];
  __shared__ float sK[32 * 32];    // T_S^K as stored: [r][b1]
  __shared__ float sV[32 * 32];    // T_S^V as stored: [b1][r]
  __shared__ float sK3[kRun * kRun];   // T_3^K as stored: [a3][e]
  __shared__ float sV3[kRun * kRun];   // T_3^V as stored: [e][a3]
  const bool three = a.fmt.i3 == kRun;

  if (tid < d) qs[tid] = h2f(a.q[(long)bhq * d + tid]);
  float acc = 0.f;                 // thread c < d owns output channel c = b1*j2 + b2
  float m_run = -INFINITY, l_run = 0.f;
  const long bh = (long)b * g.H + h;
  int cur_blk = -1;
  const int nparts = 256 / d;      // token parts in the value phase
  const int seg = d / 2;
  __syncthreads();

  for (int tile = tile_begin; tile < tile_end; ++tile) {
    const int blk = tile / g.tiles_per_block;
    const int tib = tile % g.tiles_per_block;
    const long blkid = bh * g.NB + blk;
    if (blk != cur_blk) {
      cur_blk = blk;
      const uint16_t* ks = a.cache.k_small + blkid * g.small_per_block;
      const uint16_t* vs = a.cache.v_small + blkid * g.small_per_block;
      for (int i = tid; i < j1 * j1; i += blockDim.x) { sK[i] = h2f(ks[i]); sV[i] = h2f(vs[i]); }
      if (three && tid < kRun * kRun) {
        sK3[tid] = h2f(a.cache.k_small3[blkid * (kRun * kRun) + tid]);
        sV3[tid] = h2f(a.cache.v_small3[blkid * (kRun * kRun) + tid]);
      }
      __syncthreads();
      if (tid < d) {
        const int r = tid / j2, b2 = tid % j2;
        float s = 0.f;
        for (int b1 = 0; b1 < j1; ++b1) s = fmaf(sK[r * j1 + b1], qs[b1 * j2 + b2], s);
        qf[tid] = s * a.scale;
      }
      __syncthreads();
    }
    // ---- scores: two threads per token, each one half row ----
    {
      const int tt = tid >> 1, half = tid & 1;
      const int t = tile * kTileTokens + tt;
      const int row = tib * kTileTokens + tt;
      float s = 0.f;
      // three tensors: a row is needed as soon as its run of eight holds a valid token
      const bool row_live = three ? (t - (tt & (kRun - 1))) < S : t < S;
      if (row_live) {
        const uint8_t* rowp = a.cache.k_codes + blkid * g.codes_per_block + (long)row * g.row_bytes;
        const uint16_t* scp = a.cache.k_scales + blkid * g.scales_per_block + (long)row * g.groups;
        const uint32_t* words = reinterpret_cast<const uint32_t*>(rowp) + half * seg * BITS / 32;
        if (G >= seg) {
          const int gi = (half * seg) / G;
          s = h2f(scp[gi]) * dot_codes<BITS>(words, qf + half * seg, seg);
        } else {
          const int gps = seg / G;
          for (int k = 0; k < gps; ++k)
            s = fmaf(h2f(scp[half * gps + k]),
                     dot_codes<BITS>(words + k * G * BITS / 32, qf + half * seg + k * G, G), s);
        }
      }
      s += __shfl_xor(s, 1);
      if (half == 0) sc[tt] = three ? (row_live ? s : 0.f) : ((t < S) ? s : -INFINITY);
    }
    __syncthreads();
    if (three) {   // rows -> tokens: s[a2*8 + a3] = sum_e T_3^K[e, a3] y[a2*8 + e]
      float s = -INFINITY;
      if (tid < kTileTokens && tile * kTileTokens + tid < S) {
        const int run0 = tid & ~(kRun - 1), a3 = tid & (kRun - 1);
        s = 0.f;
#pragma unroll
        for (int e = 0; e < kRun; ++e) s = fmaf(sK3[a3 * kRun + e], sc[run0 + e], s);
      }
      __syncthreads();
      if (tid < kTileTokens) sc[tid] = s;
      __syncthreads();
    }
    // ---- tile max ----
    float v = (tid < kTileTokens) ? sc[tid] : -INFINITY;
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    if ((tid & 63) == 0) red[tid >> 6] = v;
    __syncthreads();
    const float m_tile = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float m_new = fmaxf(m_run, m_tile);
    const float alpha = __expf(m_run - m_new);  // m_run = -inf gives 0
    __syncthreads();
    float p = 0.f;
    if (tid < kTileTokens) {
      p = __expf(sc[tid] - m_new);
      sc[tid] = p;
    }
    float ps = p;
    for (int o = 32; o > 0; o >>= 1) ps += __shfl_xor(ps, o);
    if ((tid & 63) == 0) red[4 + (tid >> 6)] = ps;
    __syncthreads();
    l_run = l_run * alpha + (red[4] + red[5] + red[6] + red[7]);
    m_run = m_new;
    if (three) {   // tokens -> rows: p'[a2*8 + e] = sum_a3 T_3^V[e, a3] p[a2*8 + a3]
      float pw = 0.f;
      if (tid < kTileTokens) {
        const int run0 = tid & ~(kRun - 1), e = tid & (kRun - 1);
#pragma unroll
        for (int a3 = 0; a3 < kRun; ++a3) pw = fmaf(sV3[e * kRun + a3], sc[run0 + a3], pw);
      }
      __syncthreads();
      if (tid < kTileTokens) sc[tid] = pw;
      __syncthreads();
    }
    // ---- values: thread (c', part) accumulates its share of the tile's tokens ----
    {
      const int cp = tid % d, part = tid / d;
      const int r = cp / j2, b2 = cp % j2;
      const int gi = cp / G;
      const uint8_t* vrow = a.cache.v_codes + blkid * g.codes_per_block +
                            ((long)(tib * j2 + b2) * j1 + r) * g.vrow_bytes;
      const uint16_t* vsc = a.cache.v_scales + blkid * g.scales_per_block +
                            (long)tib * kTileTokens * g.groups;
      const int tok_per_part = kTileTokens / nparts;
      const int t0 = part * tok_per_part;
      constexpr int PER = 32 / BITS;
      constexpr int MASK = (1 << BITS) - 1;
      constexpr int BIAS = 1 << (BITS - 1);
      const uint32_t* words = reinterpret_cast<const uint32_t*>(vrow) + t0 / PER;
      float o = 0.f;
      for (int w = 0; w < tok_per_part / PER; ++w) {
        const uint32_t x = words[w];
#pragma unroll
        for (int k = 0; k < PER; ++k) {
          const int tt = t0 + w * PER + k;
          const float pt = sc[tt];
          if (pt != 0.f) {  // masked tokens may carry any step bits, never touch them
            const float code = (float)((int)((x >> (k * BITS)) & MASK) - BIAS);
            o = fmaf(pt * h2f(vsc[(long)tt * g.groups + gi]), code, o);
          }
        }
      }
      opart[part][cp] = o;
    }
    __syncthreads();
    if (tid < d) {
      const int b1 = tid / j2, b2 = tid % j2;
      float s = 0.f;
      for (int r = 0; r < j1; ++r) {
        float o = 0.f;
        for (int part = 0; part < nparts; ++part) o += opart[part][r * j2 + b2];
        s = fmaf(sV[b1 * j1 + r], o, s);
      }
      acc = acc * alpha + s;
    }
    __syncthreads();
  }
  float* part = a.partials + ((long)bhq * a.n_slots + split) * (d + 2);
  if (tid < d) part[tid] = acc;
  if (tid == 0) { part[d] = m_run; part[d + 1] = l_run; }
}

// The same computation for formats with a token factor on the small tensor (format.i1 = I1 > 1;
// Eq. 2 with n = 2, i_1 > 1).  Token t = a1*i2 + a2 of a block, bond index r = rho*j1 + r':
//   q'_a1[r, b2] = scale * sum_b1 T_S^K[(a1, b1), r] q[b1, b2]              (I1 folded queries)
//   s_(a1, a2)   = sum_rho sum_c' step^K[row] code^K[row, c'] q'_a1[rho*d + c'],   row = a2*I1 + rho
//   o'_a1[r, b2] = sum_a2 p_(a1, a2) step^V[row] code^V[row, r'*j2 + b2]
//   acc[b1, b2]  = alpha * acc[b1, b2] + sum_a1 sum_r T_S^V[(a1, b1), r] o'_a1[r, b2]
// A tile of 128 rows holds 128 / I1 positions a2 and gives the scores of 128 tokens, I1 runs of
// 128 / I1 consecutive ones.  A token's rows lie all over its block, so a block with a valid token
// is worked whole.
template <int BITS, int I1>
__global__ __launch_bounds__(256) void decode_generic_i1_kernel(DecodeArgs a) {
  const Geometry g = make_geometry(a.fmt, a.cache.kv_heads, a.cache.block_capacity);
  const int d = g.d, j1 = g.j1, j2 = g.j2, G = g.G;
  const int N = I1 * j1;           // side of the small tensor, <= 32
  const int i2 = g.Tb / I1;
  constexpr int PPT = kTileTokens / I1;   // positions a2 per tile
  const int split = a.rows_on_x ? blockIdx.y : blockIdx.x;
  const int bhq = a.rows_on_x ? blockIdx.x : blockIdx.y;
  const int b = bhq / a.q_heads, hq = bhq % a.q_heads;
  const int rep = a.q_heads / g.H;
  const int h = hq / rep;
  const int tid = threadIdx.x;
  const int S = min(max(a.seq_lens[b], 0), a.max_seq_len);
  const int tpb = g.tiles_per_block;
  const int tiles_total = (S + g.Tb - 1) / g.Tb * tpb;            // whole blocks
  const int max_tiles = (a.max_seq_len + g.Tb - 1) / g.Tb * tpb;
  const int tps = (max_tiles + a.n_split - 1) / a.n_split;
  const int tile_begin = split * tps;
  const int tile_end = min(tile_begin + tps, tiles_total);

  __shared__ float qs[128];                 // the query as fp32
  __shared__ float qf[I1 * I1 * 128];       // folded queries q'_a1[rho*d + c']
  __shared__ float ys[I1][kTileTokens];     // row sums per a1
  __shared__ float sc[kTileTokens];         // scores, then weights, token index a1*PPT + a2 - a2_0
  __shared__ float red[8];
  __shared__ float opart[4][I1 * I1][128];  // [token part][a1*I1 + rho][c']
  __shared__ float sK[32 * 32];             // T_S^K as stored: [r][(a1, b1)]
  __shared__ float sV[32 * 32];             // T_S^V as stored: [(a1, b1)][r]

  if (tid < d) qs[tid] = h2f(a.q[(long)bhq * d + tid]);
  float acc = 0.f;                 // thread c < d owns output channel c = b1*j2 + b2
  float m_run = -INFINITY, l_run = 0.f;
  const long bh = (long)b * g.H + h;
  int cur_blk = -1;
  const int nparts = 256 / d;      // row parts in the value phase
  const int seg = d / 2;
  __syncthreads();

  for (int tile = tile_begin; tile < tile_end; ++tile) {
    const int blk = tile / tpb;
    const int tib = tile % tpb;
    const long blkid = bh * g.NB + blk;
    if (blk != cur_blk) {
      cur_blk = blk;
      const uint16_t* ks = a.cache.k_small + blkid * g.small_per_block;
      const uint16_t* vs = a.cache.v_small + blkid * g.small_per_block;
      for (int i = tid; i < N * N; i += blockDim.x) { sK[i] = h2f(ks[i]); sV[i] = h2f(vs[i]); }
      __syncthreads();
      for (int i = tid; i < I1 * N * j2; i += blockDim.x) {
        const int a1 = i / (N * j2), r = (i / j2) % N, b2 = i % j2;
        float s = 0.f;
        for (int b1 = 0; b1 < j1; ++b1) s = fmaf(sK[r * N + a1 * j1 + b1], qs[b1 * j2 + b2], s);
        qf[i] = s * a.scale;       // index a1*(I1*d) + rho*d + r'*j2 + b2
      }
      __syncthreads();
    }
    const int a2_0 = tib * PPT;    // the tile's first position
    // ---- row sums: two threads per row, each one half row, against every folded query ----
    {
      const int tt = tid >> 1, half = tid & 1;
      const int a2 = a2_0 + tt / I1, rho = tt % I1;
      const int row = tib * kTileTokens + tt;
      float y[I1];
#pragma unroll
      for (int a1 = 0; a1 < I1; ++a1) y[a1] = 0.f;
      // a row is needed as soon as its position holds a valid token; a1 = 0 is the first of them
      if (blk * g.Tb + a2 < S) {
        const uint8_t* rowp = a.cache.k_codes + blkid * g.codes_per_block + (long)row * g.row_bytes;
        const uint16_t* scp = a.cache.k_scales + blkid * g.scales_per_block + (long)row * g.groups;
        const uint32_t* words = reinterpret_cast<const uint32_t*>(rowp) + half * seg * BITS / 32;
#pragma unroll
        for (int a1 = 0; a1 < I1; ++a1) {
          const float* qa = qf + (a1 * I1 + rho) * d + half * seg;
          if (G >= seg) {
            y[a1] = h2f(scp[(half * seg) / G]) * dot_codes<BITS>(words, qa, seg);
          } else {
            const int gps = seg / G;
            for (int k = 0; k < gps; ++k)
              y[a1] = fmaf(h2f(scp[half * gps + k]), dot_codes<BITS>(words + k * G * BITS / 32, qa + k * G, G), y[a1]);
          }
        }
      }
#pragma unroll
      for (int a1 = 0; a1 < I1; ++a1) {
        y[a1] += __shfl_xor(y[a1], 1);
        if (half == 0) ys[a1][tt] = y[a1];
      }
    }
    __syncthreads();
    // ---- scores of the tile's 128 tokens: token (a1, a2) sums its position's I1 rows ----
    if (tid < kTileTokens) {
      const int a1 = tid / PPT, pl = tid % PPT;
      const int t = blk * g.Tb + a1 * i2 + a2_0 + pl;
      float s = -INFINITY;
      if (t < S) {
        s = 0.f;
#pragma unroll
        for (int rho = 0; rho < I1; ++rho) s += ys[a1][pl * I1 + rho];
      }
      sc[tid] = s;
    }
    __syncthreads();
    // ---- tile max ----
    float v = (tid < kTileTokens) ? sc[tid] : -INFINITY;
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    if ((tid & 63) == 0) red[tid >> 6] = v;
    __syncthreads();
    const float m_tile = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float m_new = fmaxf(m_run, m_tile);
    // a tile of a partly valid block may hold no valid token at all: nothing moves then
    const float alpha = (m_new == -INFINITY) ? 1.f : __expf(m_run - m_new);
    __syncthreads();
    float p = 0.f;
    if (tid < kTileTokens) {
      p = (m_new == -INFINITY) ? 0.f : __expf(sc[tid] - m_new);
      sc[tid] = p;
    }
    float ps = p;
    for (int o = 32; o > 0; o >>= 1) ps += __shfl_xor(ps, o);
    if ((tid & 63) == 0) red[4 + (tid >> 6)] = ps;
    __syncthreads();
    l_run = l_run * alpha + (red[4] + red[5] + red[6] + red[7]);
    m_run = m_new;
    // ---- values: thread (c', part) accumulates its share of the tile's rows, per (a1, rho) ----
    {
      const int cp = tid % d, part = tid / d;
      const int r = cp / j2, b2 = cp % j2;
      const int gi = cp / G;
      const uint8_t* vrow = a.cache.v_codes + blkid * g.codes_per_block +
                            ((long)(tib * j2 + b2) * j1 + r) * g.vrow_bytes;
      const uint16_t* vsc = a.cache.v_scales + blkid * g.scales_per_block +
                            (long)tib * kTileTokens * g.groups;
      const int rows_per_part = kTileTokens / nparts;
      const int t0 = part * rows_per_part;
      constexpr int PER = 32 / BITS;            // a multiple of I1
      constexpr int MASK = (1 << BITS) - 1;
      constexpr int BIAS = 1 << (BITS - 1);
      static_assert(PER % I1 == 0, "a word of codes holds whole positions");
      const uint32_t* words = reinterpret_cast<const uint32_t*>(vrow) + t0 / PER;
      float o[I1][I1];
#pragma unroll
      for (int a1 = 0; a1 < I1; ++a1)
#pragma unroll
        for (int rho = 0; rho < I1; ++rho) o[a1][rho] = 0.f;
      for (int w = 0; w < rows_per_part / PER; ++w) {
        const uint32_t x = words[w];
#pragma unroll
        for (int k = 0; k < PER; ++k) {
          const int tt = t0 + w * PER + k;      // row in the tile: position tt / I1, slice k % I1
          const float code = (float)((int)((x >> (k * BITS)) & MASK) - BIAS);
#pragma unroll
          for (int a1 = 0; a1 < I1; ++a1) {
            const float pt = sc[a1 * PPT + tt / I1];
            if (pt != 0.f)   // rows of positions without a valid token may carry any step bits
              o[a1][k % I1] = fmaf(pt * h2f(vsc[(long)tt * g.groups + gi]), code, o[a1][k % I1]);
          }
        }
      }
#pragma unroll
      for (int a1 = 0; a1 < I1; ++a1)
#pragma unroll
        for (int rho = 0; rho < I1; ++rho) opart[part][a1 * I1 + rho][cp] = o[a1][rho];
    }
    __syncthreads();
    if (tid < d) {
      const int b1 = tid / j2, b2 = tid % j2;
      float s = 0.f;
      for (int a1 = 0; a1 < I1; ++a1) {
        for (int r = 0; r < N; ++r) {
          const int rho = r / j1, rp = r % j1;
          float o = 0.f;
          for (int part = 0; part < nparts; ++part) o += opart[part][a1 * I1 + rho][rp * j2 + b2];
          s = fmaf(sV[(a1 * j1 + b1) * N + r], o, s);
        }
      }
      acc = acc * alpha + s;
    }
    __syncthreads();
  }
  float* part = a.partials + ((long)bhq * a.n_slots + split) * (d + 2);
  if (tid < d) part[tid] = acc;
  if (tid == 0) { part[d] = m_run; part[d + 1] = l_run; }
}

// Merge split partials: out = sum_s acc_s e^{m_s - M} / sum_s l_s e^{m_s - M}.
__global__ void combine_kernel(const float* __restrict__ partials, int n_split, int d,
                               uint16_t* __restrict__ out, float* __restrict__ out_f32) {
  const int bhq = blockIdx.x;
  const int c = threadIdx.x;
  const float* base = partials + (long)bhq * n_split * (d + 2);
  float M = -INFINITY;
  for (int s = 0; s < n_split; ++s) M = fmaxf(M, base[s * (d + 2) + d]);
  float L = 0.f, o = 0.f;
  for (int s = 0; s < n_split; ++s) {
    const float m = base[s * (d + 2) + d];
    if (m == -INFINITY) continue;
    const float w = __expf(m - M);
    L = fmaf(base[s * (d + 2) + d + 1], w, L);
    o = fmaf(base[s * (d + 2) + c], w, o);
  }
  const float r = (L > 0.f) ? o / L : 0.f;
  out[(long)bhq * d + c] = f2h_rne(r);
  if (out_f32) out_f32[(long)bhq * d + c] = r;
}

int32_t launch_combine(const DecodeArgs& a, hipStream_t st) {
  const int d = a.fmt.head_dim;
  hipLaunchKernelGGL(combine_kernel, dim3(a.cache.batch * a.q_heads), dim3(d), 0, st, a.partials, a.n_slots, d,
                     a.out, a.out_f32);
  DQ_HIP_CHECK(hipGetLastError());
  return DQ_OK;
}

// The fp16 tail as a kernel of its own (for the plain fp32 decode path): one workgroup per
// (sequence, kv head), query heads in groups of four; the partial goes to slot n_split.  m_unit
// converts the running maximum from log2 units to the unit the merging kernel expects (ln 2 for
// natural logarithms).
template <int D>
__global__ __launch_bounds__(256) void tail_partial_kernel(DecodeArgs a, float m_unit) {
  typedef TailBlock<D, 4, 4> TB;
  const int H = a.cache.kv_heads, rep = a.q_heads / H;
  const int b = blockIdx.x / H, h = blockIdx.x % H;
  __shared__ float scratch[TB::kScratchFloats];
  __shared__ float result[TB::kResultFloats];
  for (int hg = 0; hg < rep; hg += TB::HB) {
    const int nh = min(TB::HB, rep - hg);
    const long hq0 = (long)h * rep + hg;
    const int tail_len = a.tail.tail_lens[b];
    TB tb;
    tb.issue_keys(a, b, h, hq0, nh);
    tb.finish(tail_len, nh, scratch, result);
    for (int idx = threadIdx.x; idx < nh * (D + 2); idx += 256) {
      const int hd = idx / (D + 2), c = idx % (D + 2);
      float v = result[idx];
      if (c == D) v *= m_unit;   // -inf stays -inf
      a.partials[(((long)b * a.q_heads + hq0 + hd) * a.n_slots + a.n_split) * (D + 2) + c] = v;
    }
    __syncthreads();
  }
}

int32_t launch_tail_partial(const DecodeArgs& a, float m_unit, hipStream_t st) {
  const dim3 grid(a.cache.batch * a.cache.kv_heads);
  if (a.fmt.head_dim == 128) hipLaunchKernelGGL(tail_partial_kernel<128>, grid, dim3(256), 0, st, a, m_unit);
  else hipLaunchKernelGGL(tail_partial_kernel<64>, grid, dim3(256), 0, st, a, m_unit);
  DQ_HIP_CHECK(hipGetLastError());
  return DQ_OK;
}

int32_t launch_decode_generic(const DecodeArgs& a, hipStream_t st) {
  if (a.tail.k_tail) {   // the tail's partial is in natural-log units like this path's
    const int32_t rc = launch_tail_partial(a, 0.6931471805599453f, st);
    if (rc != DQ_OK) return rc;
  }
  const dim3 grid = a.rows_on_x ? dim3(a.cache.batch * a.q_heads, a.n_split) : dim3(a.n_split, a.cache.batch * a.q_heads);
  // the events, when given, receive the streaming kernel's own begin and end timestamps
  if (a.fmt.i1 > 1) {   // a token factor on the small tensor
#define DQ_LAUNCH_I1(B_)                                                                                          \
  do {                                                                                                            \
    if (a.fmt.i1 == 2)                                                                                            \
      hipExtLaunchKernelGGL((decode_generic_i1_kernel<B_, 2>), grid, dim3(256), 0, st, a.ev_start, a.ev_stop, 0, a); \
    else                                                                                                          \
      hipExtLaunchKernelGGL((decode_generic_i1_kernel<B_, 4>), grid, dim3(256), 0, st, a.ev_start, a.ev_stop, 0, a); \
  } while (0)
    if (a.fmt.bits == 2) DQ_LAUNCH_I1(2);
    else if (a.fmt.bits == 4) DQ_LAUNCH_I1(4);
    else DQ_LAUNCH_I1(8);
#undef DQ_LAUNCH_I1
    DQ_HIP_CHECK(hipGetLastError());
    return launch_combine(a, st);
  }
  switch (a.fmt.bits) {
    case 2: hipExtLaunchKernelGGL(decode_generic_kernel<2>, grid, dim3(256), 0, st, a.ev_start, a.ev_stop, 0, a); break;
    case 4: hipExtLaunchKernelGGL(decode_generic_kernel<4>, grid, dim3(256), 0, st, a.ev_start, a.ev_stop, 0, a); break;
    default: hipExtLaunchKernelGGL(decode_generic_kernel<8>, grid, dim3(256), 0, st, a.ev_start, a.ev_stop, 0, a); break;
  }
  DQ_HIP_CHECK(hipGetLastError());
  return launch_combine(a, st);
}

}  // namespace dq
