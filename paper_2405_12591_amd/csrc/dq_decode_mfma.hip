// Matrix-core decode attention over the compressed cache for the format
//   bits = 4, head_dim = 128, j1 = 16, j2 = 8, group = 128, block_tokens % 128 == 0,
//   q_heads / kv_heads in {1, 2, 4}.
//
// This is the fused "dequantize + multiply the local tensors" of Section 3.2 (arXiv
// 2405.12591) carried through the attention that follows it.  Per 128-token tile, one
// wavefront
//   1. folds the keys' small tensor into the query,  q'[r, b2] = sum_b1 T_S^K[b1, r] q[b1, b2],
//      with one 16x16x16 f16 MFMA, and splits q' into fp16 hi + lo parts (columns of B);
//   2. streams the 4-bit key codes with 128-bit loads, turns each 32-bit word into eight
//      fp16 values 64 + u by mask/shift/or (u = code + 8, so the value is code + 72), and
//      contracts them with q' on 16x16x32 f16 MFMAs; the constant 72 is removed by starting
//      the accumulator at -72 * sum(q');
//   3. runs the online softmax with one or two tokens per lane (scores cross from the MFMA
//      layout through wave-private LDS), multiplies p by the value step and splits it into
//      fp16 hi + lo, again as B columns;
//   4. streams the value codes (stored token-contiguous) the same way, o'[r, b2] = sum_t p'_t c;
//   5. applies the values' small tensor with fp32 16x16x4 MFMAs,
//      acc[b1, b2] = alpha * acc + sum_r T_S^V[b1, r] o'[r, b2].
// Sixteen B columns are available; a query head uses two (hi, lo), so up to eight heads
// sharing a kv head ride on the same code stream.
//
// MFMA operand layouts used below (lane l: n = l % 16, g = l / 16):
//   A[m][k]: lane holds row m = n, k = S*g + i (S = values per lane);  B[k][n]: column n, same k;
//   D[m][n]: lane holds column n, rows m = 4*g + i.
#include "dq_decode.h"

namespace dq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kCodeOffset = 72.0f;  // fp16 pattern 0x5400 | (u << 4) is 64 + u = code + 72

// Eight 4-bit fields of x -> eight fp16 values (64 + field), slot order [1,5,3,7,0,4,2,6].
__device__ __forceinline__ half8 unpack8(uint32_t x) {
  const uint32_t M = 0x00F000F0u, K = 0x54005400u;
  u32x4 v;
  v.x = (x & M) | K;          // fields 1, 5
  v.y = ((x >> 8) & M) | K;   // fields 3, 7
  v.z = ((x << 4) & M) | K;   // fields 0, 4
  v.w = ((x >> 4) & M) | K;   // fields 2, 6
  return __builtin_bit_cast(half8, v);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ __forceinline__ uint32_t pack_half2(_Float16 lo, _Float16 hi) {
  half2v h = {lo, hi};
  return __builtin_bit_cast(uint32_t, h);
}

// 2^e as a float for -126 <= e <= 127
__device__ __forceinline__ float pow2i(int e) {
  return __builtin_bit_cast(float, (uint32_t)(e + 127) << 23);
}

template <int R>
__global__ __launch_bounds__(256, 2) void decode_mfma_kernel(DecodeArgs a) {
  constexpr int NC = 2 * R;            // B columns in use: (hi, lo) per query head
  constexpr int F = (R + 1) / 2;       // fold MFMAs (two heads each)
  constexpr int D = 128, J1 = 16, J2 = 8, ROWB = 64;
  constexpr int WAVE_LDS = NC * 1024;  // Qs NC*256 + Ps NC*256 + Ss NC*512 bytes
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * WAVE_LDS];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, g = lane >> 4;
  const int sa = lane >> 2, sk = lane & 3;  // softmax layout: token group sa, tokens sk and sk + 4
  const int split = blockIdx.x;
  const int bh = blockIdx.y;
  const int H = a.cache.kv_heads, NB = a.cache.block_capacity;
  const int b = bh / H, h = bh % H;
  const int tpb = a.fmt.block_tokens / kTileTokens;
  const long codes_per_block = (long)a.fmt.block_tokens * ROWB;
  const long scales_per_block = a.fmt.block_tokens;

  const int S = min(max(a.seq_lens[b], 0), a.max_seq_len);
  const int tiles_total = (S + kTileTokens - 1) / kTileTokens;
  const int tps = (tiles_total + a.n_split - 1) / a.n_split;
  const int tile_begin = split * tps;
  const int tile_end = min(tile_begin + tps, tiles_total);

  unsigned char* wl = smem + wave * WAVE_LDS;
  _Float16* Qs = reinterpret_cast<_Float16*>(wl);                // [NC][16 r][8 slots]
  uint32_t* Ps = reinterpret_cast<uint32_t*>(wl + NC * 256);     // [NC][16 groups][4 pairs]
  float* Ss = reinterpret_cast<float*>(wl + NC * 512);           // [NC][128 tokens]

  // ---- loop-invariant B operands of the fold: q[k = b1][n' = (b2, head)] ----
  half4 bq[F];
  {
    const int b2 = n & 7;
#pragma unroll
    for (int f = 0; f < F; ++f) {
      const int hd = 2 * f + (n >> 3);
      half4 v = {0, 0, 0, 0};
      if (hd < R) {
        const uint16_t* qp = a.q + ((long)b * a.q_heads + (long)h * R + hd) * D;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __builtin_bit_cast(_Float16, qp[(4 * g + i) * J2 + b2]);
      }
      bq[f] = v;
    }
  }
  half8 neg_off;
#pragma unroll
  for (int i = 0; i < 8; ++i) neg_off[i] = (_Float16)(-kCodeOffset);

  float m_run[R], l_run[R];
#pragma unroll
  for (int hd = 0; hd < R; ++hd) { m_run[hd] = -INFINITY; l_run[hd] = 0.f; }
  f32x4 acc[J2];
#pragma unroll
  for (int b2 = 0; b2 < J2; ++b2) acc[b2] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const float qk_scale = a.scale * kLog2e;
  const int slotpos = (0x37152604 >> (4 * (n & 7))) & 7;  // b2 -> slot: 0->4 1->0 2->6 3->2 4->5 5->1 6->7 7->3
  const int pairpos = (0x1302 >> (4 * sk)) & 3;            // sk -> pair register: 0->2 1->0 2->3 3->1

  // ---- prefetch the first tile's key codes and small tensor ----
  u32x4 kreg[8];
  u32x2 ksm = {0, 0};
  int tile = tile_begin + wave;
  if (tile < tile_end) {
    const long blkid = (long)bh * NB + tile / tpb;
    const unsigned char* kc = a.cache.k_codes + blkid * codes_per_block + (long)(tile % tpb) * kTileTokens * ROWB;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      kreg[j] = *reinterpret_cast<const u32x4*>(kc + (16 * j + n) * ROWB + 16 * g);
    ksm = *reinterpret_cast<const u32x2*>(a.cache.k_small + blkid * (J1 * J1) + n * J1 + 4 * g);
  }

  for (; tile < tile_end; tile += 4) {
    const int blk = tile / tpb, tib = tile % tpb;
    const long blkid = (long)bh * NB + blk;
    const int tok0 = tile * kTileTokens;

    // ---- issue this tile's value-side loads ----
    u32x4 vreg[8];
    {
      const unsigned char* vc = a.cache.v_codes + blkid * codes_per_block + (long)tib * kTileTokens * ROWB;
#pragma unroll
      for (int b2 = 0; b2 < J2; ++b2)
        vreg[b2] = *reinterpret_cast<const u32x4*>(vc + b2 * (J1 * 64) + n * 64 + 16 * g);
    }
    const u32x2 vsm = *reinterpret_cast<const u32x2*>(a.cache.v_small + blkid * (J1 * J1) + n * J1 + 4 * g);
    const uint16_t* ksc = a.cache.k_scales + blkid * scales_per_block + tib * kTileTokens;
    const uint16_t* vsc = a.cache.v_scales + blkid * scales_per_block + tib * kTileTokens;
    const int tA = 8 * sa + sk, tB = tA + 4;
    const uint16_t dkA_b = ksc[tA], dkB_b = ksc[tB], dvA_b = vsc[tA], dvB_b = vsc[tB];

    // ---- 1. fold T_S^K into q, normalise, split hi/lo, stage as B operands ----
    float q_unscale;
    {
      const half4 aK = __builtin_bit_cast(half4, ksm);
      f32x4 fd[F];
      float amax = 0.f;
#pragma unroll
      for (int f = 0; f < F; ++f) {
        fd[f] = __builtin_amdgcn_mfma_f32_16x16x16f16(aK, bq[f], (f32x4){0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) amax = fmaxf(amax, fabsf(fd[f][i]));
      }
      amax = wave_max(amax) * qk_scale;
      // bring the largest |q'| into [1024, 2048) so that hi and lo are both well inside fp16
      int e = 0;
      if (amax > 0.f && amax < INFINITY) e = __builtin_amdgcn_frexp_expf(amax);  // amax = f * 2^e, f in [0.5, 1)
      e = max(min(e, 100), -100);
      const float qn = qk_scale * pow2i(11 - e);
      q_unscale = pow2i(e - 11);
#pragma unroll
      for (int f = 0; f < F; ++f) {
        const int hd = 2 * f + (n >> 3);
        if (hd < R) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float v = fd[f][i] * qn;
            const _Float16 hi = (_Float16)v;
            const _Float16 lo = (_Float16)(v - (float)hi);
            const int r = 4 * g + i;
            Qs[((2 * hd) * 16 + r) * 8 + slotpos] = hi;
            Qs[((2 * hd + 1) * 16 + r) * 8 + slotpos] = lo;
          }
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
    half8 bqs[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      u32x4 t = {0, 0, 0, 0};
      if (n < NC) t = *reinterpret_cast<const u32x4*>(Qs + (n * 16 + 4 * g + w) * 8);
      bqs[w] = __builtin_bit_cast(half8, t);
    }

    // ---- 2. scores: S[t][col] = sum_c (c + 72) q''[col][c] - 72 sum_c q''[col][c] ----
    {
      f32x4 cinit = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < 4; ++w) cinit = __builtin_amdgcn_mfma_f32_16x16x32_f16(neg_off, bqs[w], cinit, 0, 0, 0);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        f32x4 s = cinit;
        s = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack8(kreg[j].x), bqs[0], s, 0, 0, 0);
        s = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack8(kreg[j].y), bqs[1], s, 0, 0, 0);
        s = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack8(kreg[j].z), bqs[2], s, 0, 0, 0);
        s = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack8(kreg[j].w), bqs[3], s, 0, 0, 0);
        if (n < NC) *reinterpret_cast<f32x4*>(Ss + n * kTileTokens + 16 * j + 4 * g) = s;
      }
    }

    // ---- prefetch the next tile's key codes ----
    {
      const int nt = tile + 4;
      if (nt < tile_end) {
        const long nblkid = (long)bh * NB + nt / tpb;
        const unsigned char* kc = a.cache.k_codes + nblkid * codes_per_block + (long)(nt % tpb) * kTileTokens * ROWB;
#pragma unroll
        for (int j = 0; j < 8; ++j)
          kreg[j] = *reinterpret_cast<const u32x4*>(kc + (16 * j + n) * ROWB + 16 * g);
        ksm = *reinterpret_cast<const u32x2*>(a.cache.k_small + nblkid * (J1 * J1) + n * J1 + 4 * g);
      }
    }
    __builtin_amdgcn_wave_barrier();

    // ---- 3. online softmax, tokens tA and tB per lane ----
    const bool okA = (tok0 + tA) < S, okB = (tok0 + tB) < S;
    const float dkA = h2f(dkA_b) * q_unscale, dkB = h2f(dkB_b) * q_unscale;
    const float dvA = okA ? h2f(dvA_b) : 0.f, dvB = okB ? h2f(dvB_b) : 0.f;
    float v_unscale;
    float dvAs, dvBs;
    {
      const float dvmax = wave_max(fmaxf(dvA, dvB));
      int e = 0;
      if (dvmax > 0.f && dvmax < INFINITY) e = __builtin_amdgcn_frexp_expf(dvmax);
      const float vs = pow2i(12 - e);  // p * step * vs <= 4096
      v_unscale = pow2i(e - 12);
      dvAs = dvA * vs; dvBs = dvB * vs;
    }
    float alpha[R];
#pragma unroll
    for (int hd = 0; hd < R; ++hd) {
      float sA = (Ss[(2 * hd) * kTileTokens + tA] + Ss[(2 * hd + 1) * kTileTokens + tA]) * dkA;
      float sB = (Ss[(2 * hd) * kTileTokens + tB] + Ss[(2 * hd + 1) * kTileTokens + tB]) * dkB;
      sA = okA ? sA : -INFINITY;
      sB = okB ? sB : -INFINITY;
      const float mt = wave_max(fmaxf(sA, sB));
      const float m_new = fmaxf(m_run[hd], mt);          // finite: the tile has a valid token
      alpha[hd] = __builtin_amdgcn_exp2f(m_run[hd] - m_new);
      const float pA = __builtin_amdgcn_exp2f(sA - m_new);
      const float pB = __builtin_amdgcn_exp2f(sB - m_new);
      l_run[hd] = l_run[hd] * alpha[hd] + (pA + pB);
      m_run[hd] = m_new;
      const float ppA = okA ? pA * dvAs : 0.f;
      const float ppB = okB ? pB * dvBs : 0.f;
      const _Float16 hA = (_Float16)ppA, hB = (_Float16)ppB;
      const _Float16 lA = (_Float16)(ppA - (float)hA), lB = (_Float16)(ppB - (float)hB);
      Ps[((2 * hd) * 16 + sa) * 4 + pairpos] = pack_half2(hA, hB);
      Ps[((2 * hd + 1) * 16 + sa) * 4 + pairpos] = pack_half2(lA, lB);
    }
    __builtin_amdgcn_wave_barrier();

    // ---- 4 + 5. o' = P' V' per b2, then the small-tensor epilogue ----
    half8 bp[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      u32x4 t = {0, 0, 0, 0};
      if (n < NC) t = *reinterpret_cast<const u32x4*>(Ps + (n * 16 + 4 * g + v) * 4);
      bp[v] = __builtin_bit_cast(half8, t);
    }
    float alpha_col = 1.f;
#pragma unroll
    for (int hd = 0; hd < R; ++hd) alpha_col = ((n >> 1) == hd) ? alpha[hd] : alpha_col;
    float aT[4];
    {
      const half4 t = __builtin_bit_cast(half4, vsm);
#pragma unroll
      for (int i = 0; i < 4; ++i) aT[i] = (float)t[i] * v_unscale;
    }
    f32x4 cinitv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int v = 0; v < 4; ++v) cinitv = __builtin_amdgcn_mfma_f32_16x16x32_f16(neg_off, bp[v], cinitv, 0, 0, 0);
    const bool rescale = __any(alpha_col != 1.f);
#pragma unroll
    for (int b2 = 0; b2 < J2; ++b2) {
      f32x4 o = cinitv;
      o = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack8(vreg[b2].x), bp[0], o, 0, 0, 0);
      o = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack8(vreg[b2].y), bp[1], o, 0, 0, 0);
      o = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack8(vreg[b2].z), bp[2], o, 0, 0, 0);
      o = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack8(vreg[b2].w), bp[3], o, 0, 0, 0);
      f32x4 c = acc[b2];
      if (rescale) c *= alpha_col;
#pragma unroll
      for (int i = 0; i < 4; ++i) c = __builtin_amdgcn_mfma_f32_16x16x4f32(aT[i], o[i], c, 0, 0, 0);
      acc[b2] = c;
    }
    __builtin_amdgcn_wave_barrier();
  }

  // ---- merge the four waves of the workgroup, write one partial per query head ----
  float* Macc = reinterpret_cast<float*>(wl);            // [R][128] per wave (reuses the wave's LDS)
  float* Mml = Macc + R * D;                             // [R] m, [R] l
#pragma unroll
  for (int hd = 0; hd < R; ++hd) l_run[hd] = wave_sum(l_run[hd]);
#pragma unroll
  for (int b2 = 0; b2 < J2; ++b2) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float v = acc[b2][i] + __shfl_xor(acc[b2][i], 1);  // hi column + lo column
      if (n < NC && !(n & 1)) Macc[(n >> 1) * D + (4 * g + i) * J2 + b2] = v;
    }
  }
  if (lane == 0) {
#pragma unroll
    for (int hd = 0; hd < R; ++hd) { Mml[hd] = m_run[hd]; Mml[R + hd] = l_run[hd]; }
  }
  __syncthreads();
  for (int idx = tid; idx < R * D; idx += 256) {
    const int hd = idx / D, c = idx % D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, reinterpret_cast<const float*>(smem + w * WAVE_LDS)[R * D + hd]);
    float o = 0.f, L = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float* base = reinterpret_cast<const float*>(smem + w * WAVE_LDS);
      const float mw = base[R * D + hd];
      const float wgt = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - M);
      o = fmaf(base[hd * D + c], wgt, o);
      L = fmaf(base[R * D + R + hd], wgt, L);
    }
    float* part = a.partials + (((long)b * a.q_heads + (long)h * R + hd) * a.n_split + split) * (D + 2);
    part[c] = o;
    if (c == 0) { part[D] = M * kLn2; part[D + 1] = L; }
  }
}

bool mfma_supported(const dq_format* f, int q_heads, int kv_heads) {
  if (!format_ok(f) || kv_heads <= 0 || q_heads % kv_heads) return false;
  const int rep = q_heads / kv_heads;
  if (rep != 1 && rep != 2 && rep != 4) return false;
  return f->bits == 4 && f->head_dim == 128 && f->j1 == 16 && f->j2 == 8 && f->group == 128;
}

int32_t launch_combine(const DecodeArgs& a, hipStream_t st);

int32_t launch_decode_mfma(const DecodeArgs& a, hipStream_t st) {
  const dim3 grid(a.n_split, a.cache.batch * a.cache.kv_heads);
  const int rep = a.q_heads / a.cache.kv_heads;
  switch (rep) {
    case 1: hipLaunchKernelGGL(decode_mfma_kernel<1>, grid, dim3(256), 0, st, a); break;
    case 2: hipLaunchKernelGGL(decode_mfma_kernel<2>, grid, dim3(256), 0, st, a); break;
    case 4: hipLaunchKernelGGL(decode_mfma_kernel<4>, grid, dim3(256), 0, st, a); break;
    default: return DQ_EINVAL;
  }
  DQ_HIP_CHECK(hipGetLastError());
  return launch_combine(a, st);
}

}  // namespace dq
