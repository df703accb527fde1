// Instrumented build only (-DDQ_TIMELINE; the product library holds nothing of this file): a probe
// of how matrix and vector instructions of one SIMD share its issue.  Four waves per SIMD run a
// loop of four independent matrix instructions of one kind, sixteen independent fp32 FMAs, or
// both; the time per loop body tells whether the two kinds run side by side.  The decode kernel's
// choice between matrix and vector instructions for its small-tensor epilogue rests on the figures.
#include "dq_common.h"

#ifdef DQ_TIMELINE
namespace dq {

typedef float pf32x4 __attribute__((ext_vector_type(4)));
typedef int pi32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 phalf4 __attribute__((ext_vector_type(4)));

// KIND: 0 none, 1 v_mfma_f32_16x16x4_f32, 2 v_mfma_f32_16x16x16_f16, 3 v_mfma_i32_16x16x64_i8,
// 4 v_mfma_f64_16x16x4_f64
template <int KIND, bool FMA>
__global__ __launch_bounds__(256) void issue_probe_kernel(float* sink, int iters) {
  const int l = threadIdx.x;
  pf32x4 c[4];
  pi32x4 d[4];
  typedef double pf64x4 __attribute__((ext_vector_type(4)));
  pf64x4 e[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { c[i] = pf32x4{0.f, 0.f, 0.f, 0.f}; d[i] = pi32x4{0, 0, 0, 0}; e[i] = pf64x4{0.0, 0.0, 0.0, 0.0}; }
  float x[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = l * 0.001f + i;
  const float a = 1.0f + l * 1e-6f, b = 0.5f;
  const double ad = 1.0 + l * 1e-9, bd = 0.5;
  const phalf4 h = {(_Float16)1.0f, (_Float16)0.5f, (_Float16)0.25f, (_Float16)2.0f};
  const pi32x4 bi = {0x01020304, 0x01010101, 0x02020202, 0x03030303};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int rep = 0; rep < 4; ++rep) {   // four loop bodies per trip: the loop's own instructions weigh little
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (KIND == 1) c[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c[i], 0, 0, 0);
        if (KIND == 2) c[i] = __builtin_amdgcn_mfma_f32_16x16x16f16(h, h, c[i], 0, 0, 0);
        if (KIND == 3) d[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(bi, bi, d[i], 0, 0, 0);
        if (KIND == 4) e[i] = __builtin_amdgcn_mfma_f64_16x16x4f64(ad, bd, e[i], 0, 0, 0);
      }
      if (FMA) {
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = __builtin_fmaf(x[i], a, b);
      }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += x[i];
#pragma unroll
  for (int i = 0; i < 4; ++i) s += c[i][i] + (float)d[i][i] + (float)e[i][i];
  if (s == 12345.678f) sink[0] = s;   // never true: keeps the loop alive
}

}  // namespace dq

// Launches the probe (1024 workgroups of four waves: four waves per SIMD) on the stream; the caller
// times it.  kind as above, fma != 0 adds the vector FMAs.
extern "C" int32_t dq_debug_issue_probe(int32_t kind, int32_t fma, int32_t iters, float* sink, void* hip_stream) {
  using namespace dq;
  if (kind < 0 || kind > 4 || iters < 1 || iters > (1 << 20) || !sink || (kind == 0 && !fma)) return DQ_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  const dim3 grid(1024), block(256);
#define DQ_PROBE(K_)                                                                            \
  do {                                                                                          \
    if (fma) hipLaunchKernelGGL((issue_probe_kernel<K_, true>), grid, block, 0, st, sink, iters);  \
    else hipLaunchKernelGGL((issue_probe_kernel<K_, false>), grid, block, 0, st, sink, iters);     \
  } while (0)
  if (kind == 0) hipLaunchKernelGGL((issue_probe_kernel<0, true>), grid, block, 0, st, sink, iters);
  else if (kind == 1) DQ_PROBE(1);
  else if (kind == 2) DQ_PROBE(2);
  else if (kind == 3) DQ_PROBE(3);
  else DQ_PROBE(4);
#undef DQ_PROBE
  DQ_HIP_CHECK(hipGetLastError());
  return DQ_OK;
}
#endif
