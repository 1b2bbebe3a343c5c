// Per-element GEMM epilogues shared by the generic and the MFMA GEMM kernels.
#pragma once
#include "zb_common.h"

namespace zb {

struct EpiParams {
  int mode;
  int N;  // row stride of the outputs, aux and outf (elements)
  void* out0;
  void* out1;
  float* outf;
  const float* bias;
  const void* aux;
};

__host__ inline EpiParams make_epi(const GemmArgs& g) {
  EpiParams e;
  e.mode = g.epilogue; e.N = g.N; e.out0 = g.out0; e.out1 = g.out1; e.outf = g.outf; e.bias = g.bias; e.aux = g.aux;
  return e;
}

// one output element (m, n) with fp32 accumulator value acc
template <typename T, int MODE>
__device__ __forceinline__ void epilogue_one(const EpiParams& e, int m, int n, float acc) {
  const size_t idx = (size_t)m * e.N + n;
  if (MODE == EPI_STORE) {
    ((T*)e.out0)[idx] = from_f32<T>(acc);
  } else if (MODE == EPI_BIAS) {
    ((T*)e.out0)[idx] = from_f32<T>(acc + e.bias[n]);
  } else if (MODE == EPI_BIAS_RESID) {
    ((T*)e.out0)[idx] = from_f32<T>(acc + e.bias[n] + to_f32(((const T*)e.aux)[idx]));
  } else if (MODE == EPI_BIAS_GELU) {
    const float f = acc + e.bias[n];
    ((T*)e.out0)[idx] = from_f32<T>(f);
    ((T*)e.out1)[idx] = from_f32<T>(gelu_f(f));
  } else if (MODE == EPI_DGELU) {
    ((T*)e.out0)[idx] = from_f32<T>(acc * gelu_grad_f(to_f32(((const T*)e.aux)[idx])));
  } else {  // EPI_ACCUM_F32
    e.outf[idx] += acc;
  }
}

// One 32 x 32 MFMA accumulator tile: lane holds column n and the 16 rows m0 + 8*(v/4) + (v%4), v = 0..15
// (m0 already includes the lane's 4*(lane>>5) offset).  All reads of the tile are issued before any
// write, so the loads overlap instead of each waiting for the previous store.  (The fp32 accumulate of
// the wgrad GEMM is not an epilogue in the MFMA path: its kernel starts the accumulators from C.)
template <typename T, int MODE>
__device__ __forceinline__ void epilogue_tile(const EpiParams& e, int m0, int n, const f32x16& acc) {
  size_t idx[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) idx[v] = (size_t)(m0 + (v >> 2) * 8 + (v & 3)) * e.N + n;
  if (MODE == EPI_PARTIAL) {  // e.outf already points at this K slice's [M,N] plane
#pragma unroll
    for (int v = 0; v < 16; ++v) e.outf[idx[v]] = acc[v];
  } else if (MODE == EPI_BIAS_RESID || MODE == EPI_DGELU) {
    float a[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) a[v] = to_f32(((const T*)e.aux)[idx[v]]);
    const float b = MODE == EPI_BIAS_RESID ? e.bias[n] : 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v)
      ((T*)e.out0)[idx[v]] = from_f32<T>(MODE == EPI_BIAS_RESID ? acc[v] + b + a[v] : acc[v] * gelu_grad_f(a[v]));
  } else if (MODE == EPI_BIAS_GELU) {
    const float b = e.bias[n];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float f = acc[v] + b;
      ((T*)e.out0)[idx[v]] = from_f32<T>(f);
      ((T*)e.out1)[idx[v]] = from_f32<T>(gelu_f(f));
    }
  } else {
    const float b = MODE == EPI_BIAS ? e.bias[n] : 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) ((T*)e.out0)[idx[v]] = from_f32<T>(acc[v] + b);
  }
}

}  // namespace zb
