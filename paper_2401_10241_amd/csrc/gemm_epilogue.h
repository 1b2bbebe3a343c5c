// Per-element GEMM epilogues shared by the generic and the MFMA GEMM kernels.
#pragma once
#include "zb_common.h"

namespace zb {

struct EpiParams {
  int mode;
  int N;
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

}  // namespace zb
