// Generic strided GEMM on the vector ALUs (fp32 accumulate): every shape, both data types, all
// three operand forms (forward X*W, dgrad dY*W^T, wgrad X^T*dY).  It carries the fp32 workload and
// any bf16 shape the MFMA kernel does not take.  64x64 output tile per 256-thread workgroup,
// K walked in steps of 16 through LDS, 4x4 outputs per lane.
#include "gemm_epilogue.h"

namespace zb {

template <typename T> hipError_t launch_gemm_mfma(const GemmArgs& g, hipStream_t s, bool* taken);
template <typename T> hipError_t launch_wgrad_multi_mfma(const WgradMultiArgs& w, hipStream_t s, bool* taken);

namespace {

constexpr int TM = 64, TN = 64, TK = 16;

template <typename T, int MODE>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T* __restrict__ A, const T* __restrict__ B, int M,
                                                          int N, int K, long a_sm, long a_sk, long b_sk, long b_sn,
                                                          EpiParams epi) {
  __shared__ float As[TK][TM + 4];
  __shared__ float Bs[TK][TN + 4];
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < K; k0 += TK) {
    // 64x16 elements per operand, 4 per thread; lanes run along whichever index is contiguous
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int e = r * 256 + threadIdx.x;
      int am, ak, bn, bk;
      if (a_sk == 1) { ak = e & 15; am = e >> 4; } else { am = e & 63; ak = e >> 6; }
      if (b_sk == 1) { bk = e & 15; bn = e >> 4; } else { bn = e & 63; bk = e >> 6; }
      float av = 0.f, bv = 0.f;
      if (m0 + am < M && k0 + ak < K) av = to_f32(A[(long)(m0 + am) * a_sm + (long)(k0 + ak) * a_sk]);
      if (n0 + bn < N && k0 + bk < K) bv = to_f32(B[(long)(k0 + bk) * b_sk + (long)(n0 + bn) * b_sn]);
      As[ak][am] = av;
      Bs[bk][bn] = bv;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n < N) epilogue_one<T, MODE>(epi, m, n, acc[i][j]);
    }
  }
}

template <typename T, int MODE> hipError_t run_generic(const GemmArgs& g, hipStream_t s) {
  dim3 grid((g.N + TN - 1) / TN, (g.M + TM - 1) / TM);
  gemm_generic_kernel<T, MODE><<<grid, 256, 0, s>>>((const T*)g.A, (const T*)g.B, g.M, g.N, g.K, g.a_sm, g.a_sk,
                                                   g.b_sk, g.b_sn, make_epi(g));
  return hipGetLastError();
}

}  // namespace

template <typename T> hipError_t launch_gemm_generic(const GemmArgs& g, hipStream_t s) {
  switch (g.epilogue) {
    case EPI_STORE: return run_generic<T, EPI_STORE>(g, s);
    case EPI_BIAS: return run_generic<T, EPI_BIAS>(g, s);
    case EPI_BIAS_RESID: return run_generic<T, EPI_BIAS_RESID>(g, s);
    case EPI_BIAS_GELU: return run_generic<T, EPI_BIAS_GELU>(g, s);
    case EPI_DGELU: return run_generic<T, EPI_DGELU>(g, s);
    case EPI_ACCUM_F32: return run_generic<T, EPI_ACCUM_F32>(g, s);
  }
  return hipErrorInvalidValue;
}

template <typename T> hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
  if (!((g.a_sm == 1) ^ (g.a_sk == 1)) && !(g.M == 1 || g.K == 1)) return hipErrorInvalidValue;
  if (!((g.b_sk == 1) ^ (g.b_sn == 1)) && !(g.N == 1 || g.K == 1)) return hipErrorInvalidValue;
  bool taken = false;
  hipError_t e = launch_gemm_mfma<T>(g, s, &taken);
  if (taken) return e;
  if (g.group >= 2) {  // no grouped kernel for this shape: the pairs one after the other
    if (g.group > kGemmGroupMax || g.epilogue != EPI_ACCUM_F32) return hipErrorInvalidValue;
    for (int i = 0; i < g.group; ++i) {
      GemmArgs one = g;
      one.group = 0;
      one.A = g.group_a[i];
      one.B = g.group_b[i];
      if ((e = launch_gemm<T>(one, s)) != hipSuccess) return e;
    }
    return hipSuccess;
  }
  return launch_gemm_generic<T>(g, s);
}

template <typename T> hipError_t launch_wgrad_multi(const WgradMultiArgs& w, hipStream_t s) {
  if (w.nprob < 1 || w.nprob > kWgradMaxProblems || w.ngroup < 1 || w.ngroup > kGemmGroupMax ||
      w.nprob * w.ngroup > kWgradMaxPairs || w.K <= 0)
    return hipErrorInvalidValue;
  bool taken = false;
  hipError_t e = launch_wgrad_multi_mfma<T>(w, s, &taken);
  if (taken) return e;
  for (int q = 0; q < w.nprob; ++q) {  // problem by problem (fp32, or a shape the MFMA kernel does not take)
    GemmArgs g{};
    g.M = w.M[q]; g.N = w.N[q]; g.K = w.K;
    g.a_sm = 1; g.a_sk = w.M[q]; g.b_sk = w.N[q]; g.b_sn = 1;
    g.epilogue = EPI_ACCUM_F32; g.outf = w.outf[q];
    g.A = w.a[q * w.ngroup]; g.B = w.b[q * w.ngroup];
    if (w.ngroup >= 2) {
      g.group = w.ngroup;
      for (int i = 0; i < w.ngroup; ++i) { g.group_a[i] = w.a[q * w.ngroup + i]; g.group_b[i] = w.b[q * w.ngroup + i]; }
    }
    if ((e = launch_gemm<T>(g, s)) != hipSuccess) return e;
  }
  return hipSuccess;
}

template hipError_t launch_wgrad_multi<float>(const WgradMultiArgs&, hipStream_t);
template hipError_t launch_wgrad_multi<bf16_t>(const WgradMultiArgs&, hipStream_t);
template hipError_t launch_gemm<float>(const GemmArgs&, hipStream_t);
template hipError_t launch_gemm<bf16_t>(const GemmArgs&, hipStream_t);
template hipError_t launch_gemm_generic<float>(const GemmArgs&, hipStream_t);
template hipError_t launch_gemm_generic<bf16_t>(const GemmArgs&, hipStream_t);

}  // namespace zb
