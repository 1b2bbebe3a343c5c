// Causal multi-head attention, forward and backward, on the vector ALUs: one wavefront per
// (sample, head, row).  Any head size and sequence length; fp32 arithmetic.  It carries the fp32
// workload and any bf16 shape the MFMA attention kernels do not take.
//
// forward (per query row i):   s_j = q_i.k_j / sqrt(d) for j <= i;  p = softmax(s);  o_i = sum_j p_j v_j;
//                              lse_i = log sum_j exp(s_j)  (kept for the backward)
// backward: D_i = dO_i.O_i;  p_ij = exp(s_ij - lse_i);  dP_ij = dO_i.v_j;  dS_ij = p_ij (dP_ij - D_i);
//           dQ_i = sum_j dS_ij k_j / sqrt(d);  dK_j = sum_i dS_ij q_i / sqrt(d);  dV_j = sum_i p_ij dO_i
#include "zb_common.h"

namespace zb {

template <typename T> hipError_t launch_attention_fwd_mfma(const AttnArgs& a, hipStream_t s, bool* taken);
template <typename T> hipError_t launch_attention_bwd_mfma(const AttnArgs& a, hipStream_t s, bool* taken);

namespace {

template <typename T>
__device__ __forceinline__ float dot_row(const float* __restrict__ qs, const T* __restrict__ k, int d) {
  float acc = 0.f;
  for (int e = 0; e < d; ++e) acc = fmaf(qs[e], to_f32(k[e]), acc);
  return acc;
}

template <typename T>
__global__ __launch_bounds__(64) void attn_fwd_row_kernel(const T* __restrict__ qkv, T* __restrict__ out,
                                                          float* __restrict__ lse, int s, int a, int d) {
  extern __shared__ float sm[];
  float* qs = sm;       // [d]
  float* ps = sm + d;   // [s]
  const int i = blockIdx.x, head = blockIdx.y, bi = blockIdx.z, lane = threadIdx.x;
  const int h = a * d;
  const size_t tok0 = (size_t)bi * s;
  const float scale = 1.0f / sqrtf((float)d);
  const T* q = qkv + (tok0 + i) * 3 * h + head * d;
  for (int e = lane; e < d; e += 64) qs[e] = to_f32(q[e]);
  __syncthreads();
  float mx = -INFINITY;
  for (int j = lane; j <= i; j += 64) {
    const float sc = dot_row(qs, qkv + (tok0 + j) * 3 * h + h + head * d, d) * scale;
    ps[j] = sc;
    mx = fmaxf(mx, sc);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j <= i; j += 64) {
    const float p = expf(ps[j] - mx);
    ps[j] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  if (lane == 0) lse[((size_t)bi * a + head) * s + i] = mx + logf(sum);
  __syncthreads();
  const float inv = 1.0f / sum;
  for (int e = lane; e < d; e += 64) {
    float acc = 0.f;
    const T* v = qkv + tok0 * 3 * h + 2 * h + head * d + e;
    for (int j = 0; j <= i; ++j) acc = fmaf(ps[j], to_f32(v[(size_t)j * 3 * h]), acc);
    out[(tok0 + i) * h + head * d + e] = from_f32<T>(acc * inv);
  }
}

template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dq_kernel(const T* __restrict__ qkv, const T* __restrict__ o,
                                                         const T* __restrict__ dout, const float* __restrict__ lse,
                                                         float* __restrict__ dvec, T* __restrict__ dqkv, int s,
                                                         int a, int d) {
  extern __shared__ float sm[];
  float* qs = sm;           // [d]
  float* dos = sm + d;      // [d]
  float* ds = sm + 2 * d;   // [s]
  const int i = blockIdx.x, head = blockIdx.y, bi = blockIdx.z, lane = threadIdx.x;
  const int h = a * d;
  const size_t tok0 = (size_t)bi * s;
  const float scale = 1.0f / sqrtf((float)d);
  float dpart = 0.f;
  for (int e = lane; e < d; e += 64) {
    qs[e] = to_f32(qkv[(tok0 + i) * 3 * h + head * d + e]);
    const float g = to_f32(dout[(tok0 + i) * h + head * d + e]);
    dos[e] = g;
    dpart += g * to_f32(o[(tok0 + i) * h + head * d + e]);
  }
  const float D = wave_sum(dpart);
  const size_t li = ((size_t)bi * a + head) * s + i;
  if (lane == 0) dvec[li] = D;
  const float l = lse[li];
  __syncthreads();
  for (int j = lane; j <= i; j += 64) {
    const T* krow = qkv + (tok0 + j) * 3 * h + h + head * d;
    const float p = expf(dot_row(qs, krow, d) * scale - l);
    const float dp = dot_row(dos, krow + h, d);
    ds[j] = p * (dp - D);
  }
  __syncthreads();
  for (int e = lane; e < d; e += 64) {
    float acc = 0.f;
    const T* k = qkv + tok0 * 3 * h + h + head * d + e;
    for (int j = 0; j <= i; ++j) acc = fmaf(ds[j], to_f32(k[(size_t)j * 3 * h]), acc);
    dqkv[(tok0 + i) * 3 * h + head * d + e] = from_f32<T>(acc * scale);
  }
}

template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dkv_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                          const float* __restrict__ lse,
                                                          const float* __restrict__ dvec, T* __restrict__ dqkv,
                                                          int s, int a, int d) {
  extern __shared__ float sm[];
  float* ks = sm;               // [d]
  float* vs = sm + d;           // [d]
  float* ps = sm + 2 * d;       // [s]
  float* ds = sm + 2 * d + s;   // [s]
  const int j = blockIdx.x, head = blockIdx.y, bi = blockIdx.z, lane = threadIdx.x;
  const int h = a * d;
  const size_t tok0 = (size_t)bi * s;
  const float scale = 1.0f / sqrtf((float)d);
  for (int e = lane; e < d; e += 64) {
    ks[e] = to_f32(qkv[(tok0 + j) * 3 * h + h + head * d + e]);
    vs[e] = to_f32(qkv[(tok0 + j) * 3 * h + 2 * h + head * d + e]);
  }
  __syncthreads();
  const size_t l0 = ((size_t)bi * a + head) * s;
  for (int i = j + lane; i < s; i += 64) {
    const float p = expf(dot_row(ks, qkv + (tok0 + i) * 3 * h + head * d, d) * scale - lse[l0 + i]);
    const float dp = dot_row(vs, dout + (tok0 + i) * h + head * d, d);
    ps[i] = p;
    ds[i] = p * (dp - dvec[l0 + i]);
  }
  __syncthreads();
  for (int e = lane; e < d; e += 64) {
    float dk = 0.f, dv = 0.f;
    for (int i = j; i < s; ++i) {
      dk = fmaf(ds[i], to_f32(qkv[(tok0 + i) * 3 * h + head * d + e]), dk);
      dv = fmaf(ps[i], to_f32(dout[(tok0 + i) * h + head * d + e]), dv);
    }
    dqkv[(tok0 + j) * 3 * h + h + head * d + e] = from_f32<T>(dk * scale);
    dqkv[(tok0 + j) * 3 * h + 2 * h + head * d + e] = from_f32<T>(dv);
  }
}

}  // namespace

template <typename T> hipError_t launch_attention_fwd_generic(const AttnArgs& a, hipStream_t s) {
  const size_t smem = (size_t)(a.d + a.s) * sizeof(float);
  if (smem > 60 * 1024) return hipErrorInvalidValue;
  dim3 grid(a.s, a.a, a.b);
  attn_fwd_row_kernel<T><<<grid, 64, smem, s>>>((const T*)a.qkv, (T*)a.out, a.lse, a.s, a.a, a.d);
  return hipGetLastError();
}

template <typename T> hipError_t launch_attention_bwd_generic(const AttnArgs& a, hipStream_t s) {
  const size_t smem = (size_t)(2 * a.d + 2 * a.s) * sizeof(float);
  if (smem > 60 * 1024) return hipErrorInvalidValue;
  dim3 grid(a.s, a.a, a.b);
  attn_bwd_dq_kernel<T><<<grid, 64, smem, s>>>((const T*)a.qkv, (const T*)a.o, (const T*)a.dout, a.lse, a.dvec,
                                               (T*)a.dqkv, a.s, a.a, a.d);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  attn_bwd_dkv_kernel<T><<<grid, 64, smem, s>>>((const T*)a.qkv, (const T*)a.dout, a.lse, a.dvec, (T*)a.dqkv, a.s,
                                                a.a, a.d);
  return hipGetLastError();
}

template <typename T> hipError_t launch_attention_fwd(const AttnArgs& a, hipStream_t s) {
  if (a.b <= 0 || a.s <= 0 || a.a <= 0 || a.d <= 0) return hipErrorInvalidValue;
  bool taken = false;
  hipError_t e = launch_attention_fwd_mfma<T>(a, s, &taken);
  if (taken) return e;
  return launch_attention_fwd_generic<T>(a, s);
}
template <typename T> hipError_t launch_attention_bwd(const AttnArgs& a, hipStream_t s) {
  if (a.b <= 0 || a.s <= 0 || a.a <= 0 || a.d <= 0) return hipErrorInvalidValue;
  bool taken = false;
  hipError_t e = launch_attention_bwd_mfma<T>(a, s, &taken);
  if (taken) return e;
  return launch_attention_bwd_generic<T>(a, s);
}

template hipError_t launch_attention_fwd<float>(const AttnArgs&, hipStream_t);
template hipError_t launch_attention_fwd<bf16_t>(const AttnArgs&, hipStream_t);
template hipError_t launch_attention_bwd<float>(const AttnArgs&, hipStream_t);
template hipError_t launch_attention_bwd<bf16_t>(const AttnArgs&, hipStream_t);
template hipError_t launch_attention_fwd_generic<float>(const AttnArgs&, hipStream_t);
template hipError_t launch_attention_fwd_generic<bf16_t>(const AttnArgs&, hipStream_t);
template hipError_t launch_attention_bwd_generic<float>(const AttnArgs&, hipStream_t);
template hipError_t launch_attention_bwd_generic<bf16_t>(const AttnArgs&, hipStream_t);

}  // namespace zb
