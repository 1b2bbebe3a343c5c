// Kernels of the first and the last pipeline stage (Sec. 5.1: the first stage also does the embedding
// lookup, the last the loss computation): token + position embedding and its parameter gradients (W
// pass: a fixed-order sum per table row, no atomics), softmax cross-entropy forward (row log-sum-exp,
// per-token loss, mean) and the gradient of the logits that starts the last stage's B pass.
// All bandwidth-bound; 64-lane wavefronts, 16-byte accesses where the rows allow it.
#include <cstdint>

#include "zb_common.h"

namespace zb {

namespace {

constexpr int kThreads = 256;

template <typename T> __device__ __forceinline__ void load4(const T* p, float (&v)[4]);
template <> __device__ __forceinline__ void load4<float>(const float* p, float (&v)[4]) {
  const float4 t = *reinterpret_cast<const float4*>(p);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
template <> __device__ __forceinline__ void load4<bf16_t>(const bf16_t* p, float (&v)[4]) {
  const bf16x4 t = *reinterpret_cast<const bf16x4*>(p);
  v[0] = (float)t[0]; v[1] = (float)t[1]; v[2] = (float)t[2]; v[3] = (float)t[3];
}
template <typename T> __device__ __forceinline__ void store4(T* p, const float (&v)[4]);
template <> __device__ __forceinline__ void store4<float>(float* p, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t* p, const float (&v)[4]) {
  bf16x4 t;
  t[0] = (bf16_t)v[0]; t[1] = (bf16_t)v[1]; t[2] = (bf16_t)v[2]; t[3] = (bf16_t)v[3];
  *reinterpret_cast<bf16x4*>(p) = t;
}

// X0[t] = E_tok[ids[t]] + E_pos[t mod seq]; grid (tokens, column chunks of 1024)
template <typename T>
__global__ __launch_bounds__(kThreads) void embedding_fwd_kernel(const int* __restrict__ ids, const T* __restrict__ tok,
                                                                 const T* __restrict__ pos, T* __restrict__ out,
                                                                 int h, int seq) {
  const int t = blockIdx.x;
  const int col = (blockIdx.y * kThreads + threadIdx.x) * 4;
  if (col >= h) return;
  float a[4], b[4], o[4];
  load4<T>(tok + (size_t)ids[t] * h + col, a);
  load4<T>(pos + (size_t)(t % seq) * h + col, b);
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = a[e] + b[e];
  store4<T>(out + (size_t)t * h + col, o);
}

// Token order by (id, token index): one workgroup sorts the keys id * 8192 + t in LDS (bitonic network,
// n_pad a power of two <= 8192; the padding keys sort to the end) and writes the token indices.
__global__ __launch_bounds__(1024) void sort_tokens_kernel(const int* __restrict__ ids, int* __restrict__ perm,
                                                           int tokens, int n_pad) {
  extern __shared__ unsigned keys[];
  for (int i = threadIdx.x; i < n_pad; i += blockDim.x)
    keys[i] = i < tokens ? ((unsigned)ids[i] << 13) | (unsigned)i : 0xFFFFFFFFu;
  __syncthreads();
  for (int k = 2; k <= n_pad; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = threadIdx.x; i < n_pad; i += blockDim.x) {
        const int partner = i ^ j;
        if (partner > i) {
          const unsigned a = keys[i], b = keys[partner];
          const bool up = (i & k) == 0;
          if ((a > b) == up) { keys[i] = b; keys[partner] = a; }
        }
      }
      __syncthreads();
    }
  }
  for (int i = threadIdx.x; i < tokens; i += blockDim.x) perm[i] = (int)(keys[i] & 8191u);
}

// dE_tok[v] += sum over the tokens with id v, in increasing token index.  Workgroup (i, chunk) looks at
// position i of the sorted order: if it starts a run of equal ids it adds the run's rows in order and
// then adds the sum to the table row; otherwise it has nothing to do.
template <typename T>
__global__ __launch_bounds__(kThreads) void embedding_grad_tok_kernel(const T* __restrict__ dx,
                                                                      const int* __restrict__ ids,
                                                                      const int* __restrict__ perm,
                                                                      float* __restrict__ g_tok, int tokens, int h) {
  const int i = blockIdx.x;
  const int id = ids[perm[i]];
  if (i > 0 && ids[perm[i - 1]] == id) return;
  const int col = (blockIdx.y * kThreads + threadIdx.x) * 4;
  if (col >= h) return;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int j = i; j < tokens; ++j) {
    const int t = perm[j];
    if (ids[t] != id) break;
    float v[4];
    load4<T>(dx + (size_t)t * h + col, v);
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] += v[e];
  }
  float* dst = g_tok + (size_t)id * h + col;
  float4 o = *reinterpret_cast<float4*>(dst);
  o.x += acc[0]; o.y += acc[1]; o.z += acc[2]; o.w += acc[3];
  *reinterpret_cast<float4*>(dst) = o;
}

// dE_pos[p] += sum over the microbatch's sequences of dX0[sequence * seq + p], in sequence order
template <typename T>
__global__ __launch_bounds__(kThreads) void embedding_grad_pos_kernel(const T* __restrict__ dx,
                                                                      float* __restrict__ g_pos, int seqs, int seq,
                                                                      int h) {
  const int p = blockIdx.x;
  const int col = (blockIdx.y * kThreads + threadIdx.x) * 4;
  if (col >= h) return;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int q = 0; q < seqs; ++q) {
    float v[4];
    load4<T>(dx + ((size_t)q * seq + p) * h + col, v);
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] += v[e];
  }
  float* dst = g_pos + (size_t)p * h + col;
  float4 o = *reinterpret_cast<float4*>(dst);
  o.x += acc[0]; o.y += acc[1]; o.z += acc[2]; o.w += acc[3];
  *reinterpret_cast<float4*>(dst) = o;
}

// Row log-sum-exp of the logits and the token's loss lse - logit[target]; one workgroup per row, every
// thread keeps a running (maximum, sum of exp) pair over its columns, the pairs are combined in a fixed
// order (lanes by shuffles, then the four waves).
__device__ __forceinline__ void lse_merge(float& m, float& s, float m2, float s2) {
  const float top = fmaxf(m, m2);
  s = (m == -INFINITY ? 0.f : s * __expf(m - top)) + (m2 == -INFINITY ? 0.f : s2 * __expf(m2 - top));
  m = top;
}
template <typename T>
__global__ __launch_bounds__(kThreads) void ce_fwd_kernel(const T* __restrict__ logits,
                                                          const int* __restrict__ targets, float* __restrict__ lse,
                                                          float* __restrict__ row_loss, int vocab) {
  __shared__ float red_m[4], red_s[4];
  const int row = blockIdx.x;
  const T* z = logits + (size_t)row * vocab;
  float m = -INFINITY, s = 0.f;
  if (vocab % 4 == 0) {
    for (int c = threadIdx.x * 4; c < vocab; c += kThreads * 4) {
      float v[4];
      load4<T>(z + c, v);
      const float top = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
      const float part = __expf(v[0] - top) + __expf(v[1] - top) + __expf(v[2] - top) + __expf(v[3] - top);
      lse_merge(m, s, top, part);
    }
  } else {
    for (int c = threadIdx.x; c < vocab; c += kThreads) lse_merge(m, s, to_f32(z[c]), 1.f);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float m2 = __shfl_xor(m, o, 64), s2 = __shfl_xor(s, o, 64);
    lse_merge(m, s, m2, s2);
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane == 0) { red_m[wave] = m; red_s[wave] = s; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float mm = red_m[0], ss = red_s[0];
    for (int w = 1; w < 4; ++w) lse_merge(mm, ss, red_m[w], red_s[w]);
    const float l = mm + logf(ss);
    lse[row] = l;
    row_loss[row] = l - to_f32(z[targets[row]]);
  }
}

// mean of the tokens' losses: one workgroup, fixed order
__global__ __launch_bounds__(kThreads) void loss_mean_kernel(const float* __restrict__ row_loss, int rows,
                                                             float* __restrict__ out) {
  __shared__ double red[kThreads];
  double acc = 0.0;
  const int per = (rows + kThreads - 1) / kThreads;
  for (int k = 0; k < per; ++k) {
    const int i = threadIdx.x * per + k;
    if (i < rows) acc += (double)row_loss[i];
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = kThreads / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = (float)(red[0] / rows);
}

// dLogits[t, j] = scale * (exp(logit - lse[t]) - [j == target[t]])
template <typename T>
__global__ __launch_bounds__(kThreads) void ce_bwd_kernel(const T* __restrict__ logits, const float* __restrict__ lse,
                                                          const int* __restrict__ targets, T* __restrict__ dlogits,
                                                          int vocab, float scale) {
  const int row = blockIdx.y;
  const float l = lse[row];
  const int tgt = targets[row];
  const T* z = logits + (size_t)row * vocab;
  T* d = dlogits + (size_t)row * vocab;
  if (vocab % 4 == 0) {
    const int c = (blockIdx.x * kThreads + threadIdx.x) * 4;
    if (c >= vocab) return;
    float v[4], o[4];
    load4<T>(z + c, v);
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = scale * (__expf(v[e] - l) - (c + e == tgt ? 1.f : 0.f));
    store4<T>(d + c, o);
  } else {
    for (int e = 0; e < 4; ++e) {
      const int c = (blockIdx.x * kThreads + threadIdx.x) * 4 + e;
      if (c < vocab) d[c] = from_f32<T>(scale * (__expf(to_f32(z[c]) - l) - (c == tgt ? 1.f : 0.f)));
    }
  }
}

}  // namespace

template <typename T>
hipError_t launch_embedding_fwd(const int* ids, const T* tok, const T* pos, T* out, int tokens, int h, int seq,
                                hipStream_t s) {
  if (tokens <= 0 || h <= 0 || h % 4 != 0 || seq <= 0) return hipErrorInvalidValue;
  embedding_fwd_kernel<T><<<dim3(tokens, (h + kThreads * 4 - 1) / (kThreads * 4)), kThreads, 0, s>>>(ids, tok, pos, out,
                                                                                                 h, seq);
  return hipGetLastError();
}

hipError_t launch_sort_tokens(const int* ids, int* perm, int tokens, hipStream_t s) {
  if (tokens <= 0 || tokens > kEmbeddingMaxTokens) return hipErrorInvalidValue;
  int n_pad = 2;
  while (n_pad < tokens) n_pad <<= 1;
  sort_tokens_kernel<<<1, 1024, (size_t)n_pad * sizeof(unsigned), s>>>(ids, perm, tokens, n_pad);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_embedding_grad(const T* dx, const int* ids, const int* perm, float* g_tok, float* g_pos, int tokens,
                                 int h, int seq, hipStream_t s) {
  if (tokens <= 0 || h <= 0 || h % 4 != 0 || seq <= 0 || tokens % seq != 0) return hipErrorInvalidValue;
  const int chunks = (h + kThreads * 4 - 1) / (kThreads * 4);
  embedding_grad_tok_kernel<T><<<dim3(tokens, chunks), kThreads, 0, s>>>(dx, ids, perm, g_tok, tokens, h);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  embedding_grad_pos_kernel<T><<<dim3(seq, chunks), kThreads, 0, s>>>(dx, g_pos, tokens / seq, seq, h);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_ce_fwd(const T* logits, const int* targets, float* lse, float* row_loss, float* loss_out, int rows,
                         int vocab, hipStream_t s) {
  if (rows <= 0 || vocab <= 0) return hipErrorInvalidValue;
  ce_fwd_kernel<T><<<rows, kThreads, 0, s>>>(logits, targets, lse, row_loss, vocab);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  loss_mean_kernel<<<1, kThreads, 0, s>>>(row_loss, rows, loss_out);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_ce_bwd(const T* logits, const float* lse, const int* targets, T* dlogits, int rows, int vocab,
                         float scale, hipStream_t s) {
  if (rows <= 0 || vocab <= 0) return hipErrorInvalidValue;
  ce_bwd_kernel<T><<<dim3((vocab + kThreads * 4 - 1) / (kThreads * 4), rows), kThreads, 0, s>>>(logits, lse, targets,
                                                                                            dlogits, vocab, scale);
  return hipGetLastError();
}

#define ZB_INST(T)                                                                                              \
  template hipError_t launch_embedding_fwd<T>(const int*, const T*, const T*, T*, int, int, int, hipStream_t);  \
  template hipError_t launch_embedding_grad<T>(const T*, const int*, const int*, float*, float*, int, int, int, \
                                               hipStream_t);                                                    \
  template hipError_t launch_ce_fwd<T>(const T*, const int*, float*, float*, float*, int, int, hipStream_t);    \
  template hipError_t launch_ce_bwd<T>(const T*, const float*, const int*, T*, int, int, float, hipStream_t);
ZB_INST(float)
ZB_INST(bf16_t)
#undef ZB_INST

}  // namespace zb
