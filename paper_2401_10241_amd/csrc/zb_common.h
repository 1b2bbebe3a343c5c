// Shared device helpers and launch declarations of the zero-bubble stage library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zb {

typedef __bf16 bf16_t;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// tanh-form GELU and its derivative (fp32)
__device__ __forceinline__ float gelu_f(float x) {
  const float c = 0.7978845608028654f, a = 0.044715f;
  float u = c * (x + a * x * x * x);
  return 0.5f * x * (1.0f + tanhf(u));
}
__device__ __forceinline__ float gelu_grad_f(float x) {
  const float c = 0.7978845608028654f, a = 0.044715f;
  float t = tanhf(c * (x + a * x * x * x));
  return 0.5f * (1.0f + t) + 0.5f * x * (1.0f - t * t) * c * (1.0f + 3.0f * a * x * x);
}

// ---------------------------------------------------------------------------------------
// GEMM:  C[M,N] (op)= sum_k A(m,k) * B(k,n).   A element (m,k) sits at A[m*a_sm + k*a_sk],
// B element (k,n) at B[k*b_sk + n*b_sn]; exactly one stride of each operand is 1.
// ---------------------------------------------------------------------------------------
enum Epilogue : int {
  EPI_STORE = 0,       // out0 = acc
  EPI_BIAS = 1,        // out0 = acc + bias[n]
  EPI_BIAS_RESID = 2,  // out0 = acc + bias[n] + resid[m,n]
  EPI_BIAS_GELU = 3,   // out0 = acc + bias[n]; out1 = gelu(out0)
  EPI_DGELU = 4,       // out0 = acc * gelu'(aux[m,n])
  EPI_ACCUM_F32 = 5,   // outf[m,n] += acc   (fp32 gradient accumulation)
  EPI_PARTIAL = 6      // internal: fp32 partial product of one K slice (split-K), finished by a fix-up kernel
};

struct GemmArgs {
  const void* A;
  const void* B;
  int M, N, K;
  long a_sm, a_sk, b_sk, b_sn;
  int epilogue;
  void* out0;          // [M,N] row-major, element type T
  void* out1;          // second output (EPI_BIAS_GELU)
  float* outf;         // fp32 [M,N] (EPI_ACCUM_F32)
  const float* bias;   // [N] fp32
  const void* aux;     // resid or pre-activation, [M,N] type T
  float* workspace;    // optional fp32 scratch for split-K partial products (device), may be null
  size_t workspace_floats;
  // Grouped wgrad (EPI_ACCUM_F32 only): group >= 2 operand pairs of the same shape and strides;
  // outf += A_0^T B_0, then += A_1^T B_1, ...: bit for bit what `group` separate launches give (whichever
  // kernel takes the shape).  A and B above are ignored then.
  int group;
  const void* group_a[16];
  const void* group_b[16];
  // Optional LayerNorm on the rows of the output (N = the LayerNorm width), taken only when the GEMM runs as K
  // slices, whose last step owns whole rows; *ln_done tells the caller (false: it runs the LayerNorm itself).
  //   ln_mode 1 (with EPI_BIAS_RESID): forward, ln_out = LayerNorm(out0; ln_gamma, ln_beta), ln_stats written
  //   ln_mode 2 (with EPI_STORE): backward of the LayerNorm whose output gradient this GEMM computes:
  //     ln_out = ln_resid + LNbwd(out0; ln_x, ln_stats, ln_gamma), ln_dgamma / ln_dbeta += ...
  int ln_mode;
  const float *ln_gamma, *ln_beta;
  float* ln_stats;
  void* ln_out;
  float ln_eps;
  const void *ln_x, *ln_resid;
  float *ln_dgamma, *ln_dbeta, *ln_partials;
  bool* ln_done;
};
constexpr int kGemmGroupMax = 16;

template <typename T> hipError_t launch_gemm(const GemmArgs& g, hipStream_t s);

// The accumulate GEMMs of one W pass in one launch: dW[q] (fp32 [M[q], N[q]], row stride N[q]) +=
// sum over g < ngroup of X[q][g]^T dY[q][g], X [K, M[q]] and dY [K, N[q]] of type T, dense, for q < nprob.
// Every dW[q] gets exactly the bits that launch_gemm gives it problem by problem.
constexpr int kWgradMaxProblems = 16, kWgradMaxPairs = 64;
struct WgradMultiArgs {
  int nprob, ngroup, K;  // nprob * ngroup <= kWgradMaxPairs, ngroup <= kGemmGroupMax
  int M[kWgradMaxProblems], N[kWgradMaxProblems];
  float* outf[kWgradMaxProblems];
  const void* a[kWgradMaxPairs];  // pair g of problem q at [q * ngroup + g]
  const void* b[kWgradMaxPairs];
  // optional: bias[q] (N[q] floats) += column sums of problem q's b operands, pair by pair in the order given.
  // *bias_done is set if the launch did it (extra workgroups of the same launch); otherwise the caller does.
  float* bias[kWgradMaxProblems];
  bool* bias_done;
};
template <typename T> hipError_t launch_wgrad_multi(const WgradMultiArgs& w, hipStream_t s);

// ---------------------------------------------------------------------------------------
// attention (causal, per head), token-major QKV [tokens, 3h] with columns [Q|K|V] head-major
// ---------------------------------------------------------------------------------------
struct AttnArgs {
  const void* qkv;   // [b*s, 3h]
  void* out;         // fwd: C [b*s, h]
  float* lse;        // [b, a, s] log-sum-exp of the scaled, masked scores
  const void* dout;  // bwd: dC [b*s, h]
  const void* o;     // bwd: C
  void* dqkv;        // bwd: [b*s, 3h]
  float* dvec;       // bwd scratch [b, a, s]: rowsum(dO * O)
  int b, s, a, d;
};
template <typename T> hipError_t launch_attention_fwd(const AttnArgs& a, hipStream_t s);
template <typename T> hipError_t launch_attention_bwd(const AttnArgs& a, hipStream_t s);

// ---------------------------------------------------------------------------------------
// row-wise / elementwise
// ---------------------------------------------------------------------------------------
template <typename T>
hipError_t launch_layernorm_fwd(const T* x, const float* gamma, const float* beta, T* out, float* stats,
                                int rows, int h, float eps, hipStream_t s);
// dx = resid + LNbwd(g) (resid may be null: no residual path); partial dgamma/dbeta of up to kLnBwdSlices row slices go to `partials`
// ([slices][2][h]) and are then added to dgamma/dbeta in slice order.
template <typename T>
hipError_t launch_layernorm_bwd(const T* g, const T* x, const float* stats, const float* gamma, const T* resid,
                                T* dx, float* dgamma, float* dbeta, float* partials, int rows, int h,
                                hipStream_t s);
constexpr int kLnBwdSlices = 16;

// The same two LayerNorm passes fused with the end of a split-K GEMM (`slices` dense fp32 planes of [rows, h],
// `plane` floats apart, added in slice order):
//   forward:  y = T(sum of planes + bias + resid) is the GEMM's output; out = LayerNorm(y), stats as above
//   backward: g = T(sum of planes) is the dgrad GEMM's output (stored to g_out); dx = resid + LNbwd(g);
//             partials as for launch_layernorm_bwd
template <typename T>
hipError_t launch_splitk_layernorm_fwd(const float* planes, int slices, size_t plane, const float* bias, const T* resid,
                                       T* y, const float* gamma, const float* beta, T* out, float* stats, int rows,
                                       int h, float eps, hipStream_t s);
template <typename T>
hipError_t launch_splitk_layernorm_bwd(const float* planes, int slices, size_t plane, T* g_out, const T* x,
                                       const float* stats, const float* gamma, const T* resid, T* dx, float* dgamma,
                                       float* dbeta, float* partials, int rows, int h, hipStream_t s);

// bias gradients: db[q][c] += sum_rows dy[q][r, c] for `count` <= 4 matrices dy[q] of [rows, n[q]] in one launch
// pair; row slices are added in a fixed order; scratch holds kColsumSlices * (n[0] + ... + n[count-1]) floats
constexpr int kColsumSlices = 8;
struct ColsumSegs {
  const void* dy[4];
  float* db[4];
  int n[4];
  int blk0[4];  // first column block of each matrix in the launch
  int col0[4];  // first column of each matrix in the scratch rows
  int total;    // n[0] + ... + n[count-1]
};
template <typename T>
hipError_t launch_colsum_accum_multi(const void* const* dy, float* const* db, const int* n, int count,
                                     float* scratch, int rows, hipStream_t s);

hipError_t launch_fill_f32(float* p, size_t n, float v, hipStream_t s);
hipError_t launch_transpose_bf16(const bf16_t* src, bf16_t* dst, int rows, int cols, hipStream_t s);
template <typename T> hipError_t launch_convert_from_f32(const float* src, T* dst, size_t n, hipStream_t s);
template <typename T> hipError_t launch_convert_to_f32(const T* src, float* dst, size_t n, hipStream_t s);
template <typename T> hipError_t launch_poke(T* dst, size_t idx, float v, hipStream_t s);
// dst[r, c] (fp32, dense [rows, ncols]) = src[r * ld + cols[c]]; cols is a device array
template <typename T>
hipError_t launch_gather_columns(const T* src, long ld, int rows, const int* cols, int ncols, float* dst,
                                 hipStream_t s);

// ---------------------------------------------------------------------------------------
// first / last stage (Sec. 5.1): embedding lookup and its gradients, softmax cross-entropy
// ---------------------------------------------------------------------------------------
constexpr int kEmbeddingMaxTokens = 8192;  // tokens per microbatch the token sort takes (keys id * 8192 + t)
constexpr int kEmbeddingMaxVocab = 1 << 18;
// out[t] = tok[ids[t]] + pos[t mod seq], rows of h elements
template <typename T>
hipError_t launch_embedding_fwd(const int* ids, const T* tok, const T* pos, T* out, int tokens, int h, int seq,
                                hipStream_t s);
// perm = token indices ordered by (id, token index)
hipError_t launch_sort_tokens(const int* ids, int* perm, int tokens, hipStream_t s);
// g_tok[v] += sum of dx[t] over the tokens with ids[t] = v (increasing t); g_pos[p] += sum over the sequences
template <typename T>
hipError_t launch_embedding_grad(const T* dx, const int* ids, const int* perm, float* g_tok, float* g_pos, int tokens,
                                 int h, int seq, hipStream_t s);
// lse[r] = log sum exp of row r; row_loss[r] = lse[r] - logits[r, targets[r]]; *loss_out = mean of row_loss
template <typename T>
hipError_t launch_ce_fwd(const T* logits, const int* targets, float* lse, float* row_loss, float* loss_out, int rows,
                         int vocab, hipStream_t s);
// dlogits[r, j] = scale * (exp(logits[r, j] - lse[r]) - [j == targets[r]])
template <typename T>
hipError_t launch_ce_bwd(const T* logits, const float* lse, const int* targets, T* dlogits, int rows, int vocab,
                         float scale, hipStream_t s);

// ---------------------------------------------------------------------------------------
// optimizer (Sec. 4 and Appendix C).  All decisions live in OptDevState on the device.
// ---------------------------------------------------------------------------------------
struct OptDevState {
  double local_sq;
  double global_norm;
  double clip_coef;
  unsigned long long mismatch;
  int local_nonfinite;
  int t;                 // Algorithm 1's time stamp
  int stepped;           // optimistic step taken
  int do_step;           // predicate of the next step kernel
  int do_rollback;       // predicate of the rollback kernel
  int outcome;
  float step_coef;       // gradient scale of the next step kernel
  float bc1, bc2;        // 1 - beta1^t, 1 - beta2^t for the step / rollback at time t
  int journal_current;   // the next step writes no journal: it comes after the validation (final), and after a rollback theta, m, v equal the journal anyway
};

struct OptHyper {
  float lr, beta1, beta2, eps, weight_decay, clip;
};

// Sum of squares and non-finite flag of n gradients (n % 4 == 0) in three levels, every sum in a fixed
// order: per workgroup of 4096 elements, per kSumsqFan of those, then one workgroup.  partial_sq and
// partial_nf need grad_sumsq_partials(n) entries each.
constexpr int kSumsqFan = 1024;
size_t grad_sumsq_partials(size_t n);
hipError_t launch_grad_sumsq(const float* g, size_t n, double* partial_sq, int* partial_nf,
                             OptDevState* st, hipStream_t s);
hipError_t launch_decide_optimistic(OptDevState* st, OptHyper hp, double prev_sq, int prev_nf, int force,
                                    hipStream_t s);
hipError_t launch_decide_validate(OptDevState* st, OptHyper hp, double prev_sq, double rest_sq, int prev_nf,
                                  int rest_nf, hipStream_t s);
hipError_t launch_decide_after_rollback(OptDevState* st, OptHyper hp, hipStream_t s);
hipError_t launch_clear_step(OptDevState* st, hipStream_t s);
// theta, m, v updated in place when st->do_step; the overwritten values go to the journal (if any);
// theta16 (if any) receives the bf16 working copy.
hipError_t launch_adamw_step(float* theta, float* m, float* v, const float* g, float* j_theta, float* j_m,
                             float* j_v, bf16_t* theta16, size_t n, OptHyper hp, const OptDevState* st,
                             hipStream_t s);
hipError_t launch_adamw_rollback(float* theta, float* m, float* v, const float* g, const float* j_theta,
                                 const float* j_m, const float* j_v, bf16_t* theta16, size_t n, OptHyper hp,
                                 OptDevState* st, hipStream_t s);

}  // namespace zb
