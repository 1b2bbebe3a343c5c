// Post-validated optimizer step (Sec. 4) and in-place AdamW Step / Rollback (Appendix C,
// Algorithm 1) over the stage's flat fp32 parameter vector.  Bandwidth-bound, 16-byte accesses.
// Every decision (step or not, gradient scale, rollback, redo) is taken by a one-thread kernel
// that writes predicates into OptDevState; the heavy kernels read them and return at once when
// switched off, so the host never waits between the steps of the protocol.
#include <mutex>

#include "../../include/zb_stage.h"
#include "zb_common.h"

namespace zb {

namespace {

__device__ __forceinline__ int nonfinite_bits(float v) {
  return (__float_as_uint(v) & 0x7F800000u) == 0x7F800000u ? 1 : 0;
}

// Level 1: kSumsqPerThread 16-byte elements per thread, a workgroup's threads side by side in each (workgroups
// in index order sweep the gradient as one moving front), one partial sum and one non-finite flag per
// workgroup.
constexpr int kSumsqPerThread = 4;
constexpr size_t kSumsqWg4 = 256 * kSumsqPerThread;  // 16-byte elements per workgroup
__global__ __launch_bounds__(256) void grad_sumsq_kernel(const float4* __restrict__ g, size_t n4,
                                                         double* __restrict__ partial_sq,
                                                         int* __restrict__ partial_nf) {
  __shared__ double red[4];
  __shared__ int redf[4];
  double acc = 0.0;
  int bad = 0;
  const size_t i0 = (size_t)blockIdx.x * kSumsqWg4 + threadIdx.x;
  float4 v[kSumsqPerThread];
#pragma unroll
  for (int k = 0; k < kSumsqPerThread; ++k) {
    const size_t i = i0 + (size_t)k * 256;
    v[k] = i < n4 ? g[i] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
#pragma unroll
  for (int k = 0; k < kSumsqPerThread; ++k) {
    bad |= nonfinite_bits(v[k].x) | nonfinite_bits(v[k].y) | nonfinite_bits(v[k].z) | nonfinite_bits(v[k].w);
    acc += ((double)v[k].x * v[k].x + (double)v[k].y * v[k].y) + ((double)v[k].z * v[k].z + (double)v[k].w * v[k].w);
  }
  acc = wave_sum(acc);
  bad = __any(bad);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane == 0) { red[wave] = acc; redf[wave] = bad; }
  __syncthreads();
  if (threadIdx.x == 0) {
    partial_sq[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
    partial_nf[blockIdx.x] = redf[0] | redf[1] | redf[2] | redf[3];
  }
}

// Level 2: workgroup b adds partials [b * kSumsqFan, (b + 1) * kSumsqFan) in a fixed order.
__global__ __launch_bounds__(256) void grad_sumsq_mid_kernel(const double* __restrict__ in_sq,
                                                             const int* __restrict__ in_nf, size_t count,
                                                             double* __restrict__ out_sq,
                                                             int* __restrict__ out_nf) {
  __shared__ double red[256];
  __shared__ int redf[256];
  constexpr int per = kSumsqFan / 256;
  double acc = 0.0;
  int bad = 0;
#pragma unroll
  for (int k = 0; k < per; ++k) {
    const size_t i = (size_t)blockIdx.x * kSumsqFan + (size_t)threadIdx.x * per + k;
    if (i < count) { acc += in_sq[i]; bad |= in_nf[i]; }
  }
  red[threadIdx.x] = acc;
  redf[threadIdx.x] = bad;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) { red[threadIdx.x] += red[threadIdx.x + o]; redf[threadIdx.x] |= redf[threadIdx.x + o]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { out_sq[blockIdx.x] = red[0]; out_nf[blockIdx.x] = redf[0]; }
}

// one workgroup; partial sums are added in a fixed order
__global__ __launch_bounds__(256) void grad_sumsq_final_kernel(const double* __restrict__ partial_sq,
                                                               const int* __restrict__ partial_nf, int blocks,
                                                               double* __restrict__ out_sq, int* __restrict__ out_nf) {
  __shared__ double red[256];
  __shared__ int redf[256];
  double acc = 0.0;
  int bad = 0;
  const int per = (blocks + 255) / 256;
  for (int k = 0; k < per; ++k) {
    const int i = threadIdx.x * per + k;
    if (i < blocks) { acc += partial_sq[i]; bad |= partial_nf[i]; }
  }
  red[threadIdx.x] = acc;
  redf[threadIdx.x] = bad;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) { red[threadIdx.x] += red[threadIdx.x + o]; redf[threadIdx.x] |= redf[threadIdx.x + o]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    *out_sq = red[0];
    *out_nf = redf[0] ? 1 : 0;
  }
}

__device__ __forceinline__ double clip_coef_d(double norm, double clip) {
  const double c = clip / (norm + 1e-6);
  return c < 1.0 ? c : 1.0;
}
__device__ __forceinline__ void advance_time(OptDevState* st, OptHyper hp) {
  st->t += 1;
  st->bc1 = (float)(1.0 - pow((double)hp.beta1, (double)st->t));
  st->bc2 = (float)(1.0 - pow((double)hp.beta2, (double)st->t));
}

// partial state = stages before this one (+) this stage; controls the optimistic step
__global__ void decide_optimistic_kernel(OptDevState* st, OptHyper hp, double prev_sq, int prev_nf, int force) {
  const bool part_nf = st->local_nonfinite || prev_nf;
  const double part_sq = prev_sq + st->local_sq;
  const bool part_bad = part_nf || !isfinite(part_sq);
  const bool part_clips = !part_bad && clip_coef_d(sqrt(part_sq), (double)hp.clip) < 1.0;
  const int go = (force || !(part_bad || part_clips)) ? 1 : 0;
  st->stepped = go;
  st->do_step = go;
  st->do_rollback = 0;
  st->step_coef = 1.0f;
  st->mismatch = 0ull;
  st->journal_current = 0;
  if (go) advance_time(st, hp);
}

// full state = partial (+) stages after this one; validates the step that was (not) taken
__global__ void decide_validate_kernel(OptDevState* st, OptHyper hp, double prev_sq, double rest_sq, int prev_nf,
                                       int rest_nf) {
  const bool part_nf = st->local_nonfinite || prev_nf;
  const double part_sq = prev_sq + st->local_sq;
  const bool part_bad = part_nf || !isfinite(part_sq);
  const bool full_nf = part_nf || rest_nf;
  const double full_sq = part_sq + rest_sq;
  const bool full_bad = full_nf || !isfinite(full_sq);
  st->do_step = 0;
  st->do_rollback = 0;
  if (full_bad) {
    st->global_norm = __longlong_as_double(0x7FF8000000000000ll);
    st->clip_coef = 0.0;
    if (st->stepped) { st->do_rollback = 1; st->outcome = 2; }
    else st->outcome = part_bad ? 1 : 5;
    return;
  }
  const double norm = sqrt(full_sq);
  const double c = clip_coef_d(norm, (double)hp.clip);
  st->global_norm = norm;
  st->clip_coef = c;
  if (c < 1.0) {
    if (st->stepped) { st->do_rollback = 1; st->outcome = 3; }
    else st->outcome = 4;
    st->do_step = 1;
    st->step_coef = (float)c;
  } else {
    st->outcome = 0;
  }
}

// bookkeeping between the rollback and the redo
__global__ void decide_after_rollback_kernel(OptDevState* st, OptHyper hp) {
  // A step taken after the validation is final (nothing can roll it back), so it writes no journal: the redo
  // after a rollback (theta, m, v equal the journal anyway) and the deferred clipped step alike.
  if (st->do_rollback) { st->t -= 1; st->do_rollback = 0; }
  st->journal_current = 1;
  if (st->do_step) advance_time(st, hp);
}

__global__ void clear_step_kernel(OptDevState* st) { st->do_step = 0; }

__device__ __forceinline__ void store_bf16x4(bf16_t* p, float4 v) {
  bf16x4 t;
  t[0] = (bf16_t)v.x; t[1] = (bf16_t)v.y; t[2] = (bf16_t)v.z; t[3] = (bf16_t)v.w;
  *reinterpret_cast<bf16x4*>(p) = t;
}

// AdamW with decoupled weight decay and bias-corrected moments (Appendix C, Algorithm 1), one element
__device__ __forceinline__ void step_one(float& th, float& m, float& v, float g, const OptHyper& hp, float bc1,
                                         float bc2) {
  m = hp.beta1 * m + (1.0f - hp.beta1) * g;
  v = hp.beta2 * v + (1.0f - hp.beta2) * (g * g);
  const float mh = m / bc1;
  const float vh = v / bc2;
  th = th - hp.lr * hp.weight_decay * th - hp.lr * mh / (sqrtf(vh) + hp.eps);
}
// its arithmetic inverse (same algorithm): theta from the new moments, then the moments
__device__ __forceinline__ void rollback_one(float& th, float& m, float& v, float g, const OptHyper& hp, float bc1,
                                             float bc2) {
  const float mh = m / bc1;
  const float vh = v / bc2;
  th = (th + hp.lr * mh / (sqrtf(vh) + hp.eps)) / (1.0f - hp.lr * hp.weight_decay);
  m = (m - (1.0f - hp.beta1) * g) / hp.beta1;
  v = (v - (1.0f - hp.beta2) * (g * g)) / hp.beta2;
}

template <bool JOURNAL, bool BF16>
__global__ __launch_bounds__(256) void adamw_step_kernel(float4* __restrict__ theta, float4* __restrict__ m,
                                                         float4* __restrict__ v, const float4* __restrict__ g,
                                                         float4* __restrict__ j_theta, float4* __restrict__ j_m,
                                                         float4* __restrict__ j_v, bf16_t* __restrict__ theta16,
                                                         size_t n4, OptHyper hp, const OptDevState* __restrict__ st) {
  if (!st->do_step) return;
  const float coef = st->step_coef, bc1 = st->bc1, bc2 = st->bc2;
  const bool keep = JOURNAL && !st->journal_current;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n4) {
    float4 th = theta[i], mm = m[i], vv = v[i], gg = g[i];
    if (keep) { j_theta[i] = th; j_m[i] = mm; j_v[i] = vv; }
    if (coef != 1.0f) { gg.x *= coef; gg.y *= coef; gg.z *= coef; gg.w *= coef; }
    step_one(th.x, mm.x, vv.x, gg.x, hp, bc1, bc2);
    step_one(th.y, mm.y, vv.y, gg.y, hp, bc1, bc2);
    step_one(th.z, mm.z, vv.z, gg.z, hp, bc1, bc2);
    step_one(th.w, mm.w, vv.w, gg.w, hp, bc1, bc2);
    theta[i] = th; m[i] = mm; v[i] = vv;
    if (BF16) store_bf16x4(theta16 + 4 * i, th);
  }
}

__device__ __forceinline__ unsigned bits_differ(float a0, float a1, float b0, float b1, float c0, float c1) {
  return (__float_as_uint(a0) != __float_as_uint(a1) || __float_as_uint(b0) != __float_as_uint(b1) ||
          __float_as_uint(c0) != __float_as_uint(c1)) ? 1u : 0u;
}

// Undoes the optimistic step (which always used the unscaled gradient).  With a journal the
// pre-step values are restored bit for bit and Algorithm 1's arithmetic inverse is evaluated only
// to count the elements where it would have differed; without one the arithmetic inverse is stored.
template <bool JOURNAL, bool BF16>
__global__ __launch_bounds__(256) void adamw_rollback_kernel(float4* __restrict__ theta, float4* __restrict__ m,
                                                             float4* __restrict__ v, const float4* __restrict__ g,
                                                             const float4* __restrict__ j_theta,
                                                             const float4* __restrict__ j_m,
                                                             const float4* __restrict__ j_v,
                                                             bf16_t* __restrict__ theta16, size_t n4, OptHyper hp,
                                                             OptDevState* __restrict__ st) {
  if (!st->do_rollback) return;
  const float bc1 = st->bc1, bc2 = st->bc2;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  unsigned long long mism = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    float4 th = theta[i], mm = m[i], vv = v[i];
    const float4 gg = g[i];
    rollback_one(th.x, mm.x, vv.x, gg.x, hp, bc1, bc2);
    rollback_one(th.y, mm.y, vv.y, gg.y, hp, bc1, bc2);
    rollback_one(th.z, mm.z, vv.z, gg.z, hp, bc1, bc2);
    rollback_one(th.w, mm.w, vv.w, gg.w, hp, bc1, bc2);
    if (JOURNAL) {
      const float4 jt = j_theta[i], jm = j_m[i], jv = j_v[i];
      // an element mismatches if any of its three values differs in any bit
      mism += bits_differ(th.x, jt.x, mm.x, jm.x, vv.x, jv.x) + bits_differ(th.y, jt.y, mm.y, jm.y, vv.y, jv.y) +
              bits_differ(th.z, jt.z, mm.z, jm.z, vv.z, jv.z) + bits_differ(th.w, jt.w, mm.w, jm.w, vv.w, jv.w);
      th = jt; mm = jm; vv = jv;
    }
    theta[i] = th; m[i] = mm; v[i] = vv;
    if (BF16) store_bf16x4(theta16 + 4 * i, th);
  }
  if (JOURNAL) {
    // integer atomics: the count does not depend on the order of arrival
    double s = wave_sum((double)mism);
    if ((threadIdx.x & 63) == 0 && s > 0.0) atomicAdd(&st->mismatch, (unsigned long long)s);
  }
}

// One 16-byte element per thread and as many 256-thread workgroups as that takes: the workgroups
// start in index order, so the chip sweeps every array as one moving front, which the HBM likes
// better than a grid-stride loop (measured: read-modify-write 5.9 TB/s against 4.5-4.9).
inline unsigned opt_grid(size_t n4) { return (unsigned)((n4 + 255) / 256); }

}  // namespace

size_t grad_sumsq_partials(size_t n) {
  const size_t p1 = (n / 4 + kSumsqWg4 - 1) / kSumsqWg4, p2 = (p1 + kSumsqFan - 1) / kSumsqFan;
  return p1 + p2;
}

// the three levels; the result goes to *out_sq / *out_nf (device)
static hipError_t sumsq_levels(const float* g, size_t n, double* partial_sq, int* partial_nf, double* out_sq,
                               int* out_nf, hipStream_t s) {
  if (n % 4 != 0 || n == 0) return hipErrorInvalidValue;
  const size_t n4 = n / 4;
  const size_t p1 = (n4 + kSumsqWg4 - 1) / kSumsqWg4, p2 = (p1 + kSumsqFan - 1) / kSumsqFan;
  if (p1 > ((size_t)1 << 31) - 1) return hipErrorInvalidValue;
  grad_sumsq_kernel<<<(unsigned)p1, 256, 0, s>>>((const float4*)g, n4, partial_sq, partial_nf);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  grad_sumsq_mid_kernel<<<(unsigned)p2, 256, 0, s>>>(partial_sq, partial_nf, p1, partial_sq + p1, partial_nf + p1);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  grad_sumsq_final_kernel<<<1, 256, 0, s>>>(partial_sq + p1, partial_nf + p1, (int)p2, out_sq, out_nf);
  return hipGetLastError();
}
hipError_t launch_grad_sumsq(const float* g, size_t n, double* partial_sq, int* partial_nf, OptDevState* st,
                             hipStream_t s) {
  return sumsq_levels(g, n, partial_sq, partial_nf, &st->local_sq, &st->local_nonfinite, s);
}
hipError_t launch_decide_optimistic(OptDevState* st, OptHyper hp, double prev_sq, int prev_nf, int force,
                                    hipStream_t s) {
  decide_optimistic_kernel<<<1, 1, 0, s>>>(st, hp, prev_sq, prev_nf, force);
  return hipGetLastError();
}
hipError_t launch_decide_validate(OptDevState* st, OptHyper hp, double prev_sq, double rest_sq, int prev_nf,
                                  int rest_nf, hipStream_t s) {
  decide_validate_kernel<<<1, 1, 0, s>>>(st, hp, prev_sq, rest_sq, prev_nf, rest_nf);
  return hipGetLastError();
}
hipError_t launch_decide_after_rollback(OptDevState* st, OptHyper hp, hipStream_t s) {
  decide_after_rollback_kernel<<<1, 1, 0, s>>>(st, hp);
  return hipGetLastError();
}
hipError_t launch_clear_step(OptDevState* st, hipStream_t s) {
  clear_step_kernel<<<1, 1, 0, s>>>(st);
  return hipGetLastError();
}

hipError_t launch_adamw_step(float* theta, float* m, float* v, const float* g, float* j_theta, float* j_m,
                             float* j_v, bf16_t* theta16, size_t n, OptHyper hp, const OptDevState* st,
                             hipStream_t s) {
  if (n % 4 != 0) return hipErrorInvalidValue;
  const size_t n4 = n / 4;
  if (n4 == 0 || n4 > ((size_t)1 << 39)) return hipErrorInvalidValue;
  const unsigned grid = opt_grid(n4);
  const bool J = j_theta != nullptr, H = theta16 != nullptr;
#define ZB_STEP(JJ, HH)                                                                                          \
  adamw_step_kernel<JJ, HH><<<grid, 256, 0, s>>>((float4*)theta, (float4*)m, (float4*)v, (const float4*)g,        \
                                                 (float4*)j_theta, (float4*)j_m, (float4*)j_v, theta16, n4, hp, st)
  if (J && H) ZB_STEP(true, true);
  else if (J) ZB_STEP(true, false);
  else if (H) ZB_STEP(false, true);
  else ZB_STEP(false, false);
#undef ZB_STEP
  return hipGetLastError();
}

hipError_t launch_adamw_rollback(float* theta, float* m, float* v, const float* g, const float* j_theta,
                                 const float* j_m, const float* j_v, bf16_t* theta16, size_t n, OptHyper hp,
                                 OptDevState* st, hipStream_t s) {
  if (n % 4 != 0) return hipErrorInvalidValue;
  const size_t n4 = n / 4;
  if (n4 == 0 || n4 > ((size_t)1 << 39)) return hipErrorInvalidValue;
  // grid-stride here: the mismatch count costs one atomic per wavefront, and a rollback is the rare path
  const unsigned grid = opt_grid(n4) < 8192u ? opt_grid(n4) : 8192u;
  const bool J = j_theta != nullptr, H = theta16 != nullptr;
#define ZB_RB(JJ, HH)                                                                                             \
  adamw_rollback_kernel<JJ, HH><<<grid, 256, 0, s>>>((float4*)theta, (float4*)m, (float4*)v, (const float4*)g,     \
                                                     (const float4*)j_theta, (const float4*)j_m,                   \
                                                     (const float4*)j_v, theta16, n4, hp, st)
  if (J && H) ZB_RB(true, true);
  else if (J) ZB_RB(true, false);
  else if (H) ZB_RB(false, true);
  else ZB_RB(false, false);
#undef ZB_RB
  return hipGetLastError();
}

}  // namespace zb

// ---------------------------------------------------------------------------------------------------------
// Squared gradient norm and non-finite flag for callers that cannot allocate: the partial sums of the three
// reduction levels live in a file-scope device array instead of the stage's arena.
// ---------------------------------------------------------------------------------------------------------
namespace {

constexpr size_t kStaticMaxFloats = (size_t)1 << 30;  // == ZB_GRAD_NORM_STATIC_MAX_FLOATS
constexpr size_t kStaticP1 = (kStaticMaxFloats / 4 + zb::kSumsqWg4 - 1) / zb::kSumsqWg4;
constexpr size_t kStaticPartials = kStaticP1 + (kStaticP1 + zb::kSumsqFan - 1) / zb::kSumsqFan;
constexpr size_t kStaticSqBytes = (kStaticPartials * sizeof(double) + 255) / 256 * 256;
constexpr size_t kStaticBytes = kStaticSqBytes + kStaticPartials * sizeof(int);  // about 3.2 MB
static_assert(kStaticMaxFloats == ZB_GRAD_NORM_STATIC_MAX_FLOATS, "header and kernel file disagree");

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

// Every device holds its own copy of `scratch` at its own address: looked up once per device, with that
// device current, and only this pointer (never the array's name) is handed to kernels.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

hipError_t scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" zb_status zb_grad_norm_static(const float* grads, size_t n, double* sq_out, int32_t* nonfinite_out,
                                         void* hip_stream) {
  if (!grads || !sq_out || !nonfinite_out) return ZB_EINVAL;
  if (n == 0 || n % 4 != 0 || n > kStaticMaxFloats) return ZB_EINVAL;
  if (reinterpret_cast<uintptr_t>(grads) & 15) return ZB_EINVAL;
  void* base = nullptr;
  if (scratch_of_current_device(&base) != hipSuccess) return ZB_EDEVICE;
  double* partial_sq = reinterpret_cast<double*>(base);
  int* partial_nf = reinterpret_cast<int*>(reinterpret_cast<unsigned char*>(base) + kStaticSqBytes);
  // every partial the later levels read is written by the level before it in the same call: nothing has to
  // start at zero, whatever the previous call left behind
  const hipError_t e = zb::sumsq_levels(grads, n, partial_sq, partial_nf, sq_out, nonfinite_out, (hipStream_t)hip_stream);
  return e == hipSuccess ? ZB_OK : ZB_EDEVICE;
}
