// Bandwidth-bound row-wise and elementwise kernels: LayerNorm forward / backward-input
// (with the gamma/beta gradients, which this build produces in the B pass), bias-gradient
// column sums (W pass), fills and type conversions.  One wavefront = 64 lanes; reductions
// use cross-lane shuffles, then LDS across the four waves of a 256-thread workgroup.
#include <cstdint>

#include "zb_common.h"

namespace zb {

namespace {

constexpr int kThreads = 256;
constexpr int kVec = 4;       // elements per lane per chunk
constexpr int kMaxChunks = 8; // rows up to 256*4*8 = 8192 elements stay in registers

template <typename T> struct Vec4;
template <> struct Vec4<float> {
  static __device__ __forceinline__ void load(const float* p, float (&v)[4]) {
    float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <> struct Vec4<bf16_t> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[4]) {
    bf16x4 t = *reinterpret_cast<const bf16x4*>(p);
    v[0] = (float)t[0]; v[1] = (float)t[1]; v[2] = (float)t[2]; v[3] = (float)t[3];
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[4]) {
    bf16x4 t;
    t[0] = (bf16_t)v[0]; t[1] = (bf16_t)v[1]; t[2] = (bf16_t)v[2]; t[3] = (bf16_t)v[3];
    *reinterpret_cast<bf16x4*>(p) = t;
  }
};

// sum over the 256 threads of a workgroup; every thread gets the result
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

template <typename T>
__global__ __launch_bounds__(kThreads) void layernorm_fwd_kernel(const T* __restrict__ x,
                                                                 const float* __restrict__ gamma,
                                                                 const float* __restrict__ beta,
                                                                 T* __restrict__ out, float* __restrict__ stats,
                                                                 int h, float eps) {
  __shared__ float red[4];
  const size_t row = blockIdx.x;
  const T* xr = x + row * h;
  float v[kMaxChunks][kVec];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    const int col = (c * kThreads + threadIdx.x) * kVec;
    if (col < h) {
      Vec4<T>::load(xr + col, v[c]);
      sum += (v[c][0] + v[c][1]) + (v[c][2] + v[c][3]);
    }
  }
  const float mean = block_sum(sum, red) / (float)h;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    const int col = (c * kThreads + threadIdx.x) * kVec;
    if (col < h) {
#pragma unroll
      for (int e = 0; e < kVec; ++e) {
        const float d = v[c][e] - mean;
        sq += d * d;
      }
    }
  }
  const float var = block_sum(sq, red) / (float)h;
  const float rstd = 1.0f / sqrtf(var + eps);
  if (threadIdx.x == 0) {
    stats[row * 2] = mean;
    stats[row * 2 + 1] = rstd;
  }
  T* outr = out + row * h;
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    const int col = (c * kThreads + threadIdx.x) * kVec;
    if (col < h) {
      float g[4], b[4], o[4];
      Vec4<float>::load(gamma + col, g);
      Vec4<float>::load(beta + col, b);
#pragma unroll
      for (int e = 0; e < kVec; ++e) o[e] = (v[c][e] - mean) * rstd * g[e] + b[e];
      Vec4<T>::store(outr + col, o);
    }
  }
}

// LayerNorm forward fused with the end of a split-K GEMM whose output it normalises: the row's GEMM result is
// the sum of `slices` fp32 planes (added in slice order) + bias + residual, rounded to T and stored as the
// GEMM's output; the LayerNorm of those rounded values follows in the same registers.
template <typename T>
__global__ __launch_bounds__(kThreads) void splitk_layernorm_fwd_kernel(const float* __restrict__ planes, int slices,
                                                                        size_t plane, const float* __restrict__ bias,
                                                                        const T* __restrict__ resid,
                                                                        T* __restrict__ y, const float* __restrict__ gamma,
                                                                        const float* __restrict__ beta,
                                                                        T* __restrict__ out, float* __restrict__ stats,
                                                                        int h, float eps) {
  __shared__ float red[4];
  const size_t row = blockIdx.x;
  const size_t off = row * h;
  float v[kMaxChunks][kVec];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    const int col = (c * kThreads + threadIdx.x) * kVec;
    if (col < h) {
      float acc[4], b[4], r[4];
      Vec4<float>::load(planes + off + col, acc);
      for (int sl = 1; sl < slices; ++sl) {
        float p[4];
        Vec4<float>::load(planes + (size_t)sl * plane + off + col, p);
#pragma unroll
        for (int e = 0; e < kVec; ++e) acc[e] += p[e];
      }
      Vec4<float>::load(bias + col, b);
      Vec4<T>::load(resid + off + col, r);
#pragma unroll
      for (int e = 0; e < kVec; ++e) v[c][e] = to_f32(from_f32<T>(acc[e] + b[e] + r[e]));
      Vec4<T>::store(y + off + col, v[c]);
      sum += (v[c][0] + v[c][1]) + (v[c][2] + v[c][3]);
    }
  }
  const float mean = block_sum(sum, red) / (float)h;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    const int col = (c * kThreads + threadIdx.x) * kVec;
    if (col < h) {
#pragma unroll
      for (int e = 0; e < kVec; ++e) {
        const float d = v[c][e] - mean;
        sq += d * d;
      }
    }
  }
  const float var = block_sum(sq, red) / (float)h;
  const float rstd = 1.0f / sqrtf(var + eps);
  if (threadIdx.x == 0) {
    stats[row * 2] = mean;
    stats[row * 2 + 1] = rstd;
  }
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    const int col = (c * kThreads + threadIdx.x) * kVec;
    if (col < h) {
      float g[4], b[4], o[4];
      Vec4<float>::load(gamma + col, g);
      Vec4<float>::load(beta + col, b);
#pragma unroll
      for (int e = 0; e < kVec; ++e) o[e] = (v[c][e] - mean) * rstd * g[e] + b[e];
      Vec4<T>::store(out + off + col, o);
    }
  }
}

// sums of two values over the 256 threads of a workgroup with one exchange
__device__ __forceinline__ void block_sum2(float& a, float& b, float (*red)[2]) {
  a = wave_sum(a);
  b = wave_sum(b);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) { red[wave][0] = a; red[wave][1] = b; }
  __syncthreads();
  a = (red[0][0] + red[1][0]) + (red[2][0] + red[3][0]);
  b = (red[0][1] + red[1][1]) + (red[2][1] + red[3][1]);
}

// dx of one row per workgroup: dx = resid + rstd * (g*gamma - mean(g*gamma) - xhat * mean(g*gamma*xhat)).
// NCH = ceil(h / 1024) chunks of 4 per lane; the whole row stays in registers between the two passes.
template <typename T, int NCH>
__device__ __forceinline__ void layernorm_bwd_dx_body(int row, const T* __restrict__ g, const T* __restrict__ x,
                                                      const float* __restrict__ stats,
                                                      const float* __restrict__ gamma, const T* __restrict__ resid,
                                                      T* __restrict__ dx, int h) {
  __shared__ float red[4][2];
  const size_t off = (size_t)row * h;
  const float mean = stats[row * 2], rstd = stats[row * 2 + 1];
  float gg[NCH][kVec], xh[NCH][kVec], rr[NCH][kVec];
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (c * kThreads + threadIdx.x) * kVec;
    if (col < h) {
      float gam[kVec];
      Vec4<T>::load(g + off + col, gg[c]);
      Vec4<T>::load(x + off + col, xh[c]);
      if (resid) Vec4<T>::load(resid + off + col, rr[c]);
      else rr[c][0] = rr[c][1] = rr[c][2] = rr[c][3] = 0.f;
      Vec4<float>::load(gamma + col, gam);
#pragma unroll
      for (int e = 0; e < kVec; ++e) {
        xh[c][e] = (xh[c][e] - mean) * rstd;
        gg[c][e] *= gam[e];
        s1 += gg[c][e];
        s2 += gg[c][e] * xh[c][e];
      }
    }
  }
  block_sum2(s1, s2, red);
  const float m1 = s1 / (float)h, m2 = s2 / (float)h;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (c * kThreads + threadIdx.x) * kVec;
    if (col < h) {
      float o[4];
#pragma unroll
      for (int e = 0; e < kVec; ++e) o[e] = rr[c][e] + rstd * (gg[c][e] - m1 - xh[c][e] * m2);
      Vec4<T>::store(dx + off + col, o);
    }
  }
}

// Column sums of g*xhat and g over one slice of rows: partials[slice][0][h] and partials[slice][1][h].
// 256 threads = 16 column-lanes (8 consecutive columns each) x 16 row groups; grid.y = row slices.
template <typename T>
__device__ __forceinline__ void layernorm_bwd_param_body(int bx, int by, const T* __restrict__ g,
                                                         const T* __restrict__ x, const float* __restrict__ stats,
                                                         float* __restrict__ partials, int rows, int h,
                                                         int rows_per_slice) {
  __shared__ float red[2][16][129];
  const int cl = threadIdx.x & 15, rg = threadIdx.x >> 4;
  const int col = (bx * 16 + cl) * 8;
  const int r_begin = by * rows_per_slice;
  const int r_end = min(rows, r_begin + rows_per_slice);
  float ag[8], ab[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) ag[e] = ab[e] = 0.f;
  for (int r = r_begin + rg; r < r_end; r += 16) {
    const float mean = stats[r * 2], rstd = stats[r * 2 + 1];
    const size_t off = (size_t)r * h + col;
#pragma unroll
    for (int q = 0; q < 8; q += 4) {
      if (col + q < h) {
        float gv[4], xv[4];
        Vec4<T>::load(g + off + q, gv);
        Vec4<T>::load(x + off + q, xv);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          ag[q + e] += gv[e] * ((xv[e] - mean) * rstd);
          ab[q + e] += gv[e];
        }
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    red[0][rg][cl * 8 + e] = ag[e];
    red[1][rg][cl * 8 + e] = ab[e];
  }
  __syncthreads();
  const int which = threadIdx.x >> 7, t = threadIdx.x & 127;
  const int c = bx * 128 + t;
  if (c < h) {
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += red[which][r][t];
    partials[((size_t)by * 2 + which) * h + c] = sum;
  }
}

// LayerNorm backward fused with the end of the split-K dgrad GEMM that produces its incoming gradient g: one
// row per workgroup; g = the sum of the `slices` planes (slice order), rounded to T and stored (the gamma /
// beta sums read it afterwards); dx as in layernorm_bwd_dx_body, from the same registers.
template <typename T, int NCH>
__global__ __launch_bounds__(kThreads) void splitk_layernorm_bwd_kernel(const float* __restrict__ planes, int slices,
                                                                        size_t plane, T* __restrict__ g_out,
                                                                        const T* __restrict__ x,
                                                                        const float* __restrict__ stats,
                                                                        const float* __restrict__ gamma,
                                                                        const T* __restrict__ resid, T* __restrict__ dx,
                                                                        int h) {
  __shared__ float red[4][2];
  const int row = blockIdx.x;
  const size_t off = (size_t)row * h;
  const float mean = stats[row * 2], rstd = stats[row * 2 + 1];
  float gg[NCH][kVec], xh[NCH][kVec], rr[NCH][kVec];
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (c * kThreads + threadIdx.x) * kVec;
    if (col < h) {
      float acc[4], gam[kVec];
      Vec4<float>::load(planes + off + col, acc);
      for (int sl = 1; sl < slices; ++sl) {
        float p[4];
        Vec4<float>::load(planes + (size_t)sl * plane + off + col, p);
#pragma unroll
        for (int e = 0; e < kVec; ++e) acc[e] += p[e];
      }
      Vec4<T>::load(x + off + col, xh[c]);
      if (resid) Vec4<T>::load(resid + off + col, rr[c]);
      else rr[c][0] = rr[c][1] = rr[c][2] = rr[c][3] = 0.f;
      Vec4<float>::load(gamma + col, gam);
#pragma unroll
      for (int e = 0; e < kVec; ++e) gg[c][e] = to_f32(from_f32<T>(acc[e]));
      Vec4<T>::store(g_out + off + col, gg[c]);
#pragma unroll
      for (int e = 0; e < kVec; ++e) {
        xh[c][e] = (xh[c][e] - mean) * rstd;
        gg[c][e] *= gam[e];
        s1 += gg[c][e];
        s2 += gg[c][e] * xh[c][e];
      }
    }
  }
  block_sum2(s1, s2, red);
  const float m1 = s1 / (float)h, m2 = s2 / (float)h;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (c * kThreads + threadIdx.x) * kVec;
    if (col < h) {
      float o[4];
#pragma unroll
      for (int e = 0; e < kVec; ++e) o[e] = rr[c][e] + rstd * (gg[c][e] - m1 - xh[c][e] * m2);
      Vec4<T>::store(dx + off + col, o);
    }
  }
}

// One launch for both: workgroups 0 .. rows-1 compute dx of one row each, the rest the gamma / beta partial
// sums (column block bx, row slice by).  Nothing downstream waits for the partial sums, so they ride along
// with the dx rows instead of taking a launch of their own.
template <typename T, int NCH>
__global__ __launch_bounds__(kThreads) void layernorm_bwd_kernel(const T* __restrict__ g, const T* __restrict__ x,
                                                                 const float* __restrict__ stats,
                                                                 const float* __restrict__ gamma,
                                                                 const T* __restrict__ resid, T* __restrict__ dx,
                                                                 float* __restrict__ partials, int rows, int h,
                                                                 int rows_per_slice, int col_blocks, int dx_rows) {
  if ((int)blockIdx.x < dx_rows) {
    layernorm_bwd_dx_body<T, NCH>(blockIdx.x, g, x, stats, gamma, resid, dx, h);
  } else {
    const int q = blockIdx.x - dx_rows;
    layernorm_bwd_param_body<T>(q % col_blocks, q / col_blocks, g, x, stats, partials, rows, h, rows_per_slice);
  }
}

// dgamma[c] += sum_b partials[b][0][c]; dbeta[c] += sum_b partials[b][1][c], always in the same order:
// 64 columns per workgroup, four groups of lanes each add a quarter of the blocks in order, then the
// four group sums are added in order.
__global__ __launch_bounds__(256) void layernorm_bwd_reduce_kernel(const float* __restrict__ partials,
                                                                   float* __restrict__ dgamma,
                                                                   float* __restrict__ dbeta, int blocks, int h) {
  __shared__ float red[4][2][64];
  const int cl = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + cl;
  float a = 0.f, b = 0.f;
  if (col < h) {
    const int per = (blocks + 3) / 4;
    const int k1 = min(blocks, (grp + 1) * per);
    for (int k = grp * per; k < k1; ++k) {
      a += partials[(size_t)k * 2 * h + col];
      b += partials[(size_t)k * 2 * h + h + col];
    }
  }
  red[grp][0][cl] = a;
  red[grp][1][cl] = b;
  __syncthreads();
  if (grp == 0 && col < h) {
    dgamma[col] += (red[0][0][cl] + red[1][0][cl]) + (red[2][0][cl] + red[3][0][cl]);
    dbeta[col] += (red[0][1][cl] + red[1][1][cl]) + (red[2][1][cl] + red[3][1][cl]);
  }
}

// Bias gradients: column sums of up to four matrices of one row count in one launch pair (the four dY of a
// layer's W pass).  Stage 1: column sums of one slice of rows; 256 threads = 16 column-lanes (each kV
// consecutive columns) x 16 row groups; grid.y = row slices; column blocks of the matrices are laid side
// by side, out[slice][total columns].
template <typename T, int kV>
__global__ __launch_bounds__(kThreads) void colsum_partial_multi_kernel(ColsumSegs sg, float* __restrict__ out,
                                                                        int rows, int rows_per_slice) {
  __shared__ float red[16][16 * kV + 1];
  int seg = 0;
#pragma unroll
  for (int q = 1; q < 4; ++q) seg += (int)blockIdx.x >= sg.blk0[q] ? 1 : 0;
  const int n = sg.n[seg];
  const T* __restrict__ dy = (const T*)sg.dy[seg];
  const int blk = blockIdx.x - sg.blk0[seg];
  const int cl = threadIdx.x & 15, rg = threadIdx.x >> 4;
  const int col = (blk * 16 + cl) * kV;
  const int r_begin = blockIdx.y * rows_per_slice;
  const int r_end = min(rows, r_begin + rows_per_slice);
  float acc[kV];
#pragma unroll
  for (int e = 0; e < kV; ++e) acc[e] = 0.f;
  if (col < n) {
    for (int r = r_begin + rg; r < r_end; r += 16) {
      const T* p = dy + (size_t)r * n + col;
#pragma unroll
      for (int e = 0; e < kV; e += 4) {
        float v[4];
        Vec4<T>::load(p + e, v);
        acc[e] += v[0]; acc[e + 1] += v[1]; acc[e + 2] += v[2]; acc[e + 3] += v[3];
      }
    }
  }
#pragma unroll
  for (int e = 0; e < kV; ++e) red[rg][cl * kV + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < 16 * kV) {
    const int c = blk * 16 * kV + threadIdx.x;
    if (c < n) {
      float t = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) t += red[r][threadIdx.x];
      out[(size_t)blockIdx.y * sg.total + sg.col0[seg] + c] = t;
    }
  }
}
// stage 2: db[c] += slices added in order
__global__ void colsum_final_multi_kernel(ColsumSegs sg, const float* __restrict__ part, int slices) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= sg.total) return;
  int seg = 0;
#pragma unroll
  for (int q = 1; q < 4; ++q) seg += c >= sg.col0[q] ? 1 : 0;
  float t = 0.f;
  for (int k = 0; k < slices; ++k) t += part[(size_t)k * sg.total + c];
  sg.db[seg][c - sg.col0[seg]] += t;
}

// dst[c][r] = src[r][c] for a [rows][cols] bf16 matrix; 64 x 64 tiles through LDS
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const unsigned short* __restrict__ src,
                                                             unsigned short* __restrict__ dst, int rows, int cols) {
  __shared__ unsigned short tile[64][66];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    tile[i][tx] = (r < rows && c < cols) ? src[(size_t)r * cols + c] : (unsigned short)0;
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int c = c0 + i, r = r0 + tx;
    if (c < cols && r < rows) dst[(size_t)c * rows + r] = tile[tx][i];
  }
}

// 64 x 64 tile with 16-byte global accesses on both sides (rows, cols multiples of 64, 16-byte aligned
// pointers).  LDS row pitch 66 elements: the gather of 8 consecutive rows of one column by 8 x 8 lanes
// (stride 8 rows = 8 banks) touches every bank once.
__global__ __launch_bounds__(256) void transpose_bf16_wide_kernel(const unsigned short* __restrict__ src,
                                                                  unsigned short* __restrict__ dst, int rows,
                                                                  int cols) {
  constexpr int P = 66;
  __shared__ __align__(4) unsigned short tile[64 * P];
  const size_t r0 = (size_t)blockIdx.y * 64, c0 = (size_t)blockIdx.x * 64;
  const int hi = threadIdx.x >> 3, lo = threadIdx.x & 7;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int r = hi + 32 * j;
    const uint4 v = *reinterpret_cast<const uint4*>(src + (r0 + r) * cols + c0 + lo * 8);
    unsigned* t = reinterpret_cast<unsigned*>(tile + r * P + lo * 8);
    t[0] = v.x; t[1] = v.y; t[2] = v.z; t[3] = v.w;
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int c = hi + 32 * j;
    unsigned w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const unsigned a = tile[(lo * 8 + 2 * k) * P + c], b = tile[(lo * 8 + 2 * k + 1) * P + c];
      w[k] = a | (b << 16);
    }
    *reinterpret_cast<uint4*>(dst + (c0 + c) * rows + r0 + lo * 8) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

__global__ void fill_f32_kernel(float* p, size_t n, float v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}
// one 16-byte store per thread, workgroups in index order: the array is written as one moving front
__global__ __launch_bounds__(256) void fill_f32x4_kernel(float4* p, size_t n4, float v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n4) p[i] = make_float4(v, v, v, v);
}
template <typename T>
__global__ void convert_from_f32_kernel(const float* __restrict__ s, T* __restrict__ d, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) d[i] = from_f32<T>(s[i]);
}
template <typename T>
__global__ void convert_to_f32_kernel(const T* __restrict__ s, float* __restrict__ d, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) d[i] = to_f32(s[i]);
}
template <typename T> __global__ void poke_kernel(T* d, size_t idx, float v) { d[idx] = from_f32<T>(v); }

inline int grid_for(size_t n) {
  size_t b = (n + 255) / 256;
  return (int)(b < 1 ? 1 : (b > 4096 ? 4096 : b));
}

}  // namespace

template <typename T>
hipError_t launch_layernorm_fwd(const T* x, const float* gamma, const float* beta, T* out, float* stats, int rows,
                                int h, float eps, hipStream_t s) {
  if (h % kVec != 0 || h > kThreads * kVec * kMaxChunks || rows <= 0) return hipErrorInvalidValue;
  layernorm_fwd_kernel<T><<<rows, kThreads, 0, s>>>(x, gamma, beta, out, stats, h, eps);
  return hipGetLastError();
}

template <typename T, int NCH>
hipError_t run_ln_bwd(const T* g, const T* x, const float* stats, const float* gamma, const T* resid, T* dx,
                      float* partials, int rows, int h, int slices, hipStream_t s) {
  const int rows_per_slice = (rows + slices - 1) / slices, col_blocks = (h + 127) / 128;
  layernorm_bwd_kernel<T, NCH><<<rows + col_blocks * slices, kThreads, 0, s>>>(g, x, stats, gamma, resid, dx, partials,
                                                                             rows, h, rows_per_slice, col_blocks, rows);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_layernorm_bwd(const T* g, const T* x, const float* stats, const float* gamma, const T* resid,
                                T* dx, float* dgamma, float* dbeta, float* partials, int rows, int h,
                                hipStream_t s) {
  if (h % kVec != 0 || h > kThreads * kVec * kMaxChunks || rows <= 0) return hipErrorInvalidValue;
  const int nch = (h + kThreads * kVec - 1) / (kThreads * kVec);
  // gamma / beta gradients: row slices of at least 16 rows, at most kLnBwdSlices of them
  int slices = (rows + 15) / 16;
  if (slices > kLnBwdSlices) slices = kLnBwdSlices;
  hipError_t e;
  switch (nch) {
    case 1: e = run_ln_bwd<T, 1>(g, x, stats, gamma, resid, dx, partials, rows, h, slices, s); break;
    case 2: e = run_ln_bwd<T, 2>(g, x, stats, gamma, resid, dx, partials, rows, h, slices, s); break;
    case 3: e = run_ln_bwd<T, 3>(g, x, stats, gamma, resid, dx, partials, rows, h, slices, s); break;
    case 4: e = run_ln_bwd<T, 4>(g, x, stats, gamma, resid, dx, partials, rows, h, slices, s); break;
    case 5: e = run_ln_bwd<T, 5>(g, x, stats, gamma, resid, dx, partials, rows, h, slices, s); break;
    case 6: e = run_ln_bwd<T, 6>(g, x, stats, gamma, resid, dx, partials, rows, h, slices, s); break;
    default: e = run_ln_bwd<T, 8>(g, x, stats, gamma, resid, dx, partials, rows, h, slices, s); break;
  }
  if (e != hipSuccess) return e;
  layernorm_bwd_reduce_kernel<<<(h + 63) / 64, 256, 0, s>>>(partials, dgamma, dbeta, slices, h);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_splitk_layernorm_fwd(const float* planes, int slices, size_t plane, const float* bias, const T* resid,
                                       T* y, const float* gamma, const float* beta, T* out, float* stats, int rows,
                                       int h, float eps, hipStream_t s) {
  if (h % kVec != 0 || h > kThreads * kVec * kMaxChunks || rows <= 0 || slices < 1) return hipErrorInvalidValue;
  splitk_layernorm_fwd_kernel<T><<<rows, kThreads, 0, s>>>(planes, slices, plane, bias, resid, y, gamma, beta, out, stats,
                                                          h, eps);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_splitk_layernorm_bwd(const float* planes, int slices, size_t plane, T* g_out, const T* x,
                                       const float* stats, const float* gamma, const T* resid, T* dx, float* dgamma,
                                       float* dbeta, float* partials, int rows, int h, hipStream_t s) {
  if (h % kVec != 0 || h > kThreads * kVec * kMaxChunks || rows <= 0 || slices < 1) return hipErrorInvalidValue;
  const int nch = (h + kThreads * kVec - 1) / (kThreads * kVec);
  int pslices = (rows + 15) / 16;
  if (pslices > kLnBwdSlices) pslices = kLnBwdSlices;
  const int rows_per_slice = (rows + pslices - 1) / pslices, col_blocks = (h + 127) / 128;
#define ZB_RUN(N)                                                                                                   \
  splitk_layernorm_bwd_kernel<T, N><<<rows, kThreads, 0, s>>>(planes, slices, plane, g_out, x, stats, gamma, resid,  \
                                                              dx, h);                                               \
  layernorm_bwd_kernel<T, N><<<col_blocks * pslices, kThreads, 0, s>>>(g_out, x, stats, gamma, resid, dx, partials,  \
                                                                       rows, h, rows_per_slice, col_blocks, 0)
  switch (nch) {
    case 1: ZB_RUN(1); break;
    case 2: ZB_RUN(2); break;
    case 3: ZB_RUN(3); break;
    case 4: ZB_RUN(4); break;
    case 5: ZB_RUN(5); break;
    case 6: ZB_RUN(6); break;
    default: ZB_RUN(8); break;
  }
#undef ZB_RUN
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  layernorm_bwd_reduce_kernel<<<(h + 63) / 64, 256, 0, s>>>(partials, dgamma, dbeta, pslices, h);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_colsum_accum_multi(const void* const* dy, float* const* db, const int* n, int count, float* scratch,
                                     int rows, hipStream_t s) {
  constexpr int kV = 16 / sizeof(T);
  constexpr int per_block = 16 * kV;
  if (count < 1 || count > 4 || rows <= 0) return hipErrorInvalidValue;
  ColsumSegs sg{};
  int blocks = 0, cols = 0;
  for (int q = 0; q < 4; ++q) {
    const int nq = q < count ? n[q] : 0;
    if (q < count && (nq <= 0 || nq % kV != 0 || !dy[q] || !db[q])) return hipErrorInvalidValue;
    sg.dy[q] = q < count ? dy[q] : dy[0];
    sg.db[q] = q < count ? db[q] : db[0];
    sg.n[q] = nq;
    sg.blk0[q] = blocks;
    sg.col0[q] = cols;
    blocks += (nq + per_block - 1) / per_block;
    cols += nq;
  }
  for (int q = count; q < 4; ++q) { sg.blk0[q] = 0x7fffffff; sg.col0[q] = 0x7fffffff; }  // never selected
  sg.total = cols;
  const int slices = rows >= 8 * 16 ? kColsumSlices : 1;
  colsum_partial_multi_kernel<T, kV><<<dim3(blocks, slices), kThreads, 0, s>>>(sg, scratch, rows,
                                                                              (rows + slices - 1) / slices);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  colsum_final_multi_kernel<<<(cols + 255) / 256, 256, 0, s>>>(sg, scratch, slices);
  return hipGetLastError();
}

hipError_t launch_transpose_bf16(const bf16_t* src, bf16_t* dst, int rows, int cols, hipStream_t s) {
  if (rows <= 0 || cols <= 0) return hipErrorInvalidValue;
  dim3 grid((cols + 63) / 64, (rows + 63) / 64);
  const bool wide = rows % 64 == 0 && cols % 64 == 0 &&
                    ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) == 0;
  if (wide) transpose_bf16_wide_kernel<<<grid, 256, 0, s>>>((const unsigned short*)src, (unsigned short*)dst, rows, cols);
  else transpose_bf16_kernel<<<grid, 256, 0, s>>>((const unsigned short*)src, (unsigned short*)dst, rows, cols);
  return hipGetLastError();
}

hipError_t launch_fill_f32(float* p, size_t n, float v, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const size_t n4 = (reinterpret_cast<uintptr_t>(p) & 15) == 0 ? n / 4 : 0;
  if (n4 > 0 && n4 <= ((size_t)1 << 39)) fill_f32x4_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, s>>>((float4*)p, n4, v);
  if (n > 4 * n4) fill_f32_kernel<<<grid_for(n - 4 * n4), 256, 0, s>>>(p + 4 * n4, n - 4 * n4, v);
  return hipGetLastError();
}
template <typename T> hipError_t launch_convert_from_f32(const float* src, T* dst, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  convert_from_f32_kernel<T><<<grid_for(n), 256, 0, s>>>(src, dst, n);
  return hipGetLastError();
}
template <typename T> hipError_t launch_convert_to_f32(const T* src, float* dst, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  convert_to_f32_kernel<T><<<grid_for(n), 256, 0, s>>>(src, dst, n);
  return hipGetLastError();
}
// dst[r, c] = (float) src[r * ld + cols[c]]: a few columns of a row-major matrix, for the debug getter
template <typename T>
__global__ void gather_columns_kernel(const T* __restrict__ src, long ld, int rows, const int* __restrict__ cols,
                                      int ncols, float* __restrict__ dst) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)rows * ncols) return;
  const size_t r = i / ncols;
  const int c = (int)(i - r * ncols);
  dst[i] = to_f32(src[r * ld + cols[c]]);
}
template <typename T>
hipError_t launch_gather_columns(const T* src, long ld, int rows, const int* cols, int ncols, float* dst,
                                 hipStream_t s) {
  if (rows <= 0 || ncols <= 0) return hipErrorInvalidValue;
  gather_columns_kernel<T><<<grid_for((size_t)rows * ncols), 256, 0, s>>>(src, ld, rows, cols, ncols, dst);
  return hipGetLastError();
}
template <typename T> hipError_t launch_poke(T* dst, size_t idx, float v, hipStream_t s) {
  poke_kernel<T><<<1, 1, 0, s>>>(dst, idx, v);
  return hipGetLastError();
}

#define ZB_INST(T)                                                                                              \
  template hipError_t launch_layernorm_fwd<T>(const T*, const float*, const float*, T*, float*, int, int, float, \
                                              hipStream_t);                                                      \
  template hipError_t launch_layernorm_bwd<T>(const T*, const T*, const float*, const float*, const T*, T*,      \
                                              float*, float*, float*, int, int, hipStream_t);                    \
  template hipError_t launch_colsum_accum_multi<T>(const void* const*, float* const*, const int*, int, float*,  \
                                                   int, hipStream_t);                                           \
  template hipError_t launch_splitk_layernorm_fwd<T>(const float*, int, size_t, const float*, const T*, T*,      \
                                                     const float*, const float*, T*, float*, int, int, float,    \
                                                     hipStream_t);                                               \
  template hipError_t launch_splitk_layernorm_bwd<T>(const float*, int, size_t, T*, const T*, const float*,      \
                                                     const float*, const T*, T*, float*, float*, float*, int,    \
                                                     int, hipStream_t);                                          \
  template hipError_t launch_convert_from_f32<T>(const float*, T*, size_t, hipStream_t);                         \
  template hipError_t launch_convert_to_f32<T>(const T*, float*, size_t, hipStream_t);                           \
  template hipError_t launch_gather_columns<T>(const T*, long, int, const int*, int, float*, hipStream_t);        \
  template hipError_t launch_poke<T>(T*, size_t, float, hipStream_t);
ZB_INST(float)
ZB_INST(bf16_t)
#undef ZB_INST

}  // namespace zb
