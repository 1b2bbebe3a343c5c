// Causal attention forward for head size 128 on the gfx950 matrix cores, tuned variant of the general
// kernel in attention_mfma.hip (same mathematics, same transposed-product formulation, same results
// layout): K and V tiles go global memory -> LDS directly (global_load_lds_dwordx4, no staging
// registers), two workgroups share a compute unit so that one's softmax and loads hide behind the other's
// MFMAs, and the LDS layout is conflict-free on the 64-bank LDS.
//
// LDS tile = [64 keys][128] bf16, rows of 256 B = 16 chunks of 16 B, no padding (the DMA writes 1 KB runs);
// chunk c of row r sits at position c ^ swz(r), swz(r) = ((r & 3) << 2) | ((r >> 2) & 3).  16 consecutive
// rows reading the same columns (16-byte fragment reads) then hit 16 different positions, and the four
// rows that 32 lanes of a transposing read (ds_read_b64_tr_b16, 64 B from each row) touch fall into the four
// quarters of the banks.
#include "zb_common.h"

namespace zb {

namespace {

constexpr int D = 128;
constexpr int QB = 128;  // queries per workgroup (4 waves x 32)
constexpr int KB = 64;   // keys per tile
constexpr int TILE = KB * D;
constexpr float kLn2 = 0.6931471805599453f;

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// global [64][128] tile (row stride ld) -> LDS stage s
__device__ __forceinline__ void dma_tile(const bf16_t* __restrict__ base, long ld, bf16_t* s, int wave, int lane) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int blk = j * 4 + wave;
    const int P = blk * 64 + lane;
    const int row = P >> 4, c = (P & 15) ^ swz(row);
    __builtin_amdgcn_global_load_lds((gptr_t)(base + (long)row * ld + c * 8), (lptr_t)(s + blk * 512), 16, 0, 0);
  }
}
// operand fragment: rows rb..rb+31 of the tile, columns kk*16 .. kk*16+15
__device__ __forceinline__ bf16x8 frag_rowk(const bf16_t* __restrict__ s, int rb, int kk, int lane) {
  const int row = rb + (lane & 31);
  const int chunk = kk * 2 + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(s + row * D + ((chunk ^ swz(row)) << 3));
}
// operand fragment: rows = columns eb..eb+31 of the tile, k = tile rows in accumulator order
// (slots 0-3 = rows kl0 + 4*(lane>>5) + 0..3, slots 4-7 = the same + 8)
__device__ __forceinline__ bf16x8 frag_tr(const bf16_t* __restrict__ s, int eb, int kl0, int lane) {
  const int blk = lane >> 4, a = lane & 15;
  const int e = eb + ((blk & 1) << 4) + ((a & 3) << 2);
  const int kl = kl0 + ((blk >> 1) << 2) + (a >> 2);
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const bf16_t* p0 = s + kl * D + ((((e >> 3) ^ swz(kl)) << 3) | (e & 7));
  const bf16_t* p1 = s + (kl + 8) * D + ((((e >> 3) ^ swz(kl + 8)) << 3) | (e & 7));
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p0);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p1);
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
__device__ __forceinline__ bf16x8 pack_half(const f32x16& t, int half) {
  bf16x8 r;
#pragma unroll
  for (int j = 0; j < 8; ++j) r[j] = (bf16_t)t[half * 8 + j];
  return r;
}
__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ void store4(bf16_t* p, float a, float b, float c, float d) {
  bf16x4 t;
  t[0] = (bf16_t)a; t[1] = (bf16_t)b; t[2] = (bf16_t)c; t[3] = (bf16_t)d;
  *reinterpret_cast<bf16x4*>(p) = t;
}
constexpr int kWaitVm0 = 0 | (7 << 4) | (15 << 8);  // s_waitcnt vmcnt(0) only

__global__ __launch_bounds__(256, 2) void attn_fwd128_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out,
                                                             float* __restrict__ lse, int s, int a, float sl2) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  bf16_t* sK = reinterpret_cast<bf16_t*>(smem_raw);  // [2][TILE]
  bf16_t* sV = sK + 2 * TILE;                        // [2][TILE]
  const int qb = gridDim.x - 1 - blockIdx.x, head = blockIdx.y, bi = blockIdx.z;  // heaviest blocks first
  const int h = a * D;
  const long ld = 3L * h;
  const long tok0 = (long)bi * s;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int hi = lane >> 5, lq = lane & 31;
  const int qw0 = qb * QB + wave * 32;

  const int nkb = 2 * qb + 2;
  const bf16_t* kbase = qkv + tok0 * ld + h + head * D;
  const bf16_t* vbase = kbase + h;
  dma_tile(kbase, ld, sK, wave, lane);
  dma_tile(vbase, ld, sV, wave, lane);

  bf16x8 qf[D / 16];
  {
    const bf16_t* qp = qkv + (tok0 + qw0 + lq) * ld + head * D + hi * 8;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16);
    // have the query fragments arrive here, once, instead of a wait inside the loop
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) asm volatile("" : "+v"(qf[kk]));
  }
  f32x16 o[D / 32];
#pragma unroll
  for (int et = 0; et < D / 32; ++et)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[et][v] = 0.f;
  float m = -INFINITY, l = 0.f;

  for (int jb = 0; jb < nkb; ++jb) {
    __builtin_amdgcn_s_waitcnt(kWaitVm0);  // this wave's part of tile jb has landed
    __builtin_amdgcn_s_barrier();          // everyone's has; everyone is done with the other stage
    if (jb + 1 < nkb) {
      dma_tile(kbase + (long)(jb + 1) * KB * ld, ld, sK + ((jb + 1) & 1) * TILE, wave, lane);
      dma_tile(vbase + (long)(jb + 1) * KB * ld, ld, sV + ((jb + 1) & 1) * TILE, wave, lane);
    }
    const bf16_t* kc = sK + (jb & 1) * TILE;
    const bf16_t* vc = sV + (jb & 1) * TILE;
    const int key0 = jb * KB;
    if (key0 <= qw0 + 31) {  // this wave still has unmasked keys in the tile
      const bool act1 = key0 + 32 <= qw0 + 31;
      f32x16 st[2];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) st[t][v] = 0.f;
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        st[0] = mfma(frag_rowk(kc, 0, kk, lane), qf[kk], st[0]);
        if (act1) st[1] = mfma(frag_rowk(kc, 32, kk, lane), qf[kk], st[1]);
      }
      const bool diag = key0 + KB - 1 > qw0;
      const int myq = qw0 + lq;
      float mx = -INFINITY;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float x = st[t][v] * sl2;
          if (diag) {
            const int key = key0 + t * 32 + (v >> 2) * 8 + hi * 4 + (v & 3);
            if (key > myq) x = -INFINITY;
          }
          st[t][v] = x;
          mx = fmaxf(mx, x);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m, mx);
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);
      float rs = 0.f;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = __builtin_amdgcn_exp2f(st[t][v] - m_new);
          st[t][v] = p;
          rs += p;
        }
      rs += __shfl_xor(rs, 32, 64);
      l = l * alpha + rs;
      m = m_new;
#pragma unroll
      for (int et = 0; et < D / 32; ++et)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[et][v] *= alpha;
      bf16x8 pf[4];
      pf[0] = pack_half(st[0], 0); pf[1] = pack_half(st[0], 1);
      pf[2] = pack_half(st[1], 0); pf[3] = pack_half(st[1], 1);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        if (kk < 2 || act1) {
#pragma unroll
          for (int et = 0; et < D / 32; ++et) o[et] = mfma(frag_tr(vc, et * 32, kk * 16, lane), pf[kk], o[et]);
        }
      }
    }
  }

  const float inv = 1.0f / l;
  bf16_t* op = out + (tok0 + qw0 + lq) * h + head * D + hi * 4;
#pragma unroll
  for (int et = 0; et < D / 32; ++et)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      store4(op + et * 32 + g * 8, o[et][4 * g] * inv, o[et][4 * g + 1] * inv, o[et][4 * g + 2] * inv,
             o[et][4 * g + 3] * inv);
  if (hi == 0) lse[((long)bi * a + head) * s + qw0 + lq] = (m + __builtin_amdgcn_logf(l)) * kLn2;
}

}  // namespace

hipError_t launch_attention_fwd_d128(const AttnArgs& a, hipStream_t s) {
  static bool done = false;
  constexpr size_t smem = (size_t)4 * TILE * sizeof(bf16_t);
  if (!done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_fwd128_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    done = true;
  }
  dim3 grid(a.s / QB, a.a, a.b);
  attn_fwd128_kernel<<<grid, 256, smem, s>>>((const bf16_t*)a.qkv, (bf16_t*)a.out, a.lse, a.s, a.a,
                                             1.4426950408889634f / sqrtf((float)D));
  return hipGetLastError();
}

}  // namespace zb
