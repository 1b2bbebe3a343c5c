// Causal attention for head sizes 128 and 96 on the gfx950 matrix cores, tuned variant of the general
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

constexpr int RP = 128;  // LDS row pitch in elements (256 B) for every head size
constexpr int QB = 128;  // queries per workgroup (4 waves x 32)
constexpr int KB = 64;   // keys per tile
constexpr int TILE = KB * RP;
constexpr float kLn2 = 0.6931471805599453f;

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// global [64][D] tile (row stride ld) -> LDS stage s.  A head size below 128 leaves the chunk positions
// of columns D..127 unused: their lanes fetch a chunk of the same row again (never read from LDS).
template <int D>
__device__ __forceinline__ void dma_tile(const bf16_t* __restrict__ base, long ld, bf16_t* s, int wave, int lane) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int blk = j * 4 + wave;
    const int P = blk * 64 + lane;
    const int row = P >> 4;
    int c = (P & 15) ^ swz(row);
    if (D < 128 && c >= D / 8) c -= D / 8;
    __builtin_amdgcn_global_load_lds((gptr_t)(base + (long)row * ld + c * 8), (lptr_t)(s + blk * 512), 16, 0, 0);
  }
}
// operand fragment: rows rb..rb+31 of the tile, columns kk*16 .. kk*16+15
__device__ __forceinline__ bf16x8 frag_rowk(const bf16_t* __restrict__ s, int rb, int kk, int lane) {
  const int row = rb + (lane & 31);
  const int chunk = kk * 2 + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(s + row * RP + ((chunk ^ swz(row)) << 3));
}
// operand fragment: rows = columns eb..eb+31 of the tile, k = tile rows in accumulator order
// (slots 0-3 = rows kl0 + 4*(lane>>5) + 0..3, slots 4-7 = the same + 8)
__device__ __forceinline__ bf16x8 frag_tr(const bf16_t* __restrict__ s, int eb, int kl0, int lane) {
  const int blk = lane >> 4, a = lane & 15;
  const int e = eb + ((blk & 1) << 4) + ((a & 3) << 2);
  const int kl = kl0 + ((blk >> 1) << 2) + (a >> 2);
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const bf16_t* p0 = s + kl * RP + ((((e >> 3) ^ swz(kl)) << 3) | (e & 7));
  const bf16_t* p1 = s + (kl + 8) * RP + ((((e >> 3) ^ swz(kl + 8)) << 3) | (e & 7));
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

// Workgroup -> (row block, head, sample).  Consecutive workgroup ids go to different XCDs (8, each with
// its own L2); all row blocks of one head are sent to the same XCD so that the head's K/V (or Q/dO) tiles
// are fetched into one L2 only.  `first_heavy`: row blocks in descending order (the last query block has
// the most keys); otherwise ascending (key block 0 sees the most queries).
__device__ __forceinline__ void map_block(int id, int nrb, int a, int b, bool first_heavy, int* rb, int* head,
                                          int* bi) {
  const int heads = a * b;
  int hl, r;
  if ((heads & 7) == 0) {
    // within an XCD: heaviest row blocks of all its heads first, so the light ones fill the tail
    const int xcd = id & 7, local = id >> 3, hpx = heads >> 3;
    hl = (local % hpx) * 8 + xcd;
    r = local / hpx;
  } else {
    hl = id / nrb;
    r = id % nrb;
  }
  *rb = first_heavy ? nrb - 1 - r : r;
  *head = hl % a;
  *bi = hl / a;
}

// Forward.  A workgroup owns 128 query rows of one head and has eight waves in two groups of four: group g
// takes the key tiles g, g + 2, ... (a causal row block has an even number of 64-key tiles, so both groups get
// the same number), each with its own running maximum, sum and output accumulators, and at the end group 0
// merges group 1's state into its own (the usual rescaling by 2^(m_g - m)) and writes the rows.  The chain of
// dependent tiles of the heaviest row block is then 8 long instead of 16, and the two groups' waves share
// the SIMDs, one's MFMAs running while the other is in its softmax.  Each group has a two-stage ring of K and
// V tiles (128 KB in all, one workgroup per CU); group 1's state travels through the same memory.
template <int D>
__global__ __launch_bounds__(512, 2) void attn_fwd128_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out,
                                                             float* __restrict__ lse, int s, int a, float sl2) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  int qb, head, bi;
  map_block(blockIdx.x, s / QB, a, gridDim.x / (a * (s / QB)), true, &qb, &head, &bi);  // heaviest blocks first
  const int h = a * D;
  const long ld = 3L * h;
  const long tok0 = (long)bi * s;
  const int wave8 = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int grp = wave8 >> 2, wave = wave8 & 3;
  const int hi = lane >> 5, lq = lane & 31;
  const int qw0 = qb * QB + wave * 32;
  bf16_t* sK = reinterpret_cast<bf16_t*>(smem_raw) + grp * 4 * TILE;  // this group's [2][TILE]
  bf16_t* sV = sK + 2 * TILE;                                         // and its [2][TILE]

  const int nit = qb + 1;  // tiles per group
  const bf16_t* kbase = qkv + tok0 * ld + h + head * D;
  const bf16_t* vbase = kbase + h;
  dma_tile<D>(kbase + (long)grp * KB * ld, ld, sK, wave, lane);
  dma_tile<D>(vbase + (long)grp * KB * ld, ld, sV, wave, lane);

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

  for (int i = 0; i < nit; ++i) {
    const int jb = 2 * i + grp;
    __builtin_amdgcn_s_waitcnt(kWaitVm0);  // this wave's part of tile jb has landed
    __builtin_amdgcn_s_barrier();          // everyone's has; everyone is done with the other stage
    if (i + 1 < nit) {
      dma_tile<D>(kbase + (long)(jb + 2) * KB * ld, ld, sK + ((i + 1) & 1) * TILE, wave, lane);
      dma_tile<D>(vbase + (long)(jb + 2) * KB * ld, ld, sV + ((i + 1) & 1) * TILE, wave, lane);
    }
    const bf16_t* kc = sK + (i & 1) * TILE;
    const bf16_t* vc = sV + (i & 1) * TILE;
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

  // group 1 hands its state to group 0 through LDS: [wave][register][lane] floats, then m and l
  constexpr int NR = (D / 32) * 16;
  float* xo = reinterpret_cast<float*>(smem_raw);  // [4][NR][64]
  float* xm = xo + 4 * NR * 64;                    // [4][2][64]
  __builtin_amdgcn_s_barrier();  // every wave is done with the rings (no load is in flight: the last wait was for all)
  if (grp == 1) {
#pragma unroll
    for (int et = 0; et < D / 32; ++et)
#pragma unroll
      for (int v = 0; v < 16; ++v) xo[(wave * NR + et * 16 + v) * 64 + lane] = o[et][v];
    xm[(wave * 2 + 0) * 64 + lane] = m;
    xm[(wave * 2 + 1) * 64 + lane] = l;
  }
  __syncthreads();
  if (grp == 1) return;
  {
    // a wave of group 1 that saw no unmasked key has m = -inf, l = 0, o = 0: its factor is 0
    const float m1 = xm[(wave * 2 + 0) * 64 + lane], l1 = xm[(wave * 2 + 1) * 64 + lane];
    const float m_new = fmaxf(m, m1);  // group 0 always holds key 0: finite
    const float a0 = __builtin_amdgcn_exp2f(m - m_new), a1 = __builtin_amdgcn_exp2f(m1 - m_new);
    l = l * a0 + l1 * a1;
    m = m_new;
#pragma unroll
    for (int et = 0; et < D / 32; ++et)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[et][v] = o[et][v] * a0 + xo[(wave * NR + et * 16 + v) * 64 + lane] * a1;
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


// ------------------------------------------------------------------------------------------------
// backward, D_i = dO_i . O_i.  A workgroup takes 64 consecutive rows of one head, 16 per wavefront (one row
// per step, two elements per lane), and writes their sums as one contiguous run.
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_bwd128_prep_kernel(const bf16_t* __restrict__ o,
                                                               const bf16_t* __restrict__ dout,
                                                               float* __restrict__ dvec, int s, int a) {
  const int head = blockIdx.y, bi = blockIdx.z;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i0 = blockIdx.x * 64 + wave * 16;
  const long off = ((long)bi * s + i0) * a * D + head * D + lane * 2;
  const long rs = (long)a * D;
  float mine = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float acc = 0.f;
    if (lane * 2 < D) {
      const bf16x2 x = *reinterpret_cast<const bf16x2*>(o + off + r * rs);
      const bf16x2 y = *reinterpret_cast<const bf16x2*>(dout + off + r * rs);
      acc = (float)x[0] * (float)y[0] + (float)x[1] * (float)y[1];
    }
    acc = wave_sum(acc);
    if (lane == r) mine = acc;
  }
  if (lane < 16) dvec[((long)bi * a + head) * s + i0 + lane] = mine;
}

// ------------------------------------------------------------------------------------------------
// backward, dQ: workgroup = 128 queries, loop over key tiles up to the diagonal (same pipeline as forward)
// ------------------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void attn_bwd128_dq_body(unsigned char* smem_raw, int qb, int head, int bi,
                                                    const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                    const float* __restrict__ lse, const float* __restrict__ dvec,
                                                    bf16_t* __restrict__ dqkv, int s, int a, float scale) {
  bf16_t* sK = reinterpret_cast<bf16_t*>(smem_raw);  // [2][TILE]
  bf16_t* sV = sK + 2 * TILE;                        // [2][TILE]
  const int h = a * D;
  const long ld = 3L * h;
  const long tok0 = (long)bi * s;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int hi = lane >> 5, lq = lane & 31;
  const int qw0 = qb * QB + wave * 32;
  const float sl2 = scale * 1.4426950408889634f;

  const int nkb = 2 * qb + 2;
  const bf16_t* kbase = qkv + tok0 * ld + h + head * D;
  const bf16_t* vbase = kbase + h;
  auto issue = [&](int t) {  // 8 DMA instructions per wave
    dma_tile<D>(kbase + (long)t * KB * ld, ld, sK + (t & 1) * TILE, wave, lane);
    dma_tile<D>(vbase + (long)t * KB * ld, ld, sV + (t & 1) * TILE, wave, lane);
  };
  issue(0);

  bf16x8 qf[D / 16], dof[D / 16];
  const long srow = ((long)bi * a + head) * s + qw0 + lq;
  float lse2 = lse[srow] * 1.4426950408889634f;
  float Dq = dvec[srow];
  {
    const bf16_t* qp = qkv + (tok0 + qw0 + lq) * ld + head * D + hi * 8;
    const bf16_t* dp = dout + (tok0 + qw0 + lq) * h + head * D + hi * 8;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16);
      dof[kk] = *reinterpret_cast<const bf16x8*>(dp + kk * 16);
    }
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) asm volatile("" : "+v"(qf[kk]), "+v"(dof[kk]));
    asm volatile("" : "+v"(lse2), "+v"(Dq));
  }
  f32x16 dq[D / 32];
#pragma unroll
  for (int et = 0; et < D / 32; ++et)
#pragma unroll
    for (int v = 0; v < 16; ++v) dq[et][v] = 0.f;

  for (int jb = 0; jb < nkb; ++jb) {
    __builtin_amdgcn_s_waitcnt(kWaitVm0);  // tile jb has landed
    __builtin_amdgcn_s_barrier();
    if (jb + 1 < nkb) issue(jb + 1);
    const bf16_t* kc = sK + (jb & 1) * TILE;
    const bf16_t* vc = sV + (jb & 1) * TILE;
    const int key0 = jb * KB;
    if (key0 <= qw0 + 31) {
      const bool act1 = key0 + 32 <= qw0 + 31;
      f32x16 st[2], dpt[2];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) st[t][v] = dpt[t][v] = 0.f;
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        st[0] = mfma(frag_rowk(kc, 0, kk, lane), qf[kk], st[0]);
        dpt[0] = mfma(frag_rowk(vc, 0, kk, lane), dof[kk], dpt[0]);
        if (act1) {
          st[1] = mfma(frag_rowk(kc, 32, kk, lane), qf[kk], st[1]);
          dpt[1] = mfma(frag_rowk(vc, 32, kk, lane), dof[kk], dpt[1]);
        }
      }
      const bool diag = key0 + KB - 1 > qw0;
      const int myq = qw0 + lq;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float p = __builtin_amdgcn_exp2f(st[t][v] * sl2 - lse2);
          if (diag) {
            const int key = key0 + t * 32 + (v >> 2) * 8 + hi * 4 + (v & 3);
            if (key > myq) p = 0.f;
          }
          st[t][v] = p * (dpt[t][v] - Dq);
        }
      bf16x8 dsf[4];
      dsf[0] = pack_half(st[0], 0); dsf[1] = pack_half(st[0], 1);
      dsf[2] = pack_half(st[1], 0); dsf[3] = pack_half(st[1], 1);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        if (kk < 2 || act1) {
#pragma unroll
          for (int et = 0; et < D / 32; ++et) dq[et] = mfma(frag_tr(kc, et * 32, kk * 16, lane), dsf[kk], dq[et]);
        }
      }
    }
  }
  bf16_t* op = dqkv + (tok0 + qw0 + lq) * ld + head * D + hi * 4;
#pragma unroll
  for (int et = 0; et < D / 32; ++et)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      store4(op + et * 32 + g * 8, dq[et][4 * g] * scale, dq[et][4 * g + 1] * scale, dq[et][4 * g + 2] * scale,
             dq[et][4 * g + 3] * scale);
}

// ------------------------------------------------------------------------------------------------
// backward, dK and dV: workgroup = 128 keys, loop over query tiles from the diagonal to the end.
// Per tile and wave: 4 + 4 DMA instructions for Q and dO and one 4-byte-per-lane DMA for the row
// statistics (waves 0/1 fetch lse / D, waves 2/3 fetch the same again into a spare area so that every
// wave has the same number of loads in flight).
// ------------------------------------------------------------------------------------------------
// dK and dV with two workgroups per CU: a workgroup owns 128 keys and, of dK and dV, the D / NH columns of
// column part `half` (head size 128: NH = 2 halves of 64 columns, 64 accumulator registers instead of 128;
// head size 96: NH = 1, all 96).  With the two 32-query halves of a tile taken one after the other a wave
// stays under 256 registers; two workgroups (of this kind or of the dQ kind) then share a CU and one's MFMAs
// run while the other waits for LDS or the exponentials.  With NH = 2, S and dP are computed by both halves;
// every dK / dV element is the same chain of MFMA additions whatever NH (tile by tile, k blocks 0..3).
// Two-stage ring (tile ib+1 is fetched while ib is used).
template <int D, int NH>
__device__ __forceinline__ void attn_bwd128_dkv_half_body(unsigned char* smem_raw, int kb, int half, int head, int bi,
                                                          const bf16_t* __restrict__ qkv,
                                                          const bf16_t* __restrict__ dout,
                                                          const float* __restrict__ lse,
                                                          const float* __restrict__ dvec,
                                                          bf16_t* __restrict__ dqkv, int s, int a, float scale) {
  static_assert((D / 32) % NH == 0, "whole 32-column blocks per workgroup");
  constexpr int NE = D / 32 / NH;  // 32-column blocks of dK and dV this workgroup owns
  bf16_t* sQ = reinterpret_cast<bf16_t*>(smem_raw);  // [2][TILE]
  bf16_t* sO = sQ + 2 * TILE;                        // [2][TILE]  dO tiles
  float* sS = reinterpret_cast<float*>(sO + 2 * TILE);  // [2][4][64]: lse, D, spare, spare
  const int h = a * D;
  const long ld = 3L * h;
  const long tok0 = (long)bi * s;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int hi = lane >> 5, lk = lane & 31;
  const int kw0 = kb * QB + wave * 32;
  const float sl2 = scale * 1.4426950408889634f;

  const int ib0 = kb * (QB / KB), nib = s / KB;
  const bf16_t* qbase = qkv + tok0 * ld + head * D;
  const bf16_t* obase = dout + tok0 * h + head * D;
  const float* stat = ((wave & 1) ? dvec : lse) + ((long)bi * a + head) * s;
  auto issue = [&](int ib) {  // 9 DMA instructions per wave
    const int st = (ib - ib0) & 1;
    dma_tile<D>(qbase + (long)ib * KB * ld, ld, sQ + st * TILE, wave, lane);
    dma_tile<D>(obase + (long)ib * KB * h, h, sO + st * TILE, wave, lane);
    __builtin_amdgcn_global_load_lds((gptr_t)(stat + ib * KB + lane), (lptr_t)(sS + (st * 4 + wave) * 64), 4, 0, 0);
  };
  issue(ib0);

  bf16x8 kf[D / 16], vf[D / 16];
  {
    const bf16_t* kp = qkv + (tok0 + kw0 + lk) * ld + h + head * D + hi * 8;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      kf[kk] = *reinterpret_cast<const bf16x8*>(kp + kk * 16);
      vf[kk] = *reinterpret_cast<const bf16x8*>(kp + h + kk * 16);
    }
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) asm volatile("" : "+v"(kf[kk]), "+v"(vf[kk]));
  }
  f32x16 dk[NE], dv[NE];
#pragma unroll
  for (int et = 0; et < NE; ++et)
#pragma unroll
    for (int v = 0; v < 16; ++v) dk[et][v] = dv[et][v] = 0.f;

  for (int ib = ib0; ib < nib; ++ib) {
    __builtin_amdgcn_s_waitcnt(kWaitVm0);  // tile ib has landed
    __builtin_amdgcn_s_barrier();          // for everyone, and everyone is done with the other stage
    if (ib + 1 < nib) issue(ib + 1);
    const int stage = (ib - ib0) & 1;
    const bf16_t* qc = sQ + stage * TILE;
    const bf16_t* oc = sO + stage * TILE;
    const float* lc = sS + stage * 256;
    const float* dc = lc + 64;
    const int q0 = ib * KB;
    if (q0 + KB - 1 >= kw0) {  // some query of the tile can see this wave's keys
      const bool act0 = q0 + 31 >= kw0;
      const bool diag = q0 < kw0 + 31;
      const int mykey = kw0 + lk;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        if (t == 0 && !act0) continue;
        f32x16 st, dpt;
#pragma unroll
        for (int v = 0; v < 16; ++v) st[v] = dpt[v] = 0.f;
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) {
          st = mfma(frag_rowk(qc, t * 32, kk, lane), kf[kk], st);
          dpt = mfma(frag_rowk(oc, t * 32, kk, lane), vf[kk], dpt);
        }
        f32x16 pt;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int qi = t * 32 + g * 8 + hi * 4;
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(lc + qi);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(dc + qi);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int v = g * 4 + i;
            float p = __builtin_amdgcn_exp2f(st[v] * sl2 - l4[i] * 1.4426950408889634f);
            if (diag && mykey > q0 + qi + i) p = 0.f;
            pt[v] = p;
            st[v] = p * (dpt[v] - d4[i]);
          }
        }
        bf16x8 pf[2], dsf[2];
        pf[0] = pack_half(pt, 0); pf[1] = pack_half(pt, 1);
        dsf[0] = pack_half(st, 0); dsf[1] = pack_half(st, 1);
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
#pragma unroll
          for (int et = 0; et < NE; ++et) {
            const int eb = (half * NE + et) * 32;
            dv[et] = mfma(frag_tr(oc, eb, (t * 2 + k2) * 16, lane), pf[k2], dv[et]);
            dk[et] = mfma(frag_tr(qc, eb, (t * 2 + k2) * 16, lane), dsf[k2], dk[et]);
          }
        }
      }
    }
  }
  bf16_t* kp = dqkv + (tok0 + kw0 + lk) * ld + h + head * D + half * (NE * 32) + hi * 4;
#pragma unroll
  for (int et = 0; et < NE; ++et)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      store4(kp + et * 32 + g * 8, dk[et][4 * g] * scale, dk[et][4 * g + 1] * scale, dk[et][4 * g + 2] * scale,
             dk[et][4 * g + 3] * scale);
      store4(kp + h + et * 32 + g * 8, dv[et][4 * g], dv[et][4 * g + 1], dv[et][4 * g + 2], dv[et][4 * g + 3]);
    }
}

// dK/dV and dQ in one launch: they are independent (both recompute S), and their workgroups have very
// uneven lengths (causal: 1 to 16 tiles), so short workgroups of one kind fill the CUs that the other kind
// leaves early.  Two workgroups per CU; per head NH + 1 workgroups for each block index (the NH column parts
// of dK/dV, then dQ), issued heaviest block first over all kinds, every head on one XCD.
template <int D>
__global__ __launch_bounds__(256, 2) void attn_bwd128_kernel(const bf16_t* __restrict__ qkv,
                                                             const bf16_t* __restrict__ dout,
                                                             const float* __restrict__ lse,
                                                             const float* __restrict__ dvec,
                                                             bf16_t* __restrict__ dqkv, int s, int a, int nb, int per,
                                                             float scale) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  constexpr int NH = D == 128 ? 2 : 1, NK = NH + 1;
  const int id = blockIdx.x, nrb = s / QB;
  const int heads = a * nb;
  int blk, head, bi, kind;  // kind < NH: dK/dV column part; NH: dQ
  if ((heads & 7) == 0) {
    const int xcd = id & 7, local = id >> 3, hpx = heads >> 3;
    const int level = local / (NK * hpx), rem = local - level * NK * hpx;  // level 0: the blocks with the most tiles
    kind = rem / hpx;
    const int hl = (rem - kind * hpx) * 8 + xcd;
    blk = kind < NH ? level : nrb - 1 - level;
    head = hl % a;
    bi = hl / a;
  } else {
    kind = id / per;
    map_block(id - kind * per, nrb, a, nb, kind == NH, &blk, &head, &bi);
  }
  if (kind < NH) attn_bwd128_dkv_half_body<D, NH>(smem_raw, blk, kind, head, bi, qkv, dout, lse, dvec, dqkv, s, a, scale);
  else attn_bwd128_dq_body<D>(smem_raw, blk, head, bi, qkv, dout, lse, dvec, dqkv, s, a, scale);
}

template <int D> hipError_t run_fwd_dma(const AttnArgs& a, hipStream_t s) {
  static bool done = false;
  constexpr size_t smem = (size_t)8 * TILE * sizeof(bf16_t);  // two groups x (K, V) x two stages
  static_assert(smem >= ((size_t)4 * (D / 32) * 16 * 64 + 4 * 2 * 64) * sizeof(float), "group 1's state fits");
  if (!done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_fwd128_kernel<D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    done = true;
  }
  dim3 grid((a.s / QB) * a.a * a.b);
  attn_fwd128_kernel<D><<<grid, 512, smem, s>>>((const bf16_t*)a.qkv, (bf16_t*)a.out, a.lse, a.s, a.a,
                                                1.4426950408889634f / sqrtf((float)D));
  return hipGetLastError();
}

template <int D> hipError_t run_bwd_dma(const AttnArgs& a, hipStream_t s) {
  static bool done = false;
  constexpr size_t smem_q = (size_t)4 * TILE * sizeof(bf16_t);
  constexpr int kv_stages = 2;
  constexpr size_t smem_kv = (size_t)2 * kv_stages * TILE * sizeof(bf16_t) + kv_stages * 4 * 64 * sizeof(float);
  constexpr size_t smem = smem_kv > smem_q ? smem_kv : smem_q;
  static_assert(2 * smem <= 160 * 1024, "two workgroups per CU");
  if (!done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bwd128_kernel<D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    done = true;
  }
  const float scale = 1.0f / sqrtf((float)D);
  dim3 grid1(a.s / 64, a.a, a.b);
  attn_bwd128_prep_kernel<D><<<grid1, 256, 0, s>>>((const bf16_t*)a.o, (const bf16_t*)a.dout, a.dvec, a.s, a.a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int per = (a.s / QB) * a.a * a.b;
  attn_bwd128_kernel<D><<<(D == 128 ? 3 : 2) * per, 256, smem, s>>>((const bf16_t*)a.qkv, (const bf16_t*)a.dout, a.lse,
                                                                    a.dvec, (bf16_t*)a.dqkv, a.s, a.a, a.b, per, scale);
  return hipGetLastError();
}

}  // namespace

// head sizes 96 and 128 (a.s a multiple of 128 tokens, checked by the caller)
hipError_t launch_attention_fwd_d128(const AttnArgs& a, hipStream_t s) {
  if (a.d == 128) return run_fwd_dma<128>(a, s);
  if (a.d == 96) return run_fwd_dma<96>(a, s);
  return hipErrorInvalidValue;
}
hipError_t launch_attention_bwd_d128(const AttnArgs& a, hipStream_t s) {
  if (a.d == 128) return run_bwd_dma<128>(a, s);
  if (a.d == 96) return run_bwd_dma<96>(a, s);
  return hipErrorInvalidValue;
}

}  // namespace zb
