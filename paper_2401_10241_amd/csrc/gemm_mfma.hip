// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// One 512-thread workgroup (8 wavefronts, 2 x 4) owns a BM x 256 output tile (BM = 256 or 128) and
// walks K in steps of 32 through a ring of four LDS stages.  Tiles travel global memory -> LDS
// directly (global_load_lds_dwordx4: each lane's 16 bytes land at consecutive LDS addresses, no
// registers in between); three tiles are in flight while the MFMAs of a fourth run.  Per step:
// wait until this wave's loads of the current tile have landed (s_waitcnt vmcnt), one barrier
// (all waves' loads landed, all waves done with the stage about to be refilled), issue the loads of
// the tile three steps ahead, then fragments + MFMAs.
//
// LDS layouts (no padding: the DMA writes 1 KB runs; conflicts are avoided by choosing WHICH global
// chunk each lane fetches).  The LDS has 64 banks of 4 bytes; 16-byte accesses go 16 lanes at a time,
// 8-byte accesses 32 lanes at a time.
//   K-contiguous source ([row][k] in memory):  LDS [R][32], 64 B per row = 4 chunks of 16 B; chunk c of
//     row r sits at position c ^ ((r >> 2) & 3): 16 consecutive rows reading the same k cover all banks.
//   row-contiguous source ([k][row] in memory: the weight in the forward GEMM, both operands of the
//     wgrad GEMM): LDS [32][R]; chunk c of k-line k sits at position c ^ ((k & 3) << 2).  Read back with
//     the transposing LDS load ds_read_b64_tr_b16: within 16 lanes, lane a points at 4 consecutive rows
//     (a & 3) * 4 of k-line (a >> 2) and receives, as lane r, the 4 k values of row r.  32 lanes read 64 B
//     from each of four k-lines; the swizzle puts those in different quarters of the banks.
//
// MFMA 32x32x16 operand layout: lane l supplies row (l & 31) of its operand and the 8 consecutive k
// starting at 8 * (l >> 5); it receives column (l & 31) and rows 8*(v/4) + 4*(l >> 5) + v%4 of the
// 32 x 32 result in accumulator element v.
#include "gemm_epilogue.h"
#ifndef ZB_DIAG_DMA_COND
#define ZB_DIAG_DMA_COND
#endif
#ifndef ZB_DIAG_MFMA
#define ZB_DIAG_MFMA(x) x
#endif

namespace zb {

namespace {

constexpr int BK = 32;
constexpr int BN = 256;
constexpr int NTHREADS = 512;
constexpr int WN = 64;  // wave tile columns

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

template <int R> struct Tile {
  static constexpr int ELEMS = R * BK;
  static constexpr int WAVE_LOADS = R / 128;  // 1 KB DMA instructions per wave per tile
};

// s_waitcnt immediate that waits for vmcnt <= n and nothing else (gfx9 encoding)
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// global -> LDS, one R x 32 operand tile; s = LDS base of the tile's stage
template <int R, bool TR>
__device__ __forceinline__ void dma_tile(const bf16_t* __restrict__ p, long ld, int r0, int k0, bf16_t* s, int wave,
                                         int lane) {
#pragma unroll
  for (int j = 0; j < Tile<R>::WAVE_LOADS; ++j) {
    const int blk = j * 8 + wave;     // which 1 KB run of the tile
    const int P = blk * 64 + lane;    // 16-byte chunk position in LDS
    const bf16_t* g;
    if constexpr (!TR) {
      const int r = P >> 2, c = (P & 3) ^ ((r >> 2) & 3);
      g = p + (long)(r0 + r) * ld + k0 + c * 8;
    } else {
      constexpr int CPL = R / 8;      // chunks per k-line
      const int k = P / CPL, c = (P % CPL) ^ ((k & 3) << 2);
      g = p + (long)(k0 + k) * ld + r0 + c * 8;
    }
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                     (__attribute__((address_space(3))) void*)(s + blk * 512), 16, 0, 0);
  }
}

// LDS -> one MFMA operand fragment: rows rb .. rb+31 of the tile, k = kk*16 .. kk*16+15
template <int R, bool TR>
__device__ __forceinline__ bf16x8 lfrag(const bf16_t* __restrict__ s, int rb, int kk, int lane) {
  if constexpr (!TR) {
    const int r = rb + (lane & 31);
    const int chunk = kk * 2 + (lane >> 5);
    return *reinterpret_cast<const bf16x8*>(s + r * BK + ((chunk ^ ((r >> 2) & 3)) << 3));
  } else {
    const int blk = lane >> 4, a = lane & 15;
    const int row = rb + ((blk & 1) << 4) + ((a & 3) << 2);
    const int k = kk * 16 + ((blk >> 1) << 3) + (a >> 2);
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    const bf16_t* p0 = s + k * R + ((((row >> 3) ^ ((k & 3) << 2)) << 3) | (row & 7));
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0 + 4 * R));  // k + 4: same swizzle
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
}

template <int BM, int STAGES, bool ATR, bool BTR, int MODE>
__global__ __launch_bounds__(NTHREADS) void gemm_mfma_kernel(const bf16_t* __restrict__ A,
                                                            const bf16_t* __restrict__ B, int M, int N, int K,
                                                            long lda, long ldb, EpiParams epi) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  typedef Tile<BM> TA;
  typedef Tile<BN> TB;
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_raw);  // [STAGES][TA::ELEMS]
  bf16_t* sB = sA + STAGES * TA::ELEMS;              // [STAGES][TB::ELEMS]
  constexpr int WM = BM / 2;
  constexpr int MT = WM / 32, NT = WN / 32;
  constexpr int LOADS = TA::WAVE_LOADS + TB::WAVE_LOADS;  // DMA instructions per wave per k-step

  // Consecutive workgroup ids go to different XCDs (8, each with its own L2): renumber so that every
  // XCD gets a contiguous run of tiles, M fastest, and tiles that share a weight block share an L2.
  const int tiles_m = M / BM;
  const int nblk = gridDim.x;
  int pid = blockIdx.x;
  if ((nblk & 7) == 0) pid = (pid & 7) * (nblk >> 3) + (pid >> 3);
  const int m0 = (pid % tiles_m) * BM;
  const int n0 = (pid / tiles_m) * BN;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = (wave >> 2) * WM, wn = (wave & 3) * WN;

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = K / BK;
#pragma unroll
  for (int t = 0; t < STAGES - 1; ++t)
    if (t < nk) {
      dma_tile<BM, ATR>(A, lda, m0, t * BK, sA + t * TA::ELEMS, wave, lane);
      dma_tile<BN, BTR>(B, ldb, n0, t * BK, sB + t * TB::ELEMS, wave, lane);
    }

  for (int it = 0; it < nk; ++it) {
    // tiles it+1 .. it+STAGES-2 may still be in flight; near the end fewer were issued, so wait for all
    if (it + STAGES - 2 < nk) __builtin_amdgcn_s_waitcnt(vmcnt_imm(LOADS * (STAGES - 2)));
    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __builtin_amdgcn_s_barrier();
    const int nt = it + STAGES - 1;
    if (nt < nk ZB_DIAG_DMA_COND) {  // refill the stage that step it-1 used
      dma_tile<BM, ATR>(A, lda, m0, nt * BK, sA + (nt % STAGES) * TA::ELEMS, wave, lane);
      dma_tile<BN, BTR>(B, ldb, n0, nt * BK, sB + (nt % STAGES) * TB::ELEMS, wave, lane);
    }
    const bf16_t* a_s = sA + (it % STAGES) * TA::ELEMS;
    const bf16_t* b_s = sB + (it % STAGES) * TB::ELEMS;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[MT], bfr[NT];
#pragma unroll
      for (int i = 0; i < MT; ++i) af[i] = lfrag<BM, ATR>(a_s, wm + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < NT; ++j) bfr[j] = lfrag<BN, BTR>(b_s, wn + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          ZB_DIAG_MFMA(acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0));
    }
  }

  const int lrow = lane & 31, lhi = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int n = n0 + wn + j * 32 + lrow;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm + i * 32 + (v >> 2) * 8 + lhi + (v & 3);
        epilogue_one<bf16_t, MODE>(epi, m, n, acc[i][j][v]);
      }
    }
}

template <int BM, int STAGES, bool ATR, bool BTR, int MODE>
hipError_t run_cfg(const GemmArgs& g, long lda, long ldb, hipStream_t s) {
  auto kern = gemm_mfma_kernel<BM, STAGES, ATR, BTR, MODE>;
  constexpr size_t smem = (size_t)STAGES * (Tile<BM>::ELEMS + Tile<BN>::ELEMS) * sizeof(bf16_t);
  static_assert(smem <= 160 * 1024, "LDS budget");
  static bool attr_set = false;  // one device per process in this library
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int grid = (g.M / BM) * (g.N / BN);
  kern<<<grid, NTHREADS, smem, s>>>((const bf16_t*)g.A, (const bf16_t*)g.B, g.M, g.N, g.K, lda, ldb, make_epi(g));
  return hipGetLastError();
}

template <bool ATR, bool BTR, int MODE>
hipError_t run_shape(const GemmArgs& g, long lda, long ldb, hipStream_t s, bool* taken) {
  *taken = true;
  if (g.N % BN == 0) {
    // Rounds of tiles over the 256 CUs times the tile height; the taller tile does about 1.25x the
    // work per cycle, so it wins only when it does not cost an extra, mostly empty round.
    const long t256 = g.M % 256 == 0 ? (long)(g.M / 256) * (g.N / BN) : 0;
    const long t128 = g.M % 128 == 0 ? (long)(g.M / 128) * (g.N / BN) : 0;
    const double c256 = t256 ? (double)((t256 + 255) / 256) * 256.0 / 1.25 : 1e30;
    const double c128 = t128 ? (double)((t128 + 255) / 256) * 128.0 : 1e30;
    if (t256 && c256 <= c128 && MODE != EPI_ACCUM_F32) return run_cfg<256, 4, ATR, BTR, MODE>(g, lda, ldb, s);
    if (t128) {
      // more tiles than CUs: three stages (72 KB) let two workgroups share a CU, so one's epilogue and
      // pipeline fill hide behind the other's MFMAs; otherwise one workgroup per CU with a deeper ring
      if (t128 > 256) return run_cfg<128, 3, ATR, BTR, MODE>(g, lda, ldb, s);
      return run_cfg<128, 4, ATR, BTR, MODE>(g, lda, ldb, s);
    }
  }
  *taken = false;
  return hipSuccess;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

template <typename T> hipError_t launch_gemm_mfma(const GemmArgs& g, hipStream_t s, bool* taken) {
  *taken = false;
  return hipSuccess;
}

template <> hipError_t launch_gemm_mfma<bf16_t>(const GemmArgs& g, hipStream_t s, bool* taken) {
  *taken = false;
  const bool atr = g.a_sm == 1 && g.a_sk != 1, btr = g.b_sn == 1 && g.b_sk != 1;
  const long lda = atr ? g.a_sk : g.a_sm, ldb = btr ? g.b_sk : g.b_sn;
  if (g.K % BK != 0 || lda % 8 != 0 || ldb % 8 != 0 || !aligned16(g.A) || !aligned16(g.B)) return hipSuccess;
  if (!atr && btr) {  // forward: X[M,K] * W[K,N]
    if (g.epilogue == EPI_BIAS) return run_shape<false, true, EPI_BIAS>(g, lda, ldb, s, taken);
    if (g.epilogue == EPI_BIAS_RESID) return run_shape<false, true, EPI_BIAS_RESID>(g, lda, ldb, s, taken);
    if (g.epilogue == EPI_BIAS_GELU) return run_shape<false, true, EPI_BIAS_GELU>(g, lda, ldb, s, taken);
  } else if (!atr && !btr) {  // dgrad: dY[M,K'] * W[N,K']^T
    if (g.epilogue == EPI_STORE) return run_shape<false, false, EPI_STORE>(g, lda, ldb, s, taken);
    if (g.epilogue == EPI_DGELU) return run_shape<false, false, EPI_DGELU>(g, lda, ldb, s, taken);
  } else if (atr && btr) {  // wgrad: X[K,M]^T * dY[K,N]
    if (g.epilogue == EPI_ACCUM_F32) return run_shape<true, true, EPI_ACCUM_F32>(g, lda, ldb, s, taken);
  }
  return hipSuccess;
}

template hipError_t launch_gemm_mfma<float>(const GemmArgs&, hipStream_t, bool*);

}  // namespace zb
