// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// One 256-thread workgroup (4 wavefronts) owns a BM x BN output tile and walks K in steps of 64.
// Both operands are staged in LDS K-contiguous ([row][k], rows padded to 72 elements so that the
// 16-byte fragment reads of 8 consecutive lanes fall into different banks), double buffered, with
// the global loads of step i+1 issued before the MFMAs of step i.  An operand whose memory layout
// has the *row* index contiguous (the weight in the forward GEMM, both operands of the wgrad GEMM)
// is transposed on its way into LDS.
//
// MFMA operand layout (32x32x16): lane l supplies row (l & 31) of its operand and the 8 consecutive
// k values starting at 8*(l >> 5); lane l receives column (l & 31) and rows 8*(v/4) + 4*(l>>5) + v%4
// of the 32x32 result in accumulator element v = 0..15.
#include "gemm_epilogue.h"

namespace zb {

namespace {

constexpr int BK = 64;
constexpr int LDK = BK + 8;  // padded LDS row, elements

template <int ROWS, bool TR>
struct TileLoader {
  // ROWS x 64 tile of an operand.  !TR: element (r,k) at p[r*ld + k]; TR: at p[k*ld + r].
  static constexpr int CHUNKS = ROWS * BK / 8 / 256;  // 16-byte chunks per thread
  uint4 reg[CHUNKS];

  __device__ __forceinline__ void gload(const bf16_t* __restrict__ p, long ld, int r0, int k0) {
#pragma unroll
    for (int j = 0; j < CHUNKS; ++j) {
      const int c = threadIdx.x + 256 * j;
      if (!TR) {
        const int r = c >> 3, kc = c & 7;
        reg[j] = *reinterpret_cast<const uint4*>(p + (long)(r0 + r) * ld + k0 + kc * 8);
      } else {
        const int k = c / (ROWS / 8), rc = c % (ROWS / 8);
        reg[j] = *reinterpret_cast<const uint4*>(p + (long)(k0 + k) * ld + r0 + rc * 8);
      }
    }
  }
  __device__ __forceinline__ void lstore(bf16_t* __restrict__ s) const {
#pragma unroll
    for (int j = 0; j < CHUNKS; ++j) {
      const int c = threadIdx.x + 256 * j;
      if (!TR) {
        const int r = c >> 3, kc = c & 7;
        *reinterpret_cast<uint4*>(s + r * LDK + kc * 8) = reg[j];
      } else {
        const int k = c / (ROWS / 8), rc = c % (ROWS / 8);
        const unsigned short* h = reinterpret_cast<const unsigned short*>(&reg[j]);
        unsigned short* d = reinterpret_cast<unsigned short*>(s) + (rc * 8) * LDK + k;
#pragma unroll
        for (int e = 0; e < 8; ++e) d[e * LDK] = h[e];
      }
    }
  }
};

template <int BM, int BN, int WM, int WN, bool ATR, bool BTR, int MODE>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                       int M, int N, int K, long lda, long ldb, EpiParams epi) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_raw);      // [2][BM][LDK]
  bf16_t* sB = sA + 2 * BM * LDK;                        // [2][BN][LDK]
  constexpr int WAVES_N = BN / WN;
  constexpr int MT = WM / 32, NT = WN / 32;
  static_assert((BM / WM) * (BN / WN) == 4, "four waves per workgroup");

  // workgroup -> tile: consecutive workgroup ids land on different XCDs (8 of them, each with its
  // own L2), so renumber to give each XCD a contiguous run of tiles, M fastest: the tiles that
  // share a weight column block then sit in one L2.
  const int tiles_m = M / BM;
  const int nblk = gridDim.x;
  int pid = blockIdx.x;
  if ((nblk & 7) == 0) pid = (pid & 7) * (nblk >> 3) + (pid >> 3);
  const int m0 = (pid % tiles_m) * BM;
  const int n0 = (pid / tiles_m) * BN;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = (wave / WAVES_N) * WM, wn = (wave % WAVES_N) * WN;
  const int lrow = lane & 31, lk = (lane >> 5) * 8;

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  TileLoader<BM, ATR> la;
  TileLoader<BN, BTR> lb;
  la.gload(A, lda, m0, 0);
  lb.gload(B, ldb, n0, 0);
  la.lstore(sA);
  lb.lstore(sB);
  __syncthreads();

  int buf = 0;
  for (int k0 = 0; k0 < K; k0 += BK) {
    const bool more = k0 + BK < K;
    if (more) {
      la.gload(A, lda, m0, k0 + BK);
      lb.gload(B, ldb, n0, k0 + BK);
    }
    const bf16_t* a_s = sA + buf * BM * LDK + (wm + lrow) * LDK + lk;
    const bf16_t* b_s = sB + buf * BN * LDK + (wn + lrow) * LDK + lk;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[MT], bfr[NT];
#pragma unroll
      for (int i = 0; i < MT; ++i) af[i] = *reinterpret_cast<const bf16x8*>(a_s + i * 32 * LDK + kk * 16);
#pragma unroll
      for (int j = 0; j < NT; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(b_s + j * 32 * LDK + kk * 16);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      la.lstore(sA + (buf ^ 1) * BM * LDK);
      lb.lstore(sB + (buf ^ 1) * BN * LDK);
    }
    __syncthreads();
    buf ^= 1;
  }

#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int n = n0 + wn + j * 32 + lrow;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        epilogue_one<bf16_t, MODE>(epi, m, n, acc[i][j][v]);
      }
    }
}

template <int BM, int BN, int WM, int WN, bool ATR, bool BTR, int MODE>
hipError_t run_cfg(const GemmArgs& g, long lda, long ldb, hipStream_t s) {
  auto kern = gemm_mfma_kernel<BM, BN, WM, WN, ATR, BTR, MODE>;
  constexpr size_t smem = (size_t)2 * (BM + BN) * LDK * sizeof(bf16_t);
  static bool attr_set = false;  // per instantiation; the attribute is per function, not per device state
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int grid = (g.M / BM) * (g.N / BN);
  kern<<<grid, 256, smem, s>>>((const bf16_t*)g.A, (const bf16_t*)g.B, g.M, g.N, g.K, lda, ldb, make_epi(g));
  return hipGetLastError();
}

template <bool ATR, bool BTR, int MODE>
hipError_t run_shape(const GemmArgs& g, long lda, long ldb, hipStream_t s, bool* taken) {
  *taken = true;
  if (g.M % 128 == 0 && g.N % 128 == 0) return run_cfg<128, 128, 64, 64, ATR, BTR, MODE>(g, lda, ldb, s);
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
