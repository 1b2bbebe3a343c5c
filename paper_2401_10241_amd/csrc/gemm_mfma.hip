// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
//   C[M,N] (epilogue)= A * B, with B always given "row-contiguous" ([k][n] in memory, n contiguous: the
//   weight W[in][out] in the forward GEMM, the transposed weight copy in the dgrad GEMM, dY in the wgrad
//   GEMM) and A either K-contiguous ([m][k]: activations in forward / dgrad) or row-contiguous ([k][m]:
//   the stashed layer input in wgrad).
//
// The wgrad GEMM (both operands row-contiguous, fp32 accumulate into C) has a kernel of its own below.
//
// One 512-thread workgroup (8 wavefronts, 2 x 4) owns a BM x 256 output tile (BM = 256 or 128) and walks K
// in steps of 32.  Tiles travel global memory -> LDS directly (global_load_lds_dwordx4: each lane's 16
// bytes land at consecutive LDS addresses, no registers in between) into rings of LDS stages, several
// steps ahead of the MFMAs.  Per step: wait until this wave's loads of the current tiles have landed
// (s_waitcnt vmcnt with the number of younger loads that may stay in flight), one barrier (all waves'
// loads landed, all waves done with the stage about to be refilled), issue the loads for the step
// BS-1 ahead, then fragments + MFMAs.
//
// LDS layouts (no padding: the DMA writes 1 KB runs; bank conflicts are avoided by choosing WHICH global
// chunk each lane fetches).  The LDS has 64 banks of 4 bytes; 16-byte accesses go 16 lanes at a time,
// 8-byte accesses 32 lanes at a time.
//   row-contiguous source: ring of BS stages of [32 k][R]; chunk c (16 B) of k-line k sits at position
//     c ^ ((k & 3) << 2).  Read back with the transposing LDS load ds_read_b64_tr_b16: within 16 lanes,
//     lane a points at 4 consecutive rows (a & 3) * 4 of k-line (a >> 2) and receives, as lane r, the 4 k
//     values of row r.  32 lanes read 64 B from each of four k-lines; the swizzle puts those in
//     different quarters of the banks.
//   K-contiguous source: 64 k at a time (128-byte rows, so every fetched cache line is used whole), two or
//     three stages of [BM][64] refilled every other step; chunk c of row r sits at position
//     c ^ ((r >> 1) & 7): 16 consecutive rows reading the same k cover all banks.
//
// Ring shape for the 256-row tile: 3 A stages (96 KB) + 4 B stages (64 KB) = the whole 160 KB.  Loads come
// back in order, so an A tile (activations, L2 hits) waits behind the B tiles (weights, streamed from
// HBM) issued before it; fetching A two tiles (four steps) ahead and B three steps ahead balances the two
// (about 1 % faster than 2 + 5 stages, which has more bytes of B in flight but A only two steps ahead).
//
// MFMA 32x32x16 operand layout: lane l supplies row (l & 31) of its operand and the 8 consecutive k
// starting at 8 * (l >> 5); it receives column (l & 31) and rows 8*(v/4) + 4*(l >> 5) + v%4 of the
// 32 x 32 result in accumulator element v.
#include <type_traits>

#include "gemm_epilogue.h"

namespace zb {

namespace {

constexpr int KS = 32;   // k per pipeline step
constexpr int BN = 256;
constexpr int NTHREADS = 512;
constexpr int WN = 64;   // wave tile columns
constexpr int LB = BN / 128;  // DMA instructions per wave per B tile

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// s_waitcnt immediate that waits for vmcnt <= n and nothing else (gfx9 encoding)
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// Direct-to-LDS loads.  Every DMA instruction of a wave writes one 1 KB run of the tile (run index
// blk = j * 8 + wave); which 16-byte global chunk a lane fetches implements the LDS swizzle.  The address
// splits into a part that is the same for the whole wave (tile origin, k offset, run) and a per-lane byte
// offset that never changes during the kernel, so the wave-uniform part is scalar arithmetic and the
// lane offset one register per operand (`wave` must be a scalar: readfirstlane'd by the caller).
//
// [32 k][R] tile of a row-contiguous operand (element (k, r) at p[k*ld + r]): run blk holds k-lines
// blk*LPB .. +LPB-1, LPB = 1024 B / (2R B).
template <int R> __device__ __forceinline__ unsigned dma_tr_lane_off(long ld, int wave, int lane) {
  constexpr int CPL = R / 8, LPB = 64 / CPL;  // chunks per k-line, k-lines per run
  const int kl = lane / CPL;
  const int k3 = (wave * LPB + kl) & 3;  // (k & 3): the runs of one wave are 8*LPB (a multiple of 4) lines apart
  const int c = (lane % CPL) ^ (k3 << 2);
  return (unsigned)((kl * ld + c * 8) * (long)sizeof(bf16_t));
}
// p0 = the tile's first element (k0, r0)
template <int R>
__device__ __forceinline__ void dma_tr(const bf16_t* __restrict__ p0, long ld, unsigned lane_off, bf16_t* s, int wave) {
  constexpr int LPB = 64 / (R / 8);
#pragma unroll
  for (int j = 0; j < R / 128; ++j) {
    const int blk = j * 8 + wave;
    const char* base = reinterpret_cast<const char*>(p0 + (long)(blk * LPB) * ld);
    __builtin_amdgcn_global_load_lds((gptr_t)(base + lane_off), (lptr_t)(s + blk * 512), 16, 0, 0);
  }
}
// [R][64 k] tile of a K-contiguous operand (element (r, k) at p[r*ld + k]): run blk holds rows blk*8 .. +7.
__device__ __forceinline__ unsigned dma_rows_lane_off(long ld, int wave, int lane) {
  const int rl = lane >> 3;
  const int c = (lane & 7) ^ ((((wave & 1) << 2) | (lane >> 4)) & 7);  // ((r >> 1) & 7), r = blk*8 + rl
  return (unsigned)((rl * ld + c * 8) * (long)sizeof(bf16_t));
}
template <int R>
__device__ __forceinline__ void dma_rows(const bf16_t* __restrict__ p0, long ld, unsigned lane_off, bf16_t* s, int wave) {
#pragma unroll
  for (int j = 0; j < R / 64; ++j) {
    const int blk = j * 8 + wave;
    const char* base = reinterpret_cast<const char*>(p0 + (long)(blk * 8) * ld);
    __builtin_amdgcn_global_load_lds((gptr_t)(base + lane_off), (lptr_t)(s + blk * 512), 16, 0, 0);
  }
}

// fragment of a [32][R] tile: operand rows rb..rb+31, k = kk*16 .. kk*16+15 (kk = 0, 1)
template <int R> __device__ __forceinline__ bf16x8 frag_tr(const bf16_t* __restrict__ s, int rb, int kk, int lane) {
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
// fragment of a [R][64] tile: rows rb..rb+31, k = kk*16 .. kk*16+15 (kk = 0..3)
__device__ __forceinline__ bf16x8 frag_rows(const bf16_t* __restrict__ s, int rb, int kk, int lane) {
  const int r = rb + (lane & 31);
  const int chunk = kk * 2 + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(s + r * 64 + ((chunk ^ ((r >> 1) & 7)) << 3));
}

// Number of even step indices in [it-BS+2, it-1] for a (large) step index of the given parity: the
// steps whose A refill (K-contiguous A is refilled on even steps only) is younger than B tile `it`.
constexpr int even_steps_in_window(int BS, int parity) {
  int n = 0;
  for (int i = 1000 + parity - BS + 2; i <= 1000 + parity - 1; ++i) n += (i % 2 == 0);
  return n;
}

// AS = LDS stages of a K-contiguous A (64 k each, refilled on even steps AS-1 tiles ahead); a row-contiguous A
// travels with B in the BS-stage ring.
template <int BM, int BS, bool ATR, int AS = 2> struct Cfg {
  static constexpr int A_ELEMS = ATR ? KS * BM : BM * 64;      // per A stage
  static constexpr int A_STAGES = ATR ? BS : AS;
  static constexpr int B_ELEMS = KS * BN;
  static constexpr int LA = ATR ? BM / 128 : BM / 64;           // DMA instructions per wave per A refill
  static constexpr size_t SMEM = ((size_t)A_STAGES * A_ELEMS + (size_t)BS * B_ELEMS) * sizeof(bf16_t);
  // younger loads that may still be in flight when step `it` starts computing
  static constexpr int allowed(int parity) {
    if (ATR) return (BS - 2) * (LA + LB);
    // after B tile `it`: the refills of steps it-BS+2 .. it-1
    const int wrt_b = (BS - 2) * LB + LA * even_steps_in_window(BS, parity);
    if (parity) return wrt_b;               // the A tile of this pair was checked on the even step
    // after A tile it/2 (issued on step it-2(AS-1), before that step's B): the B tiles of steps
    // it-2(AS-1) .. it-1 and the A tiles of the AS-2 even steps between
    const int wrt_a = 2 * (AS - 1) * LB + (AS - 2) * LA;
    return wrt_b < wrt_a ? wrt_b : wrt_a;
  }
};

template <int BM, int BS, int MODE, int AS>
__global__ __launch_bounds__(NTHREADS, (BM == 128 && BS == 3) ? 4 : 2) void gemm_mfma_kernel(const bf16_t* __restrict__ A,
                                                            const bf16_t* __restrict__ B, int M, int N, int K,
                                                            long lda, long ldb, EpiParams epi, int ksplit) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  typedef Cfg<BM, BS, false, AS> C;
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_raw);
  bf16_t* sB = sA + C::A_STAGES * C::A_ELEMS;
  constexpr int WM = BM / 2;
  constexpr int MT = WM / 32, NT = WN / 32;

  // Consecutive workgroup ids go to different XCDs (8, each with its own L2): renumber so that every
  // XCD gets a contiguous run of tiles, M fastest, and tiles that share a weight block share an L2.
  const int tiles_m = M / BM;
  const int nblk = gridDim.x;
  int pid = blockIdx.x;
  if ((nblk & 7) == 0) pid = (pid & 7) * (nblk >> 3) + (pid >> 3);
  if constexpr (MODE == EPI_PARTIAL) {
    // split-K: the K range is cut into ksplit slices of whole 64-k blocks; slice s of every tile writes its
    // fp32 partial product to plane s of the workspace (a fix-up kernel adds the planes in order)
    const int tiles = nblk / ksplit;
    const int slice = pid / tiles;
    pid -= slice * tiles;
    const int blocks64 = K / 64, per = (blocks64 + ksplit - 1) / ksplit;
    const int kb0 = slice * per, kb1 = min(blocks64, kb0 + per);
    A += (long)kb0 * 64;          // K-contiguous A
    B += (long)kb0 * 64 * ldb;    // row-contiguous B
    K = (kb1 - kb0) * 64;
    epi.outf += (size_t)slice * M * N;
  }
  // Tiles are walked in bands of GROUP_M tile rows, M fastest within a band: the 64 or so workgroups that
  // an XCD runs at one time then cover a block of about GROUP_M x 8 tiles and share, through its L2, both
  // the A panels (8 ways) and the B panels (GROUP_M ways) instead of streaming all of A once per column.
  constexpr int GROUP_M = 8;
  const int tiles_n = N / BN;
  const int band = pid / (GROUP_M * tiles_n);
  const int band_rows = min(tiles_m - band * GROUP_M, GROUP_M);
  const int in_band = pid - band * GROUP_M * tiles_n;
  const int m0 = (band * GROUP_M + in_band % band_rows) * BM;
  const int n0 = (in_band / band_rows) * BN;

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = (wave >> 2) * WM, wn = (wave & 3) * WN;
  const unsigned a_off = dma_rows_lane_off(lda, wave, lane), b_off = dma_tr_lane_off<BN>(ldb, wave, lane);
  const bf16_t* a_tile = A + (long)m0 * lda;  // + k
  const bf16_t* b_tile = B + n0;              // + k * ldb

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = K / KS;  // even

  // refills issued by step `it` (also used, with negative it, for the pipeline fill so that the order of
  // loads is the same from the first step on)
  auto issue = [&](int it) {
    if ((it & 1) == 0) {
      const int j = (it >> 1) + AS - 1;  // A tile j covers steps 2j, 2j+1 (negative early in the fill: nothing)
      if (j >= 0 && 2 * j < nk) dma_rows<BM>(a_tile + j * 64, lda, a_off, sA + (j % AS) * C::A_ELEMS, wave);
    }
    const int nt = it + BS - 1;
    if (nt >= 0 && nt < nk)
      dma_tr<BN>(b_tile + (long)(nt * KS) * ldb, ldb, b_off, sB + (nt % BS) * C::B_ELEMS, wave);
  };
  // With one workgroup per CU (BS > 3) the MFMAs of the second half of every tile are issued after the
  // NEXT step's barrier: a wave then reaches the barrier with matrix work still queued, and the matrix
  // pipe stays busy while the waves re-synchronise and the first fragments of the new tile come out of
  // LDS.  With two workgroups per CU the other workgroup fills those gaps and registers are scarce.
  constexpr bool XBAR = BS > 3;
  bf16x8 af1[MT], bf1[NT];  // fragments of the current tile's second half, kept across the barrier
  auto load_frags = [&](int it, int parity, int kk, bf16x8 (&af)[MT], bf16x8 (&bfr)[NT]) {
    const bf16_t* b_s = sB + (it % BS) * C::B_ELEMS;
    const bf16_t* a_s = sA + ((it >> 1) % AS) * C::A_ELEMS;
#pragma unroll
    for (int i = 0; i < MT; ++i) af[i] = frag_rows(a_s, wm + i * 32, parity * 2 + kk, lane);
#pragma unroll
    for (int j = 0; j < NT; ++j) bfr[j] = frag_tr<BN>(b_s, wn + j * 32, kk, lane);
  };
  auto mfmas = [&](const bf16x8 (&af)[MT], const bf16x8 (&bfr)[NT]) {
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
  };
  auto step = [&](int it, auto parity_tag) {
    constexpr int parity = decltype(parity_tag)::value;
    // near the end fewer loads were issued than the constant assumes: wait for everything
    constexpr int AHEAD = (BS - 2) > (2 * AS - 3) ? (BS - 2) : (2 * AS - 3);  // last step whose refills all exist
    if (it + AHEAD < nk) __builtin_amdgcn_s_waitcnt(vmcnt_imm(C::allowed(parity)));
    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __builtin_amdgcn_s_barrier();
    // The refill of the stage that step it-1 used may be issued any time after the barrier; with the deep
    // ring it goes after the fragment reads so that the matrix pipe gets its work first.
    if constexpr (!XBAR) issue(it);  // shallow ring, two workgroups per CU: refill at once
    bf16x8 af0[MT], bf0[NT];
    load_frags(it, parity, 0, af0, bf0);
    if constexpr (XBAR) {
      if (it > 0) mfmas(af1, bf1);  // second half of tile it-1
      mfmas(af0, bf0);
      load_frags(it, parity, 1, af1, bf1);
      issue(it);
      // these LDS reads must have completed before the next barrier lets another wave refill the stage
      __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0) only
    } else {
      mfmas(af0, bf0);
      load_frags(it, parity, 1, af1, bf1);
      mfmas(af1, bf1);
    }
  };

  // pipeline fill: the same sequence of refills as in the loop, from the first step that issues anything
  constexpr int FILL0 = (1 - BS) < -2 * (AS - 1) ? (1 - BS) : -2 * (AS - 1);
#pragma unroll
  for (int it = FILL0; it < 0; ++it) issue(it);
  for (int it = 0; it < nk; it += 2) {
    step(it, std::integral_constant<int, 0>());
    step(it + 1, std::integral_constant<int, 1>());
  }
  if constexpr (XBAR) mfmas(af1, bf1);

  const int lrow = lane & 31, lhi = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      epilogue_tile<bf16_t, MODE>(epi, m0 + wm + i * 32 + lhi, n0 + wn + j * 32 + lrow, acc[i][j]);
    }
}

// ldo: row stride of the outputs when the GEMM covers a column range of a wider matrix (0: g.N)
template <int BM, int BS, int MODE, int AS = 2>
hipError_t run_cfg(const GemmArgs& g, long lda, long ldb, hipStream_t s, int ksplit = 1, int ldo = 0) {
  auto kern = gemm_mfma_kernel<BM, BS, MODE, AS>;
  constexpr size_t smem = Cfg<BM, BS, false, AS>::SMEM;
  static_assert(smem <= 160 * 1024, "LDS budget");
  static bool attr_set = false;  // one device per process in this library
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int grid = (g.M / BM) * (g.N / BN) * ksplit;
  EpiParams epi = make_epi(g);
  if (ldo) epi.N = ldo;
  kern<<<grid, NTHREADS, smem, s>>>((const bf16_t*)g.A, (const bf16_t*)g.B, g.M, g.N, g.K, lda, ldb, epi, ksplit);
  return hipGetLastError();
}

// Split-K fix-up: out = epilogue(sum of the K-slice planes, added in slice order), 4 columns per thread.
// The planes are [M, N] dense; the outputs (and aux) have row stride epi.N >= N.
template <int MODE>
__global__ __launch_bounds__(256) void gemm_splitk_fixup_kernel(const float* __restrict__ ws, int slices, size_t plane,
                                                                int N, EpiParams epi) {
  const size_t p4 = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (p4 >= plane) return;
  f32x4 acc = *reinterpret_cast<const f32x4*>(ws + p4);
  for (int sl = 1; sl < slices; ++sl) acc += *reinterpret_cast<const f32x4*>(ws + (size_t)sl * plane + p4);
  const int n = (int)(p4 % (size_t)N);
  const size_t i4 = (p4 / (size_t)N) * (size_t)epi.N + n;
  bf16x4 o0, o1;
  if (MODE == EPI_STORE) {
#pragma unroll
    for (int e = 0; e < 4; ++e) o0[e] = (bf16_t)acc[e];
  } else if (MODE == EPI_DGELU) {
    const bf16x4 a = *reinterpret_cast<const bf16x4*>((const bf16_t*)epi.aux + i4);
#pragma unroll
    for (int e = 0; e < 4; ++e) o0[e] = (bf16_t)(acc[e] * gelu_grad_f((float)a[e]));
  } else {
    const f32x4 b = *reinterpret_cast<const f32x4*>(epi.bias + n);
    if (MODE == EPI_BIAS_RESID) {
      const bf16x4 a = *reinterpret_cast<const bf16x4*>((const bf16_t*)epi.aux + i4);
#pragma unroll
      for (int e = 0; e < 4; ++e) o0[e] = (bf16_t)(acc[e] + b[e] + (float)a[e]);
    } else if (MODE == EPI_BIAS_GELU) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float f = acc[e] + b[e];
        o0[e] = (bf16_t)f;
        o1[e] = (bf16_t)gelu_f(f);
      }
      *reinterpret_cast<bf16x4*>((bf16_t*)epi.out1 + i4) = o1;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) o0[e] = (bf16_t)(acc[e] + b[e]);
    }
  }
  *reinterpret_cast<bf16x4*>((bf16_t*)epi.out0 + i4) = o0;
}

// wgrad: C += A_0^T B_0 + A_1^T B_1 + ... for `ngroup` >= 1 operand pairs of one shape (the W passes of one
// or of several consecutive microbatches), both operands row-contiguous ([k][m], [k][n]).  The accumulators
// START from the old C (requested before anything else, so the read travels while the ring of LDS stages
// fills) and every MFMA adds into them, pair after pair, in k order; the new C is written once at the end
// and nothing is read back there.  An element's value is therefore the same chain of fp32 MFMA additions
// whatever the tile shape, ring depth or grouping: `ngroup` pairs in one launch give exactly the bits of
// `ngroup` launches of one pair.  The ring runs on across the pairs without draining.
// One launch covers up to kWgradMaxProblems gradients (the weight matrices of one W pass: tiles of equal
// duration, so the partly filled last round of workgroups is paid once per pass instead of once per
// matrix) with `ngroup` operand pairs each.
struct WgradTable {
  int nprob, ngroup;
  int tile0[kWgradMaxProblems + 1];  // first tile of each problem in the launch
  int M[kWgradMaxProblems], N[kWgradMaxProblems];
  float* outf[kWgradMaxProblems];
  const bf16_t* a[kWgradMaxPairs];   // pair g of problem q at [q * ngroup + g]
  const bf16_t* b[kWgradMaxPairs];
  int ntiles;                        // workgroups [0, ntiles) are GEMM tiles, the rest column-sum strips
  int strip0[kWgradMaxProblems + 1]; // first strip (256 columns) of each problem; equal entries: no bias
  float* bias[kWgradMaxProblems];
};

// Bias gradient of one 256-column strip of one problem: bias[n] += sum over the Kc rows of every operand pair's
// b (the output gradient), pair by pair.  512 threads = 32 chunks of 8 columns x 16 row groups; a thread adds
// its rows in ascending order, the 16 row groups are added in ascending order, then the pair's sum goes onto
// the running value: the same chain of additions whether the pairs come in one launch or one launch each.
__device__ __forceinline__ void wgrad_bias_strip(const WgradTable& tb, int sid, int Kc, float* red) {
  int q = 0;
#pragma unroll
  for (int i = 1; i < kWgradMaxProblems; ++i) q += (i < tb.nprob && sid >= tb.strip0[i]) ? 1 : 0;
  sid -= tb.strip0[q];
  const int N = tb.N[q], ngroup = tb.ngroup;
  const int n0 = sid * BN;
  const int c = threadIdx.x & 31, g = threadIdx.x >> 5;
  float* __restrict__ bias = tb.bias[q];
  float run = 0.f;
  if (threadIdx.x < BN) run = bias[n0 + threadIdx.x];
  for (int gi = 0; gi < ngroup; ++gi) {
    const bf16_t* __restrict__ b = tb.b[q * ngroup + gi] + n0 + c * 8;
    float sum[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) sum[j] = 0.f;
#pragma unroll 8
    for (int r = g; r < Kc; r += 16) {
      const bf16x8 v = *reinterpret_cast<const bf16x8*>(b + (long)r * N);
#pragma unroll
      for (int j = 0; j < 8; ++j) sum[j] += (float)v[j];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) red[g * BN + c * 8 + j] = sum[j];
    __syncthreads();
    if (threadIdx.x < BN) {
      float t = 0.f;
#pragma unroll
      for (int gg = 0; gg < 16; ++gg) t += red[gg * BN + threadIdx.x];
      run += t;
    }
    __syncthreads();
  }
  if (threadIdx.x < BN) bias[n0 + threadIdx.x] = run;
}

template <int BM, int BS, bool XB>
__global__ __launch_bounds__(512, (BM == 128 && BS == 3) ? 4 : 2) void gemm_wgrad_kernel(WgradTable tb, int Kc) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  typedef Cfg<BM, BS, true> C;
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_raw);
  bf16_t* sB = sA + C::A_STAGES * C::A_ELEMS;
  constexpr int WM = BM / 2;
  constexpr int MT = WM / 32, NT = WN / 32;

  const int nblk = tb.ntiles;
  int pid = blockIdx.x;
  if (pid >= nblk) {  // the launch's last workgroups: bias gradients (they fill the CUs the last round of tiles leaves idle)
    wgrad_bias_strip(tb, pid - nblk, Kc, reinterpret_cast<float*>(smem_raw));
    return;
  }
  if ((nblk & 7) == 0) pid = (pid & 7) * (nblk >> 3) + (pid >> 3);
  int q = 0;  // which problem this tile belongs to
#pragma unroll
  for (int i = 1; i < kWgradMaxProblems; ++i) q += (i < tb.nprob && pid >= tb.tile0[i]) ? 1 : 0;
  pid -= tb.tile0[q];
  const int M = tb.M[q], N = tb.N[q], ngroup = tb.ngroup;
  const long lda = M, ldb = N;
  float* __restrict__ outf = tb.outf[q];
  const int pair0 = q * ngroup;
  const int tiles_m = M / BM, tiles_n = N / BN;
  // Bands of 4 tile rows: an XCD runs 32 of these tiles at a time (one per CU), a block of 4 x 8.  Its four
  // A panels (K x 256 bf16, 512 KB each at K = 1024) then stay in the 4 MB L2 for the whole walk along the
  // band while B panels and the gradient tiles (non-temporal) stream past; at 8 rows the A panels alone fill
  // the L2 and are fetched again for every block (measured on the 14.6B stage: 785 -> 841 TFLOP/s; 2 rows
  // the same as 4, 1 row 818).
  constexpr int GROUP_M = 4;
  const int band = pid / (GROUP_M * tiles_n);
  const int band_rows = min(tiles_m - band * GROUP_M, GROUP_M);
  const int in_band = pid - band * GROUP_M * tiles_n;
  const int m0 = (band * GROUP_M + in_band % band_rows) * BM;
  const int n0 = (in_band / band_rows) * BN;

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = (wave >> 2) * WM, wn = (wave & 3) * WN;
  const int lrow = lane & 31, lhi = (lane >> 5) * 4;
  const unsigned a_off = dma_tr_lane_off<BM>(lda, wave, lane), b_off = dma_tr_lane_off<BN>(ldb, wave, lane);

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const float* p0 = outf + (size_t)(m0 + wm + i * 32 + lhi) * N + n0 + wn + j * 32 + lrow;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = __builtin_nontemporal_load(p0 + (size_t)((v >> 2) * 8 + (v & 3)) * N);
      __builtin_amdgcn_sched_barrier(0);  // one tile's addresses at a time
    }

  const int spc = Kc / KS;        // steps per operand pair
  const int nk = ngroup * spc;
  int g_next = 0, k_next = 0;  // operand pair and k offset of the next tile to fetch (tiles are fetched in order)
  auto issue = [&](int it) {
    const int nt = it + BS - 1;
    if (nt < nk) {
      dma_tr<BM>(tb.a[pair0 + g_next] + (long)k_next * lda + m0, lda, a_off, sA + (nt % BS) * C::A_ELEMS, wave);
      dma_tr<BN>(tb.b[pair0 + g_next] + (long)k_next * ldb + n0, ldb, b_off, sB + (nt % BS) * C::B_ELEMS, wave);
      k_next += KS;
      if (k_next == Kc) { k_next = 0; ++g_next; }
    }
  };
  bf16x8 af1[MT], bf1[NT];  // XB: fragments of a tile's second half, carried across the next barrier
  auto load_frags = [&](int it, int kk, bf16x8 (&af)[MT], bf16x8 (&bfr)[NT]) {
    const bf16_t* a_s = sA + (it % BS) * C::A_ELEMS;
    const bf16_t* b_s = sB + (it % BS) * C::B_ELEMS;
#pragma unroll
    for (int i = 0; i < MT; ++i) af[i] = frag_tr<BM>(a_s, wm + i * 32, kk, lane);
#pragma unroll
    for (int j = 0; j < NT; ++j) bfr[j] = frag_tr<BN>(b_s, wn + j * 32, kk, lane);
  };
  auto mfmas = [&](const bf16x8 (&af)[MT], const bf16x8 (&bfr)[NT]) {
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
  };

#pragma unroll
  for (int it = 1 - BS; it < 0; ++it) issue(it);
  for (int it = 0; it < nk; ++it) {
    if (it + BS - 2 < nk) __builtin_amdgcn_s_waitcnt(vmcnt_imm(C::allowed(0)));
    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __builtin_amdgcn_s_barrier();
    bf16x8 af0[MT], bf0[NT];
    if constexpr (XB) {
      // the MFMAs of a step's second half are issued after the next step's barrier (one workgroup per CU:
      // the matrix pipe keeps work queued while the waves re-synchronise)
      load_frags(it, 0, af0, bf0);
      if (it > 0) mfmas(af1, bf1);
      mfmas(af0, bf0);
      load_frags(it, 1, af1, bf1);
      issue(it);
      __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): fragment reads done before the next barrier
    } else {
      issue(it);
      load_frags(it, 0, af0, bf0);
      mfmas(af0, bf0);
      load_frags(it, 1, af1, bf1);
      mfmas(af1, bf1);
    }
  }
  if constexpr (XB) mfmas(af1, bf1);

  // the store addresses are worked out again here (from a copy of the tile origin the compiler cannot
  // connect with the one used for the loads), or the address pairs would stay in registers across the loop
  int m0s = m0, n0s = n0;
  asm volatile("" : "+s"(m0s), "+s"(n0s));
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      float* p0 = outf + (size_t)(m0s + wm + i * 32 + lhi) * N + n0s + wn + j * 32 + lrow;
#pragma unroll
      for (int v = 0; v < 16; ++v) __builtin_nontemporal_store(acc[i][j][v], p0 + (size_t)((v >> 2) * 8 + (v & 3)) * N);
      __builtin_amdgcn_sched_barrier(0);
    }
}

// Few tiles and a long K (the N = hidden GEMMs of a 1024-token microbatch): cut K into slices so that
// every CU gets a workgroup.  Returns false if the shape is not one for split-K.
template <int MODE>
bool try_split_k(const GemmArgs& g, long lda, long ldb, hipStream_t s, hipError_t* err) {
  if (g.M % 256 != 0 || g.N % BN != 0 || g.N % 4 != 0 || g.K < 2048 || !g.workspace) return false;
  const long tiles = (long)(g.M / 256) * (g.N / BN);
  if (tiles > 128) return false;
  int slices = (int)(256 / tiles);
  if (slices > 4) slices = 4;
  const size_t plane = (size_t)g.M * g.N;
  if (slices < 2 || (size_t)slices * plane > g.workspace_floats) return false;
  GemmArgs p = g;
  p.epilogue = EPI_PARTIAL;
  p.outf = g.workspace;
  *err = run_cfg<256, 4, EPI_PARTIAL, 3>(p, lda, ldb, s, slices);
  if (*err != hipSuccess) return true;
  // The last step owns whole rows: a LayerNorm on those rows rides along instead of running as a kernel of
  // its own on the stored result.
  const bool ln_shape = g.ln_done && g.N <= 8192;
  if (MODE == EPI_BIAS_RESID && g.ln_mode == 1 && ln_shape) {
    *err = launch_splitk_layernorm_fwd<bf16_t>(g.workspace, slices, plane, g.bias, (const bf16_t*)g.aux,
                                               (bf16_t*)g.out0, g.ln_gamma, g.ln_beta, (bf16_t*)g.ln_out, g.ln_stats,
                                               g.M, g.N, g.ln_eps, s);
    *g.ln_done = *err == hipSuccess;
    return true;
  }
  if (MODE == EPI_STORE && g.ln_mode == 2 && ln_shape) {
    *err = launch_splitk_layernorm_bwd<bf16_t>(g.workspace, slices, plane, (bf16_t*)g.out0, (const bf16_t*)g.ln_x, g.ln_stats,
                                               g.ln_gamma, (const bf16_t*)g.ln_resid, (bf16_t*)g.ln_out, g.ln_dgamma,
                                               g.ln_dbeta, g.ln_partials, g.M, g.N, s);
    *g.ln_done = *err == hipSuccess;
    return true;
  }
  const size_t threads = plane / 4;
  gemm_splitk_fixup_kernel<MODE><<<(unsigned)((threads + 255) / 256), 256, 0, s>>>(g.workspace, slices, plane, g.N,
                                                                                 make_epi(g));
  *err = hipGetLastError();
  return true;
}

// A little more than a whole number of rounds of 256 x 256 tiles over the 256 CUs (N = ffn with 1024
// tokens: 320 tiles): the full rounds run as they are and the tile columns left over are cut along K so
// that they, too, fill every CU once instead of occupying a quarter of the chip for a whole round.
template <int MODE>
bool try_tail_split(const GemmArgs& g, long lda, long ldb, hipStream_t s, hipError_t* err) {
  if (g.M % 256 != 0 || g.N % BN != 0 || g.K < 2048 || !g.workspace) return false;
  const int tm = g.M / 256, tn = g.N / BN;
  if ((long)tm * tn <= 256 || tm > 256 || 256 % tm != 0) return false;
  const int cols_per_round = 256 / tm;
  const int tail_cols = tn % cols_per_round;
  if (tail_cols == 0 || tail_cols * tm > 128) return false;
  int slices = 256 / (tail_cols * tm);
  if (slices > 4) slices = 4;
  const int n_main = (tn - tail_cols) * BN, n_tail = tail_cols * BN;
  const size_t plane = (size_t)g.M * n_tail;
  if ((size_t)slices * plane > g.workspace_floats) return false;
  GemmArgs a = g;
  a.N = n_main;
  *err = run_cfg<256, 4, MODE, 3>(a, lda, ldb, s, 1, g.N);
  if (*err != hipSuccess) return true;
  GemmArgs t = g;  // the same GEMM on columns n_main .. N-1
  t.N = n_tail;
  t.B = (const bf16_t*)g.B + n_main;
  if (t.out0) t.out0 = (bf16_t*)g.out0 + n_main;
  if (t.out1) t.out1 = (bf16_t*)g.out1 + n_main;
  if (t.aux) t.aux = (const bf16_t*)g.aux + n_main;
  if (t.bias) t.bias = g.bias + n_main;
  GemmArgs p = t;
  p.epilogue = EPI_PARTIAL;
  p.outf = g.workspace;
  *err = run_cfg<256, 4, EPI_PARTIAL, 3>(p, lda, ldb, s, slices);
  if (*err != hipSuccess) return true;
  EpiParams epi = make_epi(t);
  epi.N = g.N;
  const size_t threads = plane / 4;
  gemm_splitk_fixup_kernel<MODE><<<(unsigned)((threads + 255) / 256), 256, 0, s>>>(g.workspace, slices, plane, n_tail,
                                                                                 epi);
  *err = hipGetLastError();
  return true;
}

template <int MODE>
hipError_t run_shape(const GemmArgs& g, long lda, long ldb, hipStream_t s, bool* taken) {
  *taken = true;
  hipError_t e = hipSuccess;
  if (try_split_k<MODE>(g, lda, ldb, s, &e)) return e;
  if (try_tail_split<MODE>(g, lda, ldb, s, &e)) return e;
  if (g.N % BN == 0) {
    // Rounds of tiles over the 256 CUs times the tile height; the taller tile does about 1.25x the
    // work per cycle, so it wins only when it does not cost an extra, mostly empty round.
    const long t256 = g.M % 256 == 0 ? (long)(g.M / 256) * (g.N / BN) : 0;
    const long t128 = g.M % 128 == 0 ? (long)(g.M / 128) * (g.N / BN) : 0;
    const double c256 = t256 ? (double)((t256 + 255) / 256) * 256.0 / 1.25 : 1e30;
    const double c128 = t128 ? (double)((t128 + 255) / 256) * 128.0 : 1e30;
    if (t256 && c256 <= c128) return run_cfg<256, 4, MODE, 3>(g, lda, ldb, s);
    if (t128) {
      // more tiles than CUs: a three-stage ring (<= 80 KB) lets two workgroups share a CU, so one's
      // epilogue and pipeline fill hide behind the other's MFMAs; otherwise one workgroup per CU with a
      // deeper ring
      if (t128 > 256) return run_cfg<128, 3, MODE>(g, lda, ldb, s);
      return run_cfg<128, 5, MODE>(g, lda, ldb, s);
    }
  }
  *taken = false;
  return hipSuccess;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <int BM, int BS, bool XB>
hipError_t run_wgrad(WgradTable& tb, int K, hipStream_t s) {
  auto kern = gemm_wgrad_kernel<BM, BS, XB>;
  constexpr size_t smem = Cfg<BM, BS, true>::SMEM;
  static_assert(smem <= 160 * 1024, "LDS budget");
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  int tiles = 0;
  for (int q = 0; q < tb.nprob; ++q) {
    tb.tile0[q] = tiles;
    tiles += (tb.M[q] / BM) * (tb.N[q] / BN);
  }
  for (int q = tb.nprob; q <= kWgradMaxProblems; ++q) tb.tile0[q] = tiles;
  tb.ntiles = tiles;
  int strips = 0;
  for (int q = 0; q < tb.nprob; ++q) {
    tb.strip0[q] = strips;
    if (tb.bias[q]) strips += tb.N[q] / BN;
  }
  for (int q = tb.nprob; q <= kWgradMaxProblems; ++q) tb.strip0[q] = strips;
  static_assert(smem >= 16 * BN * sizeof(float), "the strips' reduction buffer");
  kern<<<tiles + strips, NTHREADS, smem, s>>>(tb, K);
  return hipGetLastError();
}

}  // namespace

template <typename T> hipError_t launch_gemm_mfma(const GemmArgs& g, hipStream_t s, bool* taken) {
  *taken = false;
  return hipSuccess;
}

// wgrad launch for the gradients of one W pass; *taken stays false if a shape is not one for the MFMA kernel
template <typename T> hipError_t launch_wgrad_multi_mfma(const WgradMultiArgs& w, hipStream_t s, bool* taken) {
  *taken = false;
  return hipSuccess;
}
template <> hipError_t launch_wgrad_multi_mfma<bf16_t>(const WgradMultiArgs& w, hipStream_t s, bool* taken) {
  *taken = false;
  if (w.nprob < 1 || w.nprob > kWgradMaxProblems || w.ngroup < 1 || w.ngroup > kGemmGroupMax ||
      w.nprob * w.ngroup > kWgradMaxPairs || w.K <= 0 || w.K % 64 != 0)
    return hipSuccess;
  WgradTable tb{};
  tb.nprob = w.nprob;
  tb.ngroup = w.ngroup;
  bool all256 = true;
  long t256 = 0, t128 = 0;
  for (int q = 0; q < w.nprob; ++q) {
    const int M = w.M[q], N = w.N[q];
    if (M <= 0 || N <= 0 || M % 128 != 0 || N % BN != 0 || !aligned16(w.outf[q])) return hipSuccess;
    tb.M[q] = M; tb.N[q] = N; tb.outf[q] = w.outf[q];
    tb.bias[q] = w.bias_done ? w.bias[q] : nullptr;
    all256 = all256 && M % 256 == 0;
    t256 += (long)(M / 256) * (N / BN);
    t128 += (long)(M / 128) * (N / BN);
    for (int g = 0; g < w.ngroup; ++g) {
      const void* a = w.a[q * w.ngroup + g];
      const void* b = w.b[q * w.ngroup + g];
      if (!a || !b || !aligned16(a) || !aligned16(b)) return hipSuccess;
      tb.a[q * w.ngroup + g] = (const bf16_t*)a;
      tb.b[q * w.ngroup + g] = (const bf16_t*)b;
    }
  }
  if (t128 >= (1L << 30)) return hipSuccess;
  *taken = true;
  if (w.bias_done) *w.bias_done = true;
  // 256-row tiles (one workgroup per CU, four-stage ring) when they fill most of the chip; else 128-row
  // tiles, two workgroups per CU with a three-stage ring if there are more tiles than CUs, one with a
  // five-stage ring otherwise.  The choice does not change the result (see the kernel).
  if (all256 && t256 >= 192) return run_wgrad<256, 4, true>(tb, w.K, s);
  if (t128 > 256) return run_wgrad<128, 3, true>(tb, w.K, s);
  return run_wgrad<128, 5, true>(tb, w.K, s);
}
template hipError_t launch_wgrad_multi_mfma<float>(const WgradMultiArgs&, hipStream_t, bool*);

namespace {

// one accumulate GEMM (one pair, or g.group pairs) through the same kernel
hipError_t launch_wgrad(const GemmArgs& g, hipStream_t s, bool* taken) {
  const int ngroup = g.group >= 2 ? g.group : 1;
  if (g.epilogue != EPI_ACCUM_F32 || ngroup > kGemmGroupMax) return hipSuccess;
  if (!(g.a_sm == 1 && g.b_sn == 1) || g.a_sk != g.M || g.b_sk != g.N) return hipSuccess;
  WgradMultiArgs w{};
  w.nprob = 1; w.ngroup = ngroup; w.K = g.K;
  w.M[0] = g.M; w.N[0] = g.N; w.outf[0] = g.outf;
  for (int i = 0; i < ngroup; ++i) {
    w.a[i] = g.group >= 2 ? g.group_a[i] : g.A;
    w.b[i] = g.group >= 2 ? g.group_b[i] : g.B;
  }
  return launch_wgrad_multi_mfma<bf16_t>(w, s, taken);
}

}  // namespace

template <> hipError_t launch_gemm_mfma<bf16_t>(const GemmArgs& g, hipStream_t s, bool* taken) {
  *taken = false;
  if (g.epilogue == EPI_ACCUM_F32) return launch_wgrad(g, s, taken);
  // forward X[M,K] * W[K,N]; dgrad dY[M,K'] * Wt[K',N']: A K-contiguous, B row-contiguous
  if (g.a_sk != 1 || !(g.b_sn == 1 && g.b_sk != 1)) return hipSuccess;
  const long lda = g.a_sm, ldb = g.b_sk;
  if (g.K % 64 != 0 || lda % 8 != 0 || ldb % 8 != 0 || !aligned16(g.A) || !aligned16(g.B)) return hipSuccess;
  if (g.epilogue == EPI_BIAS) return run_shape<EPI_BIAS>(g, lda, ldb, s, taken);
  if (g.epilogue == EPI_BIAS_RESID) return run_shape<EPI_BIAS_RESID>(g, lda, ldb, s, taken);
  if (g.epilogue == EPI_BIAS_GELU) return run_shape<EPI_BIAS_GELU>(g, lda, ldb, s, taken);
  if (g.epilogue == EPI_STORE) return run_shape<EPI_STORE>(g, lda, ldb, s, taken);
  if (g.epilogue == EPI_DGELU) return run_shape<EPI_DGELU>(g, lda, ldb, s, taken);
  return hipSuccess;
}

template hipError_t launch_gemm_mfma<float>(const GemmArgs&, hipStream_t, bool*);

}  // namespace zb
