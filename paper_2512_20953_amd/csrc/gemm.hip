// bf16 GEMM for gfx950: MFMA 32x32x16, fp32 accumulators, tiles staged through
// LDS by direct global->LDS loads (16 B per lane), double buffered.
//
// Three operand layouts cover the linear layers of a decoder layer (the GEMM is
// the core of the stage's time, paper Section II-B):
//   NN  y  = x W        (forward)            A[M,K] k-contiguous, B[K,N] k-strided
//   NT  dx = dy W^T     (input gradient)     A[M,K], B[N,K] both k-contiguous
//   TN  dW += x^T dy    (weight gradient)    A[K,M], B[K,N] both k-strided
// A k-contiguous operand is read from LDS with 16-byte reads; a k-strided one
// with the transposing 8-byte LDS read, so no transposed copy is ever made.
//
// Work split: 256 threads = 4 waves in a 2 x 2 grid; each wave owns a
// (BM/2) x (BN/2) sub-tile as 32 x 32 MFMA blocks.  The MFMA is issued with the
// operands swapped (D = B^T A^T) so that a lane ends up with 4 consecutive
// columns of one output row: 8-byte bf16 or 16-byte fp32 accesses in the epilogue.
#include "common.h"
#include "kernels.h"
#include <cstdlib>

namespace ah {

constexpr int BK = 64;  // k-extent of one LDS stage (128 bytes of bf16)

// ---------------------------------------------------------------------------
// LDS layouts (all permutations are of 16-byte pieces, the unit of the loader)
//  k-contiguous tile: [rows][64 k]; row = 128 B = 8 pieces; piece p of row r is
//    stored at piece p ^ ((r >> 1) & 7): 16 consecutive rows hit 16 distinct
//    bank groups for the 16-byte fragment reads.
//  k-strided tile: [64 k][W cols]; row = 2W bytes; the 64-byte granule g of row
//    k is stored at granule g ^ (k & 3): the 4 rows x 64 B that half a wave
//    fetches in one transposing read cover all banks once.
// ---------------------------------------------------------------------------
template <int W, bool KS>
__device__ __forceinline__ uint32_t loader_src_offset(int chunk, int lane, int ld) {
  const int pos = chunk * 1024 + lane * 16;
  if (!KS) {
    const int r = pos >> 7, q = (pos >> 4) & 7;
    const int p = q ^ ((r >> 1) & 7);
    return (uint32_t)(r * ld + p * 8);
  } else {
    constexpr int RB = W * 2;
    const int k = pos / RB, q = (pos % RB) >> 4;
    const int p = q ^ ((k & 3) << 2);
    return (uint32_t)(k * ld + p * 8);
  }
}

template <int W, bool KS, int NW>
__device__ __forceinline__ void issue_tile_loads(const bf16* __restrict__ g, const uint32_t* off, char* __restrict__ lds, int wave) {
#pragma unroll
  for (int i = 0; i < W / 8 / NW; i++) load16_to_lds(g + off[i], lds + (wave + NW * i) * 1024);
}

// fragment (8 k-values for row/col = lane % 32 of a 32-wide block) for k-step ks
template <int W, bool KS>
__device__ __forceinline__ bf16x8 read_frag(const char* __restrict__ lds, int base, int blk, int ks, int lane) {
  if (!KS) {
    const int r = base + blk * 32 + (lane & 31);
    const int p = ks * 2 + (lane >> 5);
    const int q = p ^ ((r >> 1) & 7);
    return *(const bf16x8*)(lds + r * 128 + q * 16);
  } else {
    constexpr int RB = W * 2;
    const int k = ks * 16 + (lane >> 5) * 8 + ((lane & 15) >> 2);
    const int c = base + blk * 32 + ((lane >> 4) & 1) * 16 + 4 * (lane & 3);
    const int a0 = k * RB + ((((c >> 5) ^ (k & 3))) << 6) + ((c * 2) & 63);
    bf16x4 lo = lds_read_tr4(lds + a0);
    bf16x4 hi = lds_read_tr4(lds + a0 + 4 * RB);
    return cat4(lo, hi);
  }
}

// Fragments of one 16-wide k-step for the wave's sub-tile.
template <int BM, int BN, int WGM, int WGN, bool AKS, bool BKS>
struct Frags {
  static constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
  bf16x8 a[TM], b[TN];
  __device__ __forceinline__ void load(const char* __restrict__ cA, const char* __restrict__ cB, int ks, int wm, int wn, int lane) {
#pragma unroll
    for (int t = 0; t < TM; t++) a[t] = read_frag<BM, AKS>(cA, wm * (BM / WGM), t, ks, lane);
#pragma unroll
    for (int t = 0; t < TN; t++) b[t] = read_frag<BN, BKS>(cB, wn * (BN / WGN), t, ks, lane);
  }
};

// Scheduling hint: spread the NR LDS reads issued for the next k-step between the
// NM MFMAs of the current one (masks: 0x100 = LDS read, 0x008 = MFMA).
template <int NR, int NM>
__device__ __forceinline__ void interleave_reads_with_mfma() {
  if constexpr (NR >= NM) {
#pragma unroll
    for (int i = 0; i < NM; i++) {
      __builtin_amdgcn_sched_group_barrier(0x100, NR / NM, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
  } else {
#pragma unroll
    for (int i = 0; i < NR; i++) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, NM / NR, 0);
    }
  }
}

template <int BM, int BN, int WGM, int WGN, bool AKS, bool BKS>
__device__ __forceinline__ void mma_step(const Frags<BM, BN, WGM, WGN, AKS, BKS>& f, f32x16 (&acc)[BM / WGM / 32][BN / WGN / 32]) {
  constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
#pragma unroll
  for (int tm = 0; tm < TM; tm++)
#pragma unroll
    for (int tn = 0; tn < TN; tn++)
      acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[tn], f.a[tm], acc[tm][tn], 0, 0, 0);
}

// One k-tile of the pipeline.  On entry f0 holds the fragments of k-step 0 of
// (cA, cB).  Starts the loads of the next k-tile into (nA, nB), multiplies the
// current one while the fragments of each following k-step are fetched, and
// before the last k-step waits for the next tile (its own loads, then the
// block barrier) so that f0 can be refilled from (nA, nB) under the last MFMAs.
// The restrict qualifiers tell the compiler that LDS reads of (cA, cB) never
// touch the buffers being filled.
template <int BM, int BN, int WGM, int WGN, bool AKS, bool BKS>
__device__ __forceinline__ void pipe_step(bool prefetch, int dbg, const bf16* gA, const bf16* gB, const uint32_t* offA, const uint32_t* offB,
                                          char* __restrict__ nA, char* __restrict__ nB, const char* __restrict__ cA,
                                          const char* __restrict__ cB, Frags<BM, BN, WGM, WGN, AKS, BKS>& f0,
                                          Frags<BM, BN, WGM, WGN, AKS, BKS>& f1, f32x16 (&acc)[BM / WGM / 32][BN / WGN / 32],
                                          int wave, int wm, int wn, int lane) {
  constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
  constexpr int NR = TM * (AKS ? 2 : 1) + TN * (BKS ? 2 : 1), NM = TM * TN;
  if (prefetch) {
    issue_tile_loads<BM, AKS, WGM * WGN>(gA, offA, nA, wave);
    issue_tile_loads<BN, BKS, WGM * WGN>(gB, offB, nB, wave);
  }
  if (dbg < 3) f1.load(cA, cB, 1, wm, wn, lane);
  mma_step<BM, BN, WGM, WGN, AKS, BKS>(f0, acc);
  interleave_reads_with_mfma<NR, NM>();
  if (dbg < 3) f0.load(cA, cB, 2, wm, wn, lane);
  mma_step<BM, BN, WGM, WGN, AKS, BKS>(f1, acc);
  interleave_reads_with_mfma<NR, NM>();
  if (dbg < 3) f1.load(cA, cB, 3, wm, wn, lane);
  mma_step<BM, BN, WGM, WGN, AKS, BKS>(f0, acc);
  interleave_reads_with_mfma<NR, NM>();
  if (dbg < 2) {
    __builtin_amdgcn_s_waitcnt(0);  // own loads of the next tile have landed, own reads of this one are done
    __syncthreads();
  }
  if (dbg < 3) f0.load(nA, nB, 0, wm, wn, lane);
  mma_step<BM, BN, WGM, WGN, AKS, BKS>(f1, acc);
  interleave_reads_with_mfma<NR, NM>();
}

template <int BM, int BN, int WGM, int WGN, bool AKS, bool BKS, int EPI>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(GemmArgs g) {
  constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32, NW = WGM * WGN;
  __shared__ __attribute__((aligned(1024))) char sA0[BM * 128];
  __shared__ __attribute__((aligned(1024))) char sA1[BM * 128];
  __shared__ __attribute__((aligned(1024))) char sB0[BN * 128];
  __shared__ __attribute__((aligned(1024))) char sB1[BN * 128];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps LDS bases in scalar registers
  const int wm = wave / WGN, wn = wave % WGN;

  // block -> tile: consecutive logical tiles share an XCD (blocks are dealt to the
  // 8 XCDs round-robin), and run down groups of 8 tile-rows so that the tiles in
  // flight on one XCD reuse the same operand panels in its L2.
  const int tiles_m = g.M / BM, tiles_n = g.N / BN, ntiles = tiles_m * tiles_n;
  int logical = blockIdx.x;
  if ((ntiles & 7) == 0) logical = (blockIdx.x & 7) * (ntiles >> 3) + (blockIdx.x >> 3);
  constexpr int GROUP = 8;
  const int per_group = GROUP * tiles_n;
  const int gid = logical / per_group;
  const int first_m = gid * GROUP;
  const int gsize = min(tiles_m - first_m, GROUP);
  const int in_group = logical - gid * per_group;
  const int m0 = (first_m + in_group % gsize) * BM;
  const int n0 = (in_group / gsize) * BN;

  const bf16* gA = (const bf16*)g.A + (AKS ? (size_t)m0 : (size_t)m0 * g.lda);
  const bf16* gB = (const bf16*)g.B + (BKS ? (size_t)n0 : (size_t)n0 * g.ldb);
  const size_t stepA = AKS ? (size_t)BK * g.lda : (size_t)BK;
  const size_t stepB = BKS ? (size_t)BK * g.ldb : (size_t)BK;

  uint32_t offA[BM / 8 / NW], offB[BN / 8 / NW];
#pragma unroll
  for (int i = 0; i < BM / 8 / NW; i++) offA[i] = loader_src_offset<BM, AKS>(wave + NW * i, lane, g.lda);
#pragma unroll
  for (int i = 0; i < BN / 8 / NW; i++) offB[i] = loader_src_offset<BN, BKS>(wave + NW * i, lane, g.ldb);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  const int nk = g.K / BK;
  issue_tile_loads<BM, AKS, NW>(gA, offA, sA0, wave);
  issue_tile_loads<BN, BKS, NW>(gB, offB, sB0, wave);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  Frags<BM, BN, WGM, WGN, AKS, BKS> f0, f1;
  f0.load(sA0, sB0, 0, wm, wn, lane);
  // nk is even (K is a multiple of 128): two k-tiles per trip, buffers alternate
  for (int kt = 0; kt < nk; kt += 2) {
    gA += stepA;
    gB += stepB;
    pipe_step<BM, BN, WGM, WGN, AKS, BKS>(!g.debug_noload, g.debug_noload, gA, gB, offA, offB, sA1, sB1, sA0, sB0, f0, f1, acc, wave, wm, wn, lane);
    gA += stepA;
    gB += stepB;
    pipe_step<BM, BN, WGM, WGN, AKS, BKS>(!g.debug_noload && kt + 2 < nk, g.debug_noload, gA, gB, offA, offB, sA0, sB0, sA1, sB1, f0, f1, acc, wave,
                                          wm, wn, lane);
  }

  // ---- epilogue: lane holds C[m][n .. n+3] for 4 column groups of each 32x32 block
  const bf16* bias = (const bf16*)g.bias;
  const bf16* aux = (const bf16*)g.aux;
  const bool has_bias = (EPI != EPI_GELU_BWD && EPI != EPI_F32_ACC) && bias != nullptr;
#pragma unroll
  for (int tn = 0; tn < TN; tn++) {
#pragma unroll
    for (int q = 0; q < 4; q++) {
      const int n = n0 + wn * (BN / WGN) + tn * 32 + 8 * q + 4 * (lane >> 5);
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (has_bias) {
        bf16x4 b = *(const bf16x4*)(bias + n);
#pragma unroll
        for (int i = 0; i < 4; i++) bv[i] = bf2f(b[i]);
      }
#pragma unroll
      for (int tm = 0; tm < TM; tm++) {
        const int m = m0 + wm * (BM / WGM) + tm * 32 + (lane & 31);
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; i++) v[i] = acc[tm][tn][4 * q + i] + bv[i];
        if (EPI == EPI_F32_ACC) {
          float* cp = (float*)g.C + (size_t)m * g.ldc + n;
          if (g.beta) {
            f32x4 old = *(const f32x4*)cp;
#pragma unroll
            for (int i = 0; i < 4; i++) v[i] += old[i];
          }
          f32x4 o = {v[0], v[1], v[2], v[3]};
          *(f32x4*)cp = o;
        } else {
          if (EPI == EPI_RESID) {
            bf16x4 r = *(const bf16x4*)(aux + (size_t)m * g.ld_aux + n);
#pragma unroll
            for (int i = 0; i < 4; i++) v[i] += bf2f(r[i]);
          }
          if (EPI == EPI_GELU_BWD) {
            bf16x4 u = *(const bf16x4*)(aux + (size_t)m * g.ld_aux + n);
#pragma unroll
            for (int i = 0; i < 4; i++) v[i] *= gelu_grad_f(bf2f(u[i]));
          }
          bf16x4 o = {f2bf(v[0]), f2bf(v[1]), f2bf(v[2]), f2bf(v[3])};
          *(bf16x4*)((bf16*)g.C + (size_t)m * g.ldc + n) = o;
          if (EPI == EPI_GELU) {
            bf16x4 o2 = {f2bf(gelu_f(v[0])), f2bf(gelu_f(v[1])), f2bf(gelu_f(v[2])), f2bf(gelu_f(v[3]))};
            *(bf16x4*)((bf16*)g.C2 + (size_t)m * g.ldc + n) = o2;
          }
        }
      }
    }
  }
}

bool gemm_shape_ok(int M, int N, int K) {
  return M > 0 && N > 0 && K > 0 && (M % 128) == 0 && (N % 128) == 0 && (K % (2 * BK)) == 0;
}

namespace {

// Tile choice: the 256-CU chip runs one block per CU, so a launch costs
// ceil(tiles / 256) rounds of one tile's time.  Relative tile costs (per output
// element) are measured constants: smaller tiles re-read more from LDS and L2.
struct TileCfg { int bm, bn, wgm, wgn; float cost; };
const TileCfg kTiles[] = {{256, 256, 2, 2, 1.00f}, {256, 128, 2, 2, 1.12f}, {128, 256, 2, 2, 1.12f}, {128, 128, 2, 2, 1.35f},
                          {256, 256, 2, 4, 1.00f}, {256, 256, 4, 2, 1.00f}, {256, 128, 4, 2, 1.12f}, {128, 256, 2, 4, 1.12f}};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);
constexpr int kAutoTiles = 4;  // the automatic choice looks at the first kAutoTiles entries

int pick_tile(int M, int N) {
  static int forced = -2;
  if (forced == -2) {
    const char* e = getenv("AH_GEMM_TILE");  // tuning aid: index into kTiles
    forced = e ? atoi(e) : -1;
  }
  if (forced >= 0 && forced < kNumTiles && M % kTiles[forced].bm == 0 && N % kTiles[forced].bn == 0) return forced;
  int best = -1;
  float best_t = 0;
  for (int i = 0; i < kAutoTiles; i++) {
    if (M % kTiles[i].bm || N % kTiles[i].bn) continue;
    long tiles = (long)(M / kTiles[i].bm) * (N / kTiles[i].bn);
    long rounds = (tiles + 255) / 256;
    float t = rounds * kTiles[i].cost * kTiles[i].bm * kTiles[i].bn;
    if (best < 0 || t < best_t) { best = i; best_t = t; }
  }
  return best;
}

template <int BM, int BN, int WGM, int WGN, bool AKS, bool BKS, int EPI>
hipError_t run(const GemmArgs& a, hipStream_t s) {
  dim3 grid((a.M / BM) * (a.N / BN));
  hipLaunchKernelGGL((gemm_kernel<BM, BN, WGM, WGN, AKS, BKS, EPI>), grid, dim3(64 * WGM * WGN), 0, s, a);
  return hipGetLastError();
}

template <bool AKS, bool BKS, int EPI>
hipError_t run_tile(int t, const GemmArgs& a, hipStream_t s) {
  switch (t) {
    case 0: return run<256, 256, 2, 2, AKS, BKS, EPI>(a, s);
    case 1: return run<256, 128, 2, 2, AKS, BKS, EPI>(a, s);
    case 2: return run<128, 256, 2, 2, AKS, BKS, EPI>(a, s);
    case 3: return run<128, 128, 2, 2, AKS, BKS, EPI>(a, s);
    case 4: return run<256, 256, 2, 4, AKS, BKS, EPI>(a, s);
    case 5: return run<256, 256, 4, 2, AKS, BKS, EPI>(a, s);
    case 6: return run<256, 128, 4, 2, AKS, BKS, EPI>(a, s);
    default: return run<128, 256, 2, 4, AKS, BKS, EPI>(a, s);
  }
}

}  // namespace

hipError_t launch_gemm(GemmLayout layout, GemmEpilogue epi, const GemmArgs& a_in, hipStream_t s) {
  GemmArgs a = a_in;
  static int dbg = -1;
  if (dbg < 0) dbg = getenv("AH_GEMM_NOLOAD") ? atoi(getenv("AH_GEMM_NOLOAD")) : 0;
  a.debug_noload = dbg;
  if (!gemm_shape_ok(a.M, a.N, a.K)) return hipErrorInvalidValue;
  const int t = pick_tile(a.M, a.N);
  if (t < 0) return hipErrorInvalidValue;
  if (layout == GEMM_NN) {
    if (epi == EPI_BF16) return run_tile<false, true, EPI_BF16>(t, a, s);
    if (epi == EPI_GELU) return run_tile<false, true, EPI_GELU>(t, a, s);
    if (epi == EPI_RESID) return run_tile<false, true, EPI_RESID>(t, a, s);
  } else if (layout == GEMM_NT) {
    if (epi == EPI_BF16) return run_tile<false, false, EPI_BF16>(t, a, s);
    if (epi == EPI_GELU_BWD) return run_tile<false, false, EPI_GELU_BWD>(t, a, s);
  } else if (layout == GEMM_TN) {
    if (epi == EPI_F32_ACC) return run_tile<true, true, EPI_F32_ACC>(t, a, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace ah
