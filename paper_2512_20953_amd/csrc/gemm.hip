// bf16 GEMM for gfx950: MFMA 32x32x16, fp32 accumulators, tiles staged through
// LDS by direct global->LDS loads (16 B per lane) through a ring of operand tiles.
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
#include <algorithm>
#include <cstdlib>
#include <mutex>
#include <vector>

namespace ah {

// Two pipelines share the tile mapping, the LDS layouts, the fragment reads and the epilogue.  The forward and
// input-gradient products (at least one k-contiguous operand) use 64-wide k tiles in a ring of five operand
// buffers, so that every loader instruction fetches whole 128-byte lines of the k-contiguous operand; the weight
// gradient (both operands k-strided, rows of a tile are 256 or 512 bytes anyway) keeps 32-wide k stages in a ring of
// four, whose loads all run 2.5 stages ahead.  Measured in the stage: the first is 2-13 % faster on the former
// products, the second 1-5 % faster on the latter.

// ---------------------------------------------------------------------------
// LDS layouts, for a tile of BK = 64 or 32 k-values (all permutations are of 16-byte pieces, the unit of the loader)
//  k-contiguous tile: [rows][BK k]; row = 2 BK bytes = BK/8 pieces; piece p of row r is stored at piece
//    p ^ ((r >> 1) & 7) (BK = 64) or p ^ ((r >> 2) & 3) (BK = 32): 16 consecutive rows hit 16 distinct 16-byte bank
//    groups for the fragment reads.  With BK = 64 a loader instruction fetches 8 rows x 128 B: full cache lines
//    (64-byte row pieces, as BK = 32 gives, cost the memory pipeline twice the requests and showed up as ~10 % of
//    MFMA utilisation where an operand is k-contiguous).
//  k-strided tile: [BK k][W cols]; row = 2W bytes; the 64-byte granule g of row k is stored at granule g ^ (k & 3):
//    the 4 rows x 64 B that half a wave fetches in one transposing read cover all banks once.
// A k-strided tile may gather its columns from two column ranges of the matrix (`gw` > 0: tile columns in groups of
// gw, even groups from columns c, odd groups from columns F + c): the fused gate|up product of the SwiGLU block then
// has a gate column and its up column in the same wave's accumulators.
// ---------------------------------------------------------------------------
template <int BK, int W, bool KS>
__device__ __forceinline__ uint32_t loader_src_offset(int chunk, int lane, int ld, int gw = 0, int F = 0) {  // in bytes
  const int pos = chunk * 1024 + lane * 16;
  if (!KS) {
    constexpr int PR = BK / 8;                 // pieces per row
    constexpr int SH = BK == 64 ? 1 : 2;
    const int r = pos / (2 * BK), q = (pos >> 4) & (PR - 1);
    const int p = q ^ ((r >> SH) & (PR - 1));
    return (uint32_t)(r * ld + p * 8) * 2u;
  } else {
    constexpr int RB = W * 2;
    const int k = pos / RB, q = (pos % RB) >> 4;
    const int p = q ^ ((k & 3) << 2);
    int col = p * 8;
    if (gw > 0) col = ((col / gw) & 1) * F + (col / (2 * gw)) * gw + col % gw;
    return (uint32_t)(k * ld + col) * 2u;
  }
}

// a W x BK (or BK x W) tile is W * BK / 512 chunks of 1 KB; wave w moves chunks w, w + NW, ...
template <int BK, int W, int NW>
__device__ __forceinline__ void issue_tile_loads(const char* __restrict__ g, const uint32_t* off, char* __restrict__ lds, int wave) {
#pragma unroll
  for (int i = 0; i < W * BK / 512 / NW; i++) load16_to_lds(g + off[i], lds + (wave + NW * i) * 1024);
}

// fragment (8 k-values for row/col = lane % 32 of a 32-wide block) for k-step ks (16 k each)
template <int BK, int W, bool KS>
__device__ __forceinline__ bf16x8 read_frag(const char* __restrict__ lds, int base, int blk, int ks, int lane) {
  if (!KS) {
    constexpr int PR = BK / 8;
    constexpr int SH = BK == 64 ? 1 : 2;
    const int r = base + blk * 32 + (lane & 31);
    const int p = ks * 2 + (lane >> 5);
    const int q = p ^ ((r >> SH) & (PR - 1));
    return *(const bf16x8*)(lds + r * (2 * BK) + q * 16);
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
template <int BK, int BM, int BN, int WGM, int WGN, bool AKS, bool BKS>
struct Frags {
  static constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
  bf16x8 a[TM], b[TN];
  __device__ __forceinline__ void load(const char* __restrict__ cA, const char* __restrict__ cB, int ks, int wm, int wn, int lane) {
#pragma unroll
    for (int t = 0; t < TM; t++) a[t] = read_frag<BK, BM, AKS>(cA, wm * (BM / WGM), t, ks, lane);
#pragma unroll
    for (int t = 0; t < TN; t++) b[t] = read_frag<BK, BN, BKS>(cB, wn * (BN / WGN), t, ks, lane);
  }
};

// Scheduling hint for one k-step: between consecutive MFMAs (NM of them) place
// the NV global->LDS loads and the NR LDS reads issued for later steps, the LDS
// reads within the first three quarters so their latency is covered by the rest.
// Masks: 0x020 = vector memory read, 0x100 = LDS read, 0x008 = MFMA.
template <int I, int NM, int NR, int NV>
__device__ __forceinline__ void interleave() {
  if constexpr (I < NM) {
    constexpr int SPAN = NM * 3 / 4 > 0 ? NM * 3 / 4 : 1;
    constexpr int v = (I + 1) * NV / NM - I * NV / NM;
    constexpr int r = I < SPAN ? (I + 1) * NR / SPAN - I * NR / SPAN : 0;
    if constexpr (v > 0) __builtin_amdgcn_sched_group_barrier(0x020, v, 0);
    if constexpr (r > 0) __builtin_amdgcn_sched_group_barrier(0x100, r, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    interleave<I + 1, NM, NR, NV>();
  }
}

template <int BK, int BM, int BN, int WGM, int WGN, bool AKS, bool BKS>
__device__ __forceinline__ void mma_step(const Frags<BK, BM, BN, WGM, WGN, AKS, BKS>& f, f32x16 (&acc)[BM / WGM / 32][BN / WGN / 32]) {
  constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
#pragma unroll
  for (int tm = 0; tm < TM; tm++)
#pragma unroll
    for (int tn = 0; tn < TN; tn++)
      acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[tn], f.a[tm], acc[tm][tn], 0, 0, 0);
}

namespace k64 {
constexpr int BK = 64;  // k-extent of one operand tile in LDS (128 bytes per row of a k-contiguous operand: whole cache lines)
constexpr int NB = 5;   // operand tiles in the LDS ring (A and B tiles alternate): 2.5 k-blocks of 64

// The pipeline.  Operand tiles of 64 k are numbered A_0, B_0, A_1, B_1, ...; tile n lives in ring buffer n % 5.
// A k-block (A_j, B_j) is four k-steps of 16; fragments are double-buffered in registers (f0, f1), the fragments
// of a k-step being read from LDS under the MFMAs of the step before.  Each half of a k-block starts the loads of
// one tile three tiles ahead, into the buffer of a tile of the previous k-block.  That buffer is free: the one
// barrier per k-block (before the first fragments of the next k-block are read) is preceded by a wait for the
// wave's own LDS reads, and after it no wave reads the finished k-block again.  The same wait counts the wave's
// own loads down to the one tile issued last, so the next k-block has landed for the whole block.
// (In the code below the tile sequence is F_0, S_0, F_1, ...: F is A or B, see b_first.)
// The two halves are separate functions so that within each the buffer written is not one of the buffers read:
// the restrict qualifiers then tell the compiler that LDS reads never wait for the loads in flight.

// Which operand's tiles take the even numbers matters: an even tile is requested 2.5 half-blocks before its
// first use, an odd one 1.5.  The weights (B of the forward and input-gradient products) stream from HBM while
// the activations were just written and mostly sit in the caches, so there B goes first.
template <bool AKS>
constexpr bool b_first() { return !AKS; }

// k-steps 0 and 1 of k-block j; on entry f0 holds the fragments of k-step 0.  Starts the loads of the odd tile
// of k-block j+1.
template <int BM, int BN, int WGM, int WGN, bool AKS, bool BKS>
__device__ __forceinline__ void half_even(const char* gS, const uint32_t* offS, char* __restrict__ fill, const char* __restrict__ cA,
                                          const char* __restrict__ cB, Frags<BK, BM, BN, WGM, WGN, AKS, BKS>& f0,
                                          Frags<BK, BM, BN, WGM, WGN, AKS, BKS>& f1, f32x16 (&acc)[BM / WGM / 32][BN / WGN / 32],
                                          int wave, int wm, int wn, int lane) {
  constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32, NW = WGM * WGN;
  constexpr int NR = TM * (AKS ? 2 : 1) + TN * (BKS ? 2 : 1), NM = TM * TN;
  constexpr int WS = b_first<AKS>() ? BM : BN;  // the odd tiles are A tiles when B goes first
  issue_tile_loads<BK, WS, NW>(gS, offS, fill, wave);
  f1.load(cA, cB, 1, wm, wn, lane);
  mma_step<BK, BM, BN, WGM, WGN, AKS, BKS>(f0, acc);
  interleave<0, NM, NR, WS / 8 / NW>();
  f0.load(cA, cB, 2, wm, wn, lane);
  mma_step<BK, BM, BN, WGM, WGN, AKS, BKS>(f1, acc);
  interleave<0, NM, NR, 0>();
}

// k-steps 2 and 3 of k-block j; on entry f0 holds the fragments of k-step 2.  Starts the loads of the even tile
// of k-block j+2, waits for k-block j+1 (nA, nB) and leaves its first fragments in f0.
template <int BM, int BN, int WGM, int WGN, bool AKS, bool BKS>
__device__ __forceinline__ void half_odd(const char* gF, const uint32_t* offF, char* __restrict__ fill, const char* __restrict__ cA,
                                         const char* __restrict__ cB, const char* __restrict__ nA, const char* __restrict__ nB,
                                         Frags<BK, BM, BN, WGM, WGN, AKS, BKS>& f0, Frags<BK, BM, BN, WGM, WGN, AKS, BKS>& f1,
                                         f32x16 (&acc)[BM / WGM / 32][BN / WGN / 32], int wave, int wm, int wn, int lane) {
  constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32, NW = WGM * WGN;
  constexpr int NR = TM * (AKS ? 2 : 1) + TN * (BKS ? 2 : 1), NM = TM * TN;
  constexpr int WF = b_first<AKS>() ? BN : BM;
  issue_tile_loads<BK, WF, NW>(gF, offF, fill, wave);
  f1.load(cA, cB, 3, wm, wn, lane);
  mma_step<BK, BM, BN, WGM, WGN, AKS, BKS>(f0, acc);
  interleave<0, NM, NR, WF / 8 / NW>();
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(WF / 8 / NW));
  __builtin_amdgcn_s_barrier();
  f0.load(nA, nB, 0, wm, wn, lane);
  mma_step<BK, BM, BN, WGM, WGN, AKS, BKS>(f1, acc);
  interleave<0, NM, NR, 0>();
}

}  // namespace k64

namespace k32 {
constexpr int BK = 32;  // k-extent of one LDS stage (64 bytes of bf16)
constexpr int NS = 4;   // stages in the LDS ring: loads run 3 stages ahead of the MFMAs

// One stage (32 of k) of the pipeline.  On entry f0 holds the fragments of
// k-step 0 of the current stage (cA, cB).  Starts the loads of the stage three
// ahead into the ring slot that the previous stage just vacated (fA, fB),
// multiplies k-step 0 while fetching k-step 1, then waits until the next stage
// (nA, nB) has landed for the whole block (own loads by count: two later
// stages may stay in flight; then the barrier) and refills f0 from it under the
// MFMAs of k-step 1.  The restrict qualifiers tell the compiler that the three
// slots are distinct, so LDS reads never wait for the loads in flight.
template <int BM, int BN, int WGM, int WGN, bool AKS, bool BKS>
__device__ __forceinline__ void ring_step(const char* gA, const char* gB, const uint32_t* offA, const uint32_t* offB,
                                          char* __restrict__ fA, char* __restrict__ fB, const char* __restrict__ cA,
                                          const char* __restrict__ cB, const char* __restrict__ nA, const char* __restrict__ nB,
                                          Frags<BK, BM, BN, WGM, WGN, AKS, BKS>& f0, Frags<BK, BM, BN, WGM, WGN, AKS, BKS>& f1,
                                          f32x16 (&acc)[BM / WGM / 32][BN / WGN / 32], int wave, int wm, int wn, int lane) {
  constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32, NW = WGM * WGN;
  constexpr int NR = TM * (AKS ? 2 : 1) + TN * (BKS ? 2 : 1), NM = TM * TN;
  constexpr int LPS = (BM + BN) / 16 / NW;  // loads per stage per wave
  issue_tile_loads<BK, BM, NW>(gA, offA, fA, wave);
  issue_tile_loads<BK, BN, NW>(gB, offB, fB, wave);
  f1.load(cA, cB, 1, wm, wn, lane);
  mma_step<BK, BM, BN, WGM, WGN, AKS, BKS>(f0, acc);
  interleave<0, NM, NR, LPS>();
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(2 * LPS));
  __builtin_amdgcn_s_barrier();
  f0.load(nA, nB, 0, wm, wn, lane);
  mma_step<BK, BM, BN, WGM, WGN, AKS, BKS>(f1, acc);
  interleave<0, NM, NR, 0>();
}

}  // namespace k32

template <int BM, int BN, int WGM, int WGN, bool AKS, bool BKS, int EPI>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(GemmArgs g) {
  constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32, NW = WGM * WGN;
  constexpr bool K32 = AKS && BKS;  // which pipeline
  // EPI_SWIGLU: the B tile gathers GW gate columns and their GW up columns per wave (see loader_src_offset); the
  // launch runs over N = 2 F tile columns that stand for F logical ones.
  constexpr bool SWIGLU = EPI == EPI_SWIGLU;
  constexpr int GW = SWIGLU ? BN / WGN / 2 : 0;
  static_assert(!SWIGLU || (!AKS && BKS), "the fused SwiGLU epilogue belongs to the forward layout");
  constexpr int BUF = (BM > BN ? BM : BN) * 128;        // k64: one ring buffer holds an A or a B tile
  constexpr int RING = K32 ? k32::NS * (BM + BN) * 64 : k64::NB * BUF;
  // the epilogue reuses the ring as staging space
  __shared__ __attribute__((aligned(1024))) char ring[RING];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps LDS bases in scalar registers
  const int wm = wave / WGN, wn = wave % WGN;

  // block -> tile: consecutive logical tiles share an XCD (blocks are dealt to the
  // 8 XCDs round-robin), and run down groups of 8 tile-rows so that the tiles in
  // flight on one XCD reuse the same operand panels in its L2.
  const int tiles_m = g.M / BM, tiles_n = g.N / BN, ntiles = tiles_m * tiles_n;
  int logical = blockIdx.x;
  if ((ntiles & 7) == 0 && g.xcd_remap) logical = (blockIdx.x & 7) * (ntiles >> 3) + (blockIdx.x >> 3);
  const int GROUP = g.group;
  const int per_group = GROUP * tiles_n;
  const int gid = logical / per_group;
  const int first_m = gid * GROUP;
  const int gsize = min(tiles_m - first_m, GROUP);
  const int in_group = logical - gid * per_group;
  const int m0 = (first_m + in_group % gsize) * BM;
  const int n0 = (in_group / gsize) * BN;

  const char* gA = (const char*)((const bf16*)g.A + (AKS ? (size_t)m0 : (size_t)m0 * g.lda));
  const char* gB = (const char*)((const bf16*)g.B + (BKS ? (size_t)(SWIGLU ? n0 / 2 : n0) : (size_t)n0 * g.ldb));
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  if constexpr (K32) {
    using namespace k32;
    constexpr int LPS = (BM + BN) / 16 / NW;
    constexpr int SLOT = (BM + BN) * 64;  // ring slot t: A tile at t * SLOT, B tile behind it
    char* const sA0 = ring;
    char* const sB0 = ring + BM * 64;
    char* const sA1 = ring + SLOT;
    char* const sB1 = ring + SLOT + BM * 64;
    char* const sA2 = ring + 2 * SLOT;
    char* const sB2 = ring + 2 * SLOT + BM * 64;
    char* const sA3 = ring + 3 * SLOT;
    char* const sB3 = ring + 3 * SLOT + BM * 64;
    const size_t stepA = (size_t)BK * g.lda * 2;  // bytes per stage (both operands k-strided)
    const size_t stepB = (size_t)BK * g.ldb * 2;
    uint32_t offA[BM / 16 / NW], offB[BN / 16 / NW];
#pragma unroll
    for (int i = 0; i < BM / 16 / NW; i++) offA[i] = loader_src_offset<BK, BM, AKS>(wave + NW * i, lane, g.lda);
#pragma unroll
    for (int i = 0; i < BN / 16 / NW; i++) offB[i] = loader_src_offset<BK, BN, BKS>(wave + NW * i, lane, g.ldb, GW, g.swiglu_F);
    // nk is a multiple of 4 (K is a multiple of 128).  Stage t lives in ring slot t % 4.
    const int nk = g.K / BK;
    // The k axis may be cut into pieces that live in different buffers (kernels.h): the outer loop runs over the
    // pieces, the inner one over the stages of a piece (a multiple of 4).  The stage fetched during local step t
    // is local stage t + 3; past the end of the piece that is a stage of the next piece, past the end of the last
    // piece the last stage again (fetched into a dead slot, which keeps the in-flight load count uniform).  The
    // choice is a scalar select, so the inner loop stays one basic block.
    const int nseg = g.n_seg > 0 ? g.n_seg : 1;
    const int seg_stages = nk / nseg;
    issue_tile_loads<BK, BM, NW>(gA, offA, sA0, wave);
    issue_tile_loads<BK, BN, NW>(gB, offB, sB0, wave);
    issue_tile_loads<BK, BM, NW>(gA + stepA, offA, sA1, wave);
    issue_tile_loads<BK, BN, NW>(gB + stepB, offB, sB1, wave);
    issue_tile_loads<BK, BM, NW>(gA + 2 * stepA, offA, sA2, wave);
    issue_tile_loads<BK, BN, NW>(gB + 2 * stepB, offB, sB2, wave);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(2 * LPS));
    __builtin_amdgcn_s_barrier();

    Frags<BK, BM, BN, WGM, WGN, AKS, BKS> f0, f1;
    f0.load(sA0, sB0, 0, wm, wn, lane);
    const char *curA = gA, *curB = gB;
    for (int sg = 0; sg < nseg; sg++) {
      const bool last_piece = sg + 1 == nseg;
      const char* nxtA = last_piece ? curA : (const char*)((const bf16*)g.segA[sg + 1] + m0);
      const char* nxtB = last_piece ? curB : (const char*)((const bf16*)g.segB[sg + 1] + n0);
      const int lim = last_piece ? seg_stages - 1 : seg_stages + 2;
#define AH_STAGE_PTRS(u)                                                                                              \
  (min((u), lim) >= seg_stages ? nxtA + (size_t)(min((u), lim) - seg_stages) * stepA : curA + (size_t)min((u), lim) * stepA), \
      (min((u), lim) >= seg_stages ? nxtB + (size_t)(min((u), lim) - seg_stages) * stepB : curB + (size_t)min((u), lim) * stepB)
      for (int t = 0; t < seg_stages; t += 4) {
        ring_step<BM, BN, WGM, WGN, AKS, BKS>(AH_STAGE_PTRS(t + 3), offA, offB, sA3, sB3, sA0, sB0, sA1, sB1, f0, f1, acc, wave, wm, wn, lane);
        ring_step<BM, BN, WGM, WGN, AKS, BKS>(AH_STAGE_PTRS(t + 4), offA, offB, sA0, sB0, sA1, sB1, sA2, sB2, f0, f1, acc, wave, wm, wn, lane);
        ring_step<BM, BN, WGM, WGN, AKS, BKS>(AH_STAGE_PTRS(t + 5), offA, offB, sA1, sB1, sA2, sB2, sA3, sB3, f0, f1, acc, wave, wm, wn, lane);
        ring_step<BM, BN, WGM, WGN, AKS, BKS>(AH_STAGE_PTRS(t + 6), offA, offB, sA2, sB2, sA3, sB3, sA0, sB0, f0, f1, acc, wave, wm, wn, lane);
      }
#undef AH_STAGE_PTRS
      curA = nxtA;
      curB = nxtB;
    }
  } else {
    using namespace k64;
    constexpr int LA = BM / 8 / NW, LB = BN / 8 / NW;     // loads per tile per wave
    const size_t stepA = (AKS ? (size_t)BK * g.lda : (size_t)BK) * 2;  // bytes per k-block
    const size_t stepB = (BKS ? (size_t)BK * g.ldb : (size_t)BK) * 2;

    uint32_t offA[LA], offB[LB];
#pragma unroll
    for (int i = 0; i < LA; i++) offA[i] = loader_src_offset<BK, BM, AKS>(wave + NW * i, lane, g.lda);
#pragma unroll
    for (int i = 0; i < LB; i++) offB[i] = loader_src_offset<BK, BN, BKS>(wave + NW * i, lane, g.ldb, GW, g.swiglu_F);

    // K is a multiple of 128: an even number of k-blocks.  Past the end the last k-block is fetched again into
    // dead buffers, which keeps the number of loads in flight uniform for the counted wait.
    // F = the operand whose tiles take the even numbers, S = the other one.
    constexpr bool BF = b_first<AKS>();
    constexpr int WF = BF ? BN : BM, WS = BF ? BM : BN;
    const char* gF = BF ? gB : gA;
    const char* gS = BF ? gA : gB;
    const size_t stepF = BF ? stepB : stepA, stepS = BF ? stepA : stepB;
    const uint32_t* offF = BF ? offB : offA;
    const uint32_t* offS = BF ? offA : offB;
    const int np = g.K / BK, lastp = np - 1;
    // In the weight-gradient layout the k axis may be cut into pieces that live in different buffers (kernels.h):
    // the outer loop runs over the pieces (one piece for the other layouts), the inner one over the k-blocks of a
    // piece (an even number).  During local k-block j the tiles S_{j+1} and F_{j+2} are fetched; past the end of
    // the piece those belong to the next piece, past the end of the last piece the last k-block is fetched again.
    constexpr bool PIECES = AKS && BKS;
    const int nseg = (PIECES && g.n_seg > 0) ? g.n_seg : 1;
    const int seg_blocks = np / nseg;
    issue_tile_loads<BK, WF, NW>(gF, offF, ring, wave);                                            // F_0 -> buffer 0
    issue_tile_loads<BK, WS, NW>(gS, offS, ring + BUF, wave);                                      // S_0 -> buffer 1
    issue_tile_loads<BK, WF, NW>(gF + (size_t)min(1, lastp) * stepF, offF, ring + 2 * BUF, wave);  // F_1 -> buffer 2
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(WF / 8 / NW));
    __builtin_amdgcn_s_barrier();

    Frags<BK, BM, BN, WGM, WGN, AKS, BKS> f0, f1;
    f0.load(ring + (BF ? BUF : 0), ring + (BF ? 0 : BUF), 0, wm, wn, lane);
    int jf = 0, js = 1;  // buffers of F_j and S_j
    const char *curF = gF, *curS = gS;
    for (int sg = 0; sg < nseg; sg++) {
      const bool last_piece = sg + 1 == nseg;
      const char *nxtF = curF, *nxtS = curS;
      if constexpr (PIECES) {
        if (!last_piece) {
          nxtF = (const char*)((const bf16*)(BF ? g.segB[sg + 1] : g.segA[sg + 1]) + (BF ? n0 : m0));
          nxtS = (const char*)((const bf16*)(BF ? g.segA[sg + 1] : g.segB[sg + 1]) + (BF ? m0 : n0));
        }
      }
      const int lim = last_piece ? seg_blocks - 1 : seg_blocks + 1;
      for (int j = 0; j < seg_blocks; j++) {
        const int nf = jf + 2 >= NB ? jf + 2 - NB : jf + 2;  // F_{j+1}
        const int ns = js + 2 >= NB ? js + 2 - NB : js + 2;  // S_{j+1}: loaded now, into the buffer of F_{j-1}
        const int ff = jf + 4 >= NB ? jf + 4 - NB : jf + 4;  // F_{j+2}: into the buffer of S_{j-1}
        const char* cA = ring + (BF ? js : jf) * BUF;
        const char* cB = ring + (BF ? jf : js) * BUF;
        const char* nA = ring + (BF ? ns : nf) * BUF;
        const char* nB = ring + (BF ? nf : ns) * BUF;
        const int us = min(j + 1, lim), uf = min(j + 2, lim);
        const char* pS = (PIECES && us >= seg_blocks) ? nxtS + (size_t)(us - seg_blocks) * stepS : curS + (size_t)us * stepS;
        const char* pF = (PIECES && uf >= seg_blocks) ? nxtF + (size_t)(uf - seg_blocks) * stepF : curF + (size_t)uf * stepF;
        half_even<BM, BN, WGM, WGN, AKS, BKS>(pS, offS, ring + ns * BUF, cA, cB, f0, f1, acc, wave, wm, wn, lane);
        half_odd<BM, BN, WGM, WGN, AKS, BKS>(pF, offF, ring + ff * BUF, cA, cB, nA, nB, f0, f1, acc, wave, wm, wn, lane);
        jf = nf;
        js = ns;
      }
      curF = nxtF;
      curS = nxtS;
    }
  }
  __builtin_amdgcn_s_waitcnt(0);  // drain the redundant tail loads before the block's LDS is released

  // ---- epilogue.  A lane holds C[m][n .. n+3] for 4 column groups of each 32x32 block: stores
  // straight from that layout would touch 32 rows per instruction, 16 bytes each.  Instead each
  // wave passes its sub-tile through a private LDS strip, 32 rows at a time in fp32, and reads it
  // back row-major, so that every global access is 16 bytes per lane and whole rows per 16 lanes.
  constexpr int WN = BN / WGN, WM = BM / WGM;
  constexpr int ROWB = WN * 4 + 16;                // padded strip row
  static_assert(NW * 32 * ROWB <= RING, "staging strips must fit in the ring");
  __syncthreads();                                  // every wave is done with the ring
  char* strip = ring + wave * (32 * ROWB);
  const bf16* bias = (const bf16*)g.bias;
  const bf16* aux = (const bf16*)g.aux;
  constexpr bool RESID = EPI == EPI_RESID || EPI == EPI_RESID_F32 || EPI == EPI_RESID_F32_OUT16;
  constexpr bool AUX_F32 = EPI == EPI_RESID_F32 || EPI == EPI_RESID_F32_OUT16;   // the residual is read in fp32
  constexpr bool OUT_F32 = EPI == EPI_F32_ACC || EPI == EPI_F32_SET || EPI == EPI_RESID_F32;
  const bool has_bias = (EPI == EPI_BF16 || EPI == EPI_GELU || RESID) && bias != nullptr;
  constexpr int PPR = WN / 8;                       // 8-column pieces per strip row
  constexpr int NIT = 32 * PPR / 64;                // pieces per lane per strip
  static_assert(64 % PPR == 0, "a lane keeps its column piece across iterations");
  const int cp = lane % PPR, row0 = lane / PPR;     // piece it*64 + lane -> row row0 + it * (64 / PPR)
  // output column of the lane's piece.  SwiGLU: the first half of the wave's strip row holds GW gate columns, the
  // second half their up columns; both go to u[:, 2F] (gate at column c, up at F + c), their product to C2[:, F].
  const bool up_piece = SWIGLU && cp >= PPR / 2;
  const int nlog = SWIGLU ? n0 / 2 + wn * GW + (up_piece ? cp - PPR / 2 : cp) * 8 : 0;   // logical column of the piece
  const int n = SWIGLU ? (up_piece ? g.swiglu_F + nlog : nlog) : n0 + wn * WN + cp * 8;
  float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (has_bias) {
    const bf16x8 b = *(const bf16x8*)(bias + n);
#pragma unroll
    for (int i = 0; i < 8; i++) bv[i] = bf2f(b[i]);
  }
  float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};  // EPI_GELU_BWD: this lane's column sums over the current 64-row slab
  const bool want_colsum = EPI == EPI_GELU_BWD && g.colsum_part != nullptr;
  // EPI_ROPE: this lane's 8 pairs, the partner piece, and (cos, sin) of 64 / PPR angle steps (the distance between a
  // lane's consecutive rows), read once from the table's row of that position; per strip of 32 rows (which never
  // straddles a sequence: S is a multiple of 128) the angles of the lane's first row are read from the table and
  // carried from row to row by rotation
  const bool rot = EPI == EPI_ROPE && n < g.rope_cols;
  float rc[8], rs[8], dcs_c[8], dcs_s[8];
  int rope_pcp = 0, rope_i0 = 0;
  float rope_sgn = 0.f;
  if (EPI == EPI_ROPE && rot) {
    const int d = g.rope_d, ch = (cp * 8) % d, half = d >> 1;
    const bool lower = ch < half;
    rope_pcp = lower ? cp + (d >> 4) : cp - (d >> 4);
    rope_i0 = lower ? ch : ch - half;
    rope_sgn = lower ? -1.f : 1.f;
    const float* t = g.rope_cs + ((size_t)(64 / PPR) * half + rope_i0) * 2;
#pragma unroll
    for (int q4 = 0; q4 < 4; q4++) {
      const f32x4 e = *(const f32x4*)(t + 4 * q4);
      dcs_c[2 * q4] = e[0]; dcs_s[2 * q4] = e[1]; dcs_c[2 * q4 + 1] = e[2]; dcs_s[2 * q4 + 1] = e[3];
    }
  }
#pragma unroll
  for (int tm = 0; tm < TM; tm++) {
    const int mbase = m0 + wm * WM + tm * 32 + row0;
    if (EPI == EPI_ROPE && rot) {
      const float* t = g.rope_cs + ((size_t)(mbase % g.rope_S) * (g.rope_d >> 1) + rope_i0) * 2;
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        const f32x4 e = *(const f32x4*)(t + 4 * q4);
        rc[2 * q4] = e[0]; rs[2 * q4] = e[1]; rc[2 * q4 + 1] = e[2]; rs[2 * q4 + 1] = e[3];
      }
    }
    // operands of the epilogue that come from memory: issue their loads before the strip round trip
    bf16x8 ax[NIT], ax2[EPI == EPI_SWIGLU_BWD ? NIT : 1];
    f32x4 old0[NIT], old1[NIT];
    if (EPI == EPI_RESID || EPI == EPI_GELU_BWD || EPI == EPI_SWIGLU_BWD) {
#pragma unroll
      for (int it = 0; it < NIT; it++) ax[it] = *(const bf16x8*)(aux + (size_t)(mbase + it * (64 / PPR)) * g.ld_aux + n);
    }
    if (EPI == EPI_SWIGLU_BWD) {  // aux = gate | up: the up columns sit swiglu_F further
#pragma unroll
      for (int it = 0; it < NIT; it++) ax2[it] = *(const bf16x8*)(aux + (size_t)(mbase + it * (64 / PPR)) * g.ld_aux + g.swiglu_F + n);
    }
    if (EPI == EPI_F32_ACC || AUX_F32) {
#pragma unroll
      for (int it = 0; it < NIT; it++) {
        const float* cptr = (AUX_F32 ? (const float*)g.aux : (const float*)g.C) + (size_t)(mbase + it * (64 / PPR)) * (AUX_F32 ? g.ld_aux : g.ldc) + n;
        old0[it] = *(const f32x4*)cptr;
        old1[it] = *(const f32x4*)(cptr + 4);
      }
    }
#pragma unroll
    for (int tn = 0; tn < TN; tn++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int col = tn * 32 + 8 * q + 4 * (lane >> 5);
        f32x4 v = {acc[tm][tn][4 * q], acc[tm][tn][4 * q + 1], acc[tm][tn][4 * q + 2], acc[tm][tn][4 * q + 3]};
        *(f32x4*)(strip + (lane & 31) * ROWB + col * 4) = v;
      }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(63));
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < NIT; it++) {
      const int row = row0 + it * (64 / PPR);
      const f32x4 lo = *(const f32x4*)(strip + row * ROWB + cp * 32);
      const f32x4 hi = *(const f32x4*)(strip + row * ROWB + cp * 32 + 16);
      float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      const size_t m = (size_t)(mbase + it * (64 / PPR));
      if (OUT_F32) {
        float* cptr = (float*)g.C + m * g.ldc + n;
        if (EPI == EPI_F32_ACC || EPI == EPI_RESID_F32) {
          if (EPI == EPI_RESID_F32) {
#pragma unroll
            for (int i = 0; i < 8; i++) v[i] += bv[i];
          }
#pragma unroll
          for (int i = 0; i < 4; i++) { v[i] += old0[it][i]; v[4 + i] += old1[it][i]; }
        }
        *(f32x4*)cptr = f32x4{v[0], v[1], v[2], v[3]};
        *(f32x4*)(cptr + 4) = f32x4{v[4], v[5], v[6], v[7]};
      } else {
#pragma unroll
        for (int i = 0; i < 8; i++) v[i] += bv[i];
        if (EPI == EPI_RESID) {
#pragma unroll
          for (int i = 0; i < 8; i++) v[i] += bf2f(ax[it][i]);
        }
        if (EPI == EPI_ROPE && rot) {
          // rotary embedding on the fp32 sums: the pair of column c of a head is c +- d/2, d/16 pieces away in the
          // same strip row (a wave's strip holds whole heads: WN % d == 0, checked by the caller)
          const f32x4 plo = *(const f32x4*)(strip + row * ROWB + rope_pcp * 32);
          const f32x4 phi = *(const f32x4*)(strip + row * ROWB + rope_pcp * 32 + 16);
          const float pv[8] = {plo[0], plo[1], plo[2], plo[3], phi[0], phi[1], phi[2], phi[3]};
#pragma unroll
          for (int i = 0; i < 8; i++) {
            v[i] = v[i] * rc[i] + rope_sgn * pv[i] * rs[i];
            // the lane's next row is 64 / PPR positions further: rotate (cos, sin) by that many steps of the angle
            const float c2 = rc[i] * dcs_c[i] - rs[i] * dcs_s[i];
            rs[i] = rs[i] * dcs_c[i] + rc[i] * dcs_s[i];
            rc[i] = c2;
          }
        }
        if (EPI == EPI_RESID_F32_OUT16) {
#pragma unroll
          for (int i = 0; i < 4; i++) { v[i] += old0[it][i]; v[4 + i] += old1[it][i]; }
        }
        if (EPI == EPI_GELU_BWD) {
#pragma unroll
          for (int i = 0; i < 8; i++) v[i] *= gelu_grad_f(bf2f(ax[it][i]));
        }
        bf16x8 o;
        if (EPI == EPI_SWIGLU_BWD) {
          // v = dm; d(gate) = dm up silu'(gate) goes to column n, d(up) = dm silu(gate) to column F + n
          bf16x8 o2;
#pragma unroll
          for (int i = 0; i < 8; i++) {
            const float x = bf2f(ax[it][i]), sg = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
            o[i] = f2bf(v[i] * bf2f(ax2[it][i]) * sg * __builtin_fmaf(x, 1.0f - sg, 1.0f));
            o2[i] = f2bf(v[i] * x * sg);
          }
          *(bf16x8*)((bf16*)g.C + m * g.ldc + g.swiglu_F + n) = o2;
        } else {
#pragma unroll
          for (int i = 0; i < 8; i++) o[i] = f2bf(v[i]);
        }
        *(bf16x8*)((bf16*)g.C + m * g.ldc + n) = o;
        if (EPI == EPI_GELU) {
          bf16x8 o2;
#pragma unroll
          for (int i = 0; i < 8; i++) o2[i] = f2bf(gelu_f(v[i]));
          *(bf16x8*)((bf16*)g.C2 + m * g.ldc + n) = o2;
        }
        if (EPI == EPI_GELU_BWD) {
#pragma unroll
          for (int i = 0; i < 8; i++) cs[i] += bf2f(o[i]);
        }
        if (SWIGLU && !up_piece) {
          // silu(gate) * up from the fp32 accumulators: the up piece sits PPR / 2 pieces further in the strip row
          const f32x4 ulo = *(const f32x4*)(strip + row * ROWB + (cp + PPR / 2) * 32);
          const f32x4 uhi = *(const f32x4*)(strip + row * ROWB + (cp + PPR / 2) * 32 + 16);
          const float up[8] = {ulo[0], ulo[1], ulo[2], ulo[3], uhi[0], uhi[1], uhi[2], uhi[3]};
          bf16x8 o2;
#pragma unroll
          for (int i = 0; i < 8; i++) o2[i] = f2bf(silu_f(v[i]) * up[i]);
          *(bf16x8*)((bf16*)g.C2 + m * g.ldc2 + nlog) = o2;
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(63));  // strip reads are in registers before the next 32 rows overwrite it
    __builtin_amdgcn_wave_barrier();
    if (EPI == EPI_GELU_BWD && (tm & 1)) {
      // two strips = one 64-row slab: lanes that share a column piece (lane % PPR) add up, the first PPR lanes write
      if (want_colsum) {
#pragma unroll
        for (int i = 0; i < 8; i++) {
#pragma unroll
          for (int off = PPR; off < 64; off <<= 1) cs[i] += __shfl_xor(cs[i], off);
        }
        if (lane < PPR) {
          float* dst = g.colsum_part + (size_t)((m0 + wm * WM + tm * 32) >> 6) * g.ld_colsum + n;
          if (g.colsum_acc) {
            const f32x4 o0 = *(const f32x4*)dst, o1 = *(const f32x4*)(dst + 4);
#pragma unroll
            for (int i = 0; i < 4; i++) { cs[i] += o0[i]; cs[4 + i] += o1[i]; }
          }
          *(f32x4*)dst = f32x4{cs[0], cs[1], cs[2], cs[3]};
          *(f32x4*)(dst + 4) = f32x4{cs[4], cs[5], cs[6], cs[7]};
        }
      }
#pragma unroll
      for (int i = 0; i < 8; i++) cs[i] = 0.f;
    }
  }
}

bool gemm_shape_ok(int M, int N, int K) {
  return M > 0 && N > 0 && K > 0 && (M % 128) == 0 && (N % 128) == 0 && (K % 128) == 0;
}

bool gemm_segments_ok(int seg_k, int n_seg) {
  return seg_k > 0 && (seg_k % 128) == 0 && n_seg >= 1 && n_seg <= kMaxGemmSegments && (long)seg_k * n_seg <= (1L << 30);
}

namespace {

// Tile choice: the 256-CU chip runs one block per CU, so a launch costs
// ceil(tiles / 256) rounds of one tile's time.  Relative tile costs (per output
// element) are measured constants: smaller tiles re-read more from LDS and L2
// (4096 x 6144 x 4096, NN: 384 tiles of 256 x 256 in two rounds take 211 us, 768
// tiles of 256 x 128 in three rounds 219 us, i.e. 1.35 per element; the weight
// gradient, whose epilogue moves twice the bytes per tile, loses less: 1.25).
struct TileCfg { int bm, bn, wgm, wgn; float cost, cost_tn; };
const TileCfg kTiles[] = {{256, 256, 2, 2, 1.00f, 1.00f}, {256, 128, 2, 2, 1.35f, 1.25f}, {128, 256, 2, 2, 1.35f, 1.25f},
                          {128, 128, 2, 2, 1.60f, 1.50f}};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);
constexpr int kAutoTiles = 4;  // the automatic choice looks at the first kAutoTiles entries

int forced_tile() {
  static int forced = -2;
  if (forced == -2) {
    const char* e = getenv("AH_GEMM_TILE");  // tuning aid: index into kTiles
    forced = e ? atoi(e) : -1;
  }
  return forced;
}

// cost of covering an M x n output with tile i, in units of (tile area x relative cost) per round
float tile_cost(int i, int M, int n, bool tn) {
  const long tiles = (long)(M / kTiles[i].bm) * (n / kTiles[i].bn);
  const long rounds = (tiles + 255) / 256;
  return rounds * (tn ? kTiles[i].cost_tn : kTiles[i].cost) * kTiles[i].bm * kTiles[i].bn;
}

int pick_tile(int M, int N, bool tn) {
  const int forced = forced_tile();
  if (forced >= 0 && forced < kNumTiles && M % kTiles[forced].bm == 0 && N % kTiles[forced].bn == 0) return forced;
  int best = -1;
  float best_t = 0;
  for (int i = 0; i < kAutoTiles; i++) {
    if (M % kTiles[i].bm || N % kTiles[i].bn) continue;
    const float t = tile_cost(i, M, N, tn);
    if (best < 0 || t < best_t) { best = i; best_t = t; }
  }
  return best;
}

// How a launch covers its output: with one tile shape, or as two launches over the column ranges [0, n0) and
// [n0, N), each with its own tile shape.  The second form is for outputs whose tile count is not a good multiple
// of the 256 CUs: 4096 x 6144 is 384 tiles of 256 x 256, i.e. two rounds of which the second is half empty (2.0
// units), or 768 tiles of 256 x 128 in three rounds (2.0 .. 1.9); 256 tiles of 256 x 256 over the first 4096
// columns and then 256 tiles of 256 x 128 over the rest is two full rounds of 1.0 + 0.63 .. 0.68 units.
struct Plan { int parts; int tile[2]; int n0; };
constexpr float kSplitCost = 0.15f * 256 * 256;  // the second launch's gap, prologue and epilogue, in the same units

Plan make_plan(int M, int N, bool tn) {
  Plan p = {1, {pick_tile(M, N, tn), -1}, N};
  if (p.tile[0] < 0 || forced_tile() >= 0 || getenv("AH_GEMM_NOSPLIT")) return p;
  float best = tile_cost(p.tile[0], M, N, tn);
  for (int n0 = 128; n0 < N; n0 += 128)
    for (int i = 0; i < kAutoTiles; i++) {
      if (M % kTiles[i].bm || n0 % kTiles[i].bn) continue;
      for (int j = 0; j < kAutoTiles; j++) {
        if (j == i || M % kTiles[j].bm || (N - n0) % kTiles[j].bn) continue;
        const float t = tile_cost(i, M, n0, tn) + tile_cost(j, M, N - n0, tn) + kSplitCost;
        if (t < best) { best = t; p = {2, {i, j}, n0}; }
      }
    }
  return p;
}

// make_plan is a search over a few thousand candidates: remembered per (M, N, layout class)
Plan cached_plan(int M, int N, bool tn) {
  struct Entry { int M, N; bool tn; Plan p; };
  static std::mutex mu;
  static std::vector<Entry> cache;
  std::lock_guard<std::mutex> lock(mu);
  for (const Entry& e : cache)
    if (e.M == M && e.N == N && e.tn == tn) return e.p;
  const Plan p = make_plan(M, N, tn);
  if (cache.size() < 4096) cache.push_back({M, N, tn, p});
  return p;
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
    default: return run<128, 128, 2, 2, AKS, BKS, EPI>(a, s);
  }
}

}  // namespace

int gemm_min_wave_cols(int M, int N, GemmLayout layout) {
  if (!gemm_shape_ok(M, N, 128)) return 0;
  const Plan p = cached_plan(M, N, layout == GEMM_TN);
  if (p.tile[0] < 0) return 0;
  int w = kTiles[p.tile[0]].bn / kTiles[p.tile[0]].wgn;
  if (p.parts == 2) w = std::min(w, kTiles[p.tile[1]].bn / kTiles[p.tile[1]].wgn);
  return w;
}

int gemm_tile_area(int M, int N, GemmLayout layout) {
  if (!gemm_shape_ok(M, N, 128)) return 0;
  const Plan p = cached_plan(M, N, layout == GEMM_TN);
  return p.tile[0] < 0 ? 0 : kTiles[p.tile[0]].bm * kTiles[p.tile[0]].bn;
}

namespace {

hipError_t dispatch(GemmLayout layout, GemmEpilogue epi, int t, const GemmArgs& a, hipStream_t s) {
  if (layout == GEMM_NN) {
    if (epi == EPI_BF16) return run_tile<false, true, EPI_BF16>(t, a, s);
    if (epi == EPI_GELU) return run_tile<false, true, EPI_GELU>(t, a, s);
    if (epi == EPI_RESID) return run_tile<false, true, EPI_RESID>(t, a, s);
    if (epi == EPI_RESID_F32) return run_tile<false, true, EPI_RESID_F32>(t, a, s);
    if (epi == EPI_RESID_F32_OUT16) return run_tile<false, true, EPI_RESID_F32_OUT16>(t, a, s);
    if (epi == EPI_SWIGLU) return run_tile<false, true, EPI_SWIGLU>(t, a, s);
    if (epi == EPI_ROPE) return run_tile<false, true, EPI_ROPE>(t, a, s);
  } else if (layout == GEMM_NT) {
    if (epi == EPI_BF16) return run_tile<false, false, EPI_BF16>(t, a, s);
    if (epi == EPI_GELU_BWD) return run_tile<false, false, EPI_GELU_BWD>(t, a, s);
    if (epi == EPI_SWIGLU_BWD) return run_tile<false, false, EPI_SWIGLU_BWD>(t, a, s);
  } else if (layout == GEMM_TN) {
    if (epi == EPI_F32_ACC) return a.beta ? run_tile<true, true, EPI_F32_ACC>(t, a, s) : run_tile<true, true, EPI_F32_SET>(t, a, s);
  }
  return hipErrorInvalidValue;
}

// the same problem restricted to output columns [c0, c0 + n)
GemmArgs column_range(GemmLayout layout, GemmEpilogue epi, const GemmArgs& a, int c0, int n) {
  GemmArgs b = a;
  b.N = n;
  if (epi == EPI_SWIGLU) {  // c0 tile columns stand for c0 / 2 logical ones of each of gate, up and the product
    b.B = (const bf16*)a.B + c0 / 2;
    b.C = (bf16*)a.C + c0 / 2;
    b.C2 = (bf16*)a.C2 + c0 / 2;
    return b;
  }
  const bool f32 = layout == GEMM_TN || epi == EPI_RESID_F32;
  const bool aux_f32 = epi == EPI_RESID_F32 || epi == EPI_RESID_F32_OUT16;
  b.C = f32 ? (void*)((float*)a.C + c0) : (void*)((bf16*)a.C + c0);
  if (a.C2) b.C2 = (bf16*)a.C2 + c0;
  if (a.bias) b.bias = (const bf16*)a.bias + c0;
  if (a.aux) b.aux = aux_f32 ? (const void*)((const float*)a.aux + c0) : (const void*)((const bf16*)a.aux + c0);
  if (a.colsum_part) b.colsum_part = a.colsum_part + c0;
  b.rope_cols = a.rope_cols - c0;  // the rotated columns are counted from the launch's first column
  if (layout == GEMM_NT) {
    b.B = (const bf16*)a.B + (size_t)c0 * a.ldb;  // B is [N, K]
  } else {
    b.B = (const bf16*)a.B + c0;                  // B is [K, N]
    for (int i = 0; i < a.n_seg; i++) b.segB[i] = (const bf16*)a.segB[i] + c0;
  }
  return b;
}

}  // namespace

hipError_t launch_gemm(GemmLayout layout, GemmEpilogue epi, const GemmArgs& a_in, hipStream_t s) {
  GemmArgs a = a_in;
  static int grp = -1, remap = -1;
  if (grp < 0) { grp = getenv("AH_GEMM_GROUP") ? atoi(getenv("AH_GEMM_GROUP")) : 8; remap = getenv("AH_GEMM_NOREMAP") ? 0 : 1; }
  a.group = grp; a.xcd_remap = remap;
  if (!gemm_shape_ok(a.M, a.N, a.K)) return hipErrorInvalidValue;
  if (a.n_seg != 0) {  // pieces along k: weight-gradient layout only, and the pieces must add up to K
    if (layout != GEMM_TN || !gemm_segments_ok(a.seg_k, a.n_seg) || (long)a.seg_k * a.n_seg != a.K) return hipErrorInvalidValue;
    for (int i = 0; i < a.n_seg; i++)
      if (!a.segA[i] || !a.segB[i]) return hipErrorInvalidValue;
    a.A = a.segA[0];
    a.B = a.segB[0];
  }
  const Plan p = cached_plan(a.M, a.N, layout == GEMM_TN);
  if (p.tile[0] < 0) return hipErrorInvalidValue;
  if (p.parts == 1) return dispatch(layout, epi, p.tile[0], a, s);
  hipError_t e = dispatch(layout, epi, p.tile[0], column_range(layout, epi, a, 0, p.n0), s);
  if (e != hipSuccess) return e;
  return dispatch(layout, epi, p.tile[1], column_range(layout, epi, a, p.n0, a.N - p.n0), s);
}

}  // namespace ah
