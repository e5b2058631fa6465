// Fused self-attention (causal or bidirectional) for gfx950, forward and backward, on the packed
// projection output qkv[T, 3*nh*d] ([Q | K | V], head-major).  No S x S matrix
// ever reaches HBM: scores are produced tile by tile with MFMA 32x32x16, the
// softmax runs in fp32 registers (base-2 exponent), and the backward pass
// rebuilds the probabilities from the saved log-sum-exp.
//
// All products are computed "transposed" (keys or head-dim along the MFMA row
// axis, one query or one key per lane), so that
//   - every per-row softmax quantity is a per-lane scalar, and
//   - an accumulator tile converts to the next product's bf16 operand in
//     place: the 8 values a lane holds for a 16-wide contraction step are the
//     operand's 8 slots; the other operand is fetched from LDS in the matching
//     slot order with the transposing LDS read.
// Tiles of 64 rows of K, V (or Q, dO) are staged through LDS by direct
// global->LDS loads into a 4-slot ring; loads run 3 tiles ahead and are waited
// for by count, with one block barrier per tile.
//
// Backward is two deterministic kernels (no atomics): one block per 128
// queries accumulates dQ over the key tiles at or before it and leaves
// delta = rowsum(dO * O) of its queries behind; one block per 128 keys then
// accumulates dK and dV over the query tiles at or after it (causal; without
// the mask both walk every tile of the sequence).
#include "common.h"
#include "kernels.h"
#include <cstdlib>

namespace ah {
namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr int NSLOT = 2;  // ring slots of the forward and dQ kernels (two blocks share a CU)

// nothing is scheduled across this point
#define AH_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
// Issue priority of the wave among the waves of its SIMD: raised for the runs of matrix instructions, so that the
// other wave's vector work (softmax, masks, conversions) fills in behind them instead of delaying them.  Used in the
// forward kernel (8 % faster on launches of more than two blocks per CU); in the dQ kernel it cost 1-3 %.
#define AH_PRIO(p) __builtin_amdgcn_s_setprio(p)

// LDS tile [64 rows][D] bf16.  16-byte piece p of row r is stored at piece
// swz(r, p): conflict-free both for 16-byte reads down a column of pieces and
// for the transposing reads of 4 rows x 64 bytes.
template <int D>
__device__ __forceinline__ int swz(int r, int p) {
  if (D == 128) return p ^ ((r & 3) << 2) ^ ((r >> 2) & 3);
  return p ^ (r & 7);
}

template <int D>
__device__ __forceinline__ uint32_t tile_src_offset(int chunk, int lane, int ld) {
  constexpr int RB = 2 * D;
  const int pos = chunk * 1024 + lane * 16;
  const int r = pos / RB, q = (pos % RB) >> 4;
  return (uint32_t)(r * ld + swz<D>(r, q) * 8);
}

template <int D>
__device__ __forceinline__ void issue_tile(const bf16* __restrict__ g, const uint32_t* off, char* __restrict__ lds, int wave) {
#pragma unroll
  for (int i = 0; i < D / 32; i++) load16_to_lds(g + off[i], lds + (wave + 4 * i) * 1024);
}

// 8 consecutive head-dim values (k-step ks, half hf) of row r
template <int D>
__device__ __forceinline__ bf16x8 frag_rowmajor(const char* __restrict__ t, int r, int ks, int hf) {
  return *(const bf16x8*)(t + r * (2 * D) + swz<D>(r, 2 * ks + hf) * 16);
}

// column (dt*32 + lane%32) of rows rbase..rbase+3 and rbase+8..rbase+11
template <int D>
__device__ __forceinline__ bf16x8 frag_transposed(const char* __restrict__ t, int rbase, int dt, int lane) {
  const int r = rbase + ((lane & 15) >> 2);
  const int c = dt * 32 + ((lane >> 4) & 1) * 16 + 4 * (lane & 3);
  bf16x4 lo = lds_read_tr4(t + r * (2 * D) + swz<D>(r, c >> 3) * 16 + (c & 7) * 2);
  bf16x4 hi = lds_read_tr4(t + (r + 8) * (2 * D) + swz<D>(r + 8, c >> 3) * 16 + (c & 7) * 2);
  return cat4(lo, hi);
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& a, int s2) {
  bf16x8 p;
#pragma unroll
  for (int j = 0; j < 8; j++) p[j] = f2bf(a[8 * s2 + j]);
  return p;
}

__device__ __forceinline__ float fexp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Query block of a thread block under the causal mask (block qb walks 2*qb + 2 key tiles).  A launch that
// fits on the chip at once (two blocks per CU, 256 CUs) is placed statically, blocks i and i + grid/2 on
// the same CU, so the second half of the grid runs the light blocks in ascending order and every CU gets
// the same total; a larger launch is dispatched as CUs free up and simply goes heaviest first.
__device__ __forceinline__ int causal_query_block(int r, int nq) {
  if (gridDim.x > 512) return nq - 1 - r;
  const int half = (nq + 1) / 2;
  return r < half ? nq - 1 - r : r - half;
}

// =========================================================================== forward
template <int D>
struct FwdState {
  bf16x8 qf[D / 16];
  f32x16 oacc[D / 32];
  float m, l;
};

// The running maximum is only raised when a new score exceeds it by more than this many powers of two:
// probabilities are then at most 2^8 instead of 1, which fp32 sums and the bf16 operand of the second
// product hold with unchanged relative accuracy, and the rescaling of the output accumulator -- the
// largest block of vector arithmetic in the loop -- runs on the first tile only in practice.
constexpr float RESCALE_SLACK = 8.f;

// One key tile of 64 for the wave's 32 queries.  LDS reads are issued a phase ahead of their use (see
// dkv_tile); the mask costs vector work only on tiles that straddle the diagonal (diag is wave-uniform).
template <int D>
__device__ __forceinline__ void fwd_tile(const char* __restrict__ cK, const char* __restrict__ cV, FwdState<D>& st, int k0,
                                         int q, bool diag, float sc2, int lane) {
  constexpr int NK = D / 16, ND = D / 32;
  const int hf = lane >> 5;
  bf16x8 fk0[NK], fk1[NK];
#pragma unroll
  for (int ks = 0; ks < NK; ks++) fk0[ks] = frag_rowmajor<D>(cK, lane & 31, ks, hf);
  AH_SCHED_FENCE();
  f32x16 s0, s1;
#pragma unroll
  for (int r = 0; r < 16; r++) { s0[r] = 0.f; s1[r] = 0.f; }
  AH_PRIO(1);
#pragma unroll
  for (int ks = 0; ks < NK; ks++) s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk0[ks], st.qf[ks], s0, 0, 0, 0);
#pragma unroll
  for (int ks = 0; ks < NK; ks++) fk1[ks] = frag_rowmajor<D>(cK, 32 + (lane & 31), ks, hf);
  AH_SCHED_FENCE();
  bf16x8 v0[2][ND], v1[2][ND];
#pragma unroll
  for (int ks = 0; ks < NK; ks++) s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk1[ks], st.qf[ks], s1, 0, 0, 0);
#pragma unroll
  for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
    for (int dt = 0; dt < ND; dt++) v0[s2][dt] = frag_transposed<D>(cV, 16 * s2 + 4 * hf, dt, lane);
  AH_PRIO(0);
  AH_SCHED_FENCE();
  if (diag) {
    // element r of half t is key k0 + t*32 + 8*(r/4) + 4*hf + r%4: masked iff that exceeds q
    const int lim = q - k0 - 4 * hf;
#pragma unroll
    for (int r = 0; r < 16; r++) {
      if (8 * (r >> 2) + (r & 3) > lim) s0[r] = -INFINITY;
      if (32 + 8 * (r >> 2) + (r & 3) > lim) s1[r] = -INFINITY;
    }
  }
  float mx = fmaxf(s0[0], s1[0]);
#pragma unroll
  for (int r = 1; r < 16; r++) mx = fmaxf(mx, fmaxf(s0[r], s1[r]));
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * sc2;
  if (__any(mx > st.m + RESCALE_SLACK)) {  // wave-uniform branch
    const float m_new = fmaxf(st.m, mx);
    const float alpha = fexp2(st.m - m_new);
    st.m = m_new;
    st.l *= alpha;
#pragma unroll
    for (int dt = 0; dt < ND; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) st.oacc[dt][r] *= alpha;
  }
  const float nm = -st.m;
  float ls = 0.f;
#pragma unroll
  for (int r = 0; r < 16; r++) {
    s0[r] = fexp2(__builtin_fmaf(s0[r], sc2, nm));
    s1[r] = fexp2(__builtin_fmaf(s1[r], sc2, nm));
    ls += s0[r] + s1[r];
  }
  st.l += ls;
#pragma unroll
  for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
    for (int dt = 0; dt < ND; dt++) v1[s2][dt] = frag_transposed<D>(cV, 32 + 16 * s2 + 4 * hf, dt, lane);
  AH_SCHED_FENCE();
  AH_PRIO(1);
#pragma unroll
  for (int s2 = 0; s2 < 2; s2++) {
    const bf16x8 pf = pack8(s0, s2);
#pragma unroll
    for (int dt = 0; dt < ND; dt++) st.oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v0[s2][dt], pf, st.oacc[dt], 0, 0, 0);
  }
#pragma unroll
  for (int s2 = 0; s2 < 2; s2++) {
    const bf16x8 pf = pack8(s1, s2);
#pragma unroll
    for (int dt = 0; dt < ND; dt++) st.oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v1[s2][dt], pf, st.oacc[dt], 0, 0, 0);
  }
  AH_PRIO(0);
  AH_SCHED_FENCE();
}

// MAY_SKIP: the tile may lie wholly after the wave's queries (only the last tile of a block, under the mask)
template <int D, bool CAUSAL, bool MAY_SKIP>
__device__ __forceinline__ void fwd_step(const bf16* gK, const bf16* gV, const uint32_t* off, char* __restrict__ nK,
                                         char* __restrict__ nV, const char* __restrict__ cK, const char* __restrict__ cV,
                                         FwdState<D>& st, int k0, int q, int qw0, float sc2, int wave, int lane) {
  issue_tile<D>(gK, off, nK, wave);
  issue_tile<D>(gV, off, nV, wave);
  if (CAUSAL && MAY_SKIP && k0 > qw0 + 31) return;
  fwd_tile<D>(cK, cV, st, k0, q, CAUSAL && k0 + 63 > qw0, sc2, lane);
}

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void attn_fwd_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ o, float* __restrict__ lse,
                                                       int S, int nh, float sc2) {
  constexpr int TILEB = 64 * 2 * D, STAGE = 2 * TILEB, LPS = 2 * (D / 32);  // ring slot = K tile then V tile
  __shared__ __attribute__((aligned(1024))) char ring[NSLOT * STAGE];
  const int lane = threadIdx.x & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform: LDS bases stay scalar
  const int nbh = gridDim.x / (S / 128);
  const int bh = blockIdx.x % nbh;
  const int qb = CAUSAL ? causal_query_block(blockIdx.x / nbh, S / 128) : blockIdx.x / nbh;
  const int b = bh / nh, head = bh % nh;
  const int ld = 3 * nh * D;
  const bf16* qp = qkv + (size_t)b * S * ld + head * D;
  const bf16* kp = qp + nh * D;
  const bf16* vp = qp + 2 * nh * D;
  const int qw0 = qb * 128 + wave * 32, q = qw0 + (lane & 31);

  FwdState<D> st;
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++) st.qf[ks] = *(const bf16x8*)(qp + (size_t)q * ld + ks * 16 + hf * 8);
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int r = 0; r < 16; r++) st.oacc[dt][r] = 0.f;
  st.m = -INFINITY;
  st.l = 0.f;

  uint32_t off[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++) off[i] = tile_src_offset<D>(wave + 4 * i, lane, ld);

  // key tiles of 64 up to and including the diagonal (all of them without the mask).  Tile t lives in ring
  // slot t % NSLOT; the tile loaded during step j is min(j + NSLOT - 1, last): past the end the last tile is
  // fetched again into a dead slot, which keeps the number of loads in flight uniform for the counted wait.
  const int ntile = CAUSAL ? 2 * qb + 2 : S / 64, last = ntile - 1;
  const size_t step = (size_t)64 * ld;
#pragma unroll
  for (int t = 0; t < NSLOT - 1; t++) {
    const size_t o = (size_t)min(t, last) * step;
    issue_tile<D>(kp + o, off, ring + t * STAGE, wave);
    issue_tile<D>(vp + o, off, ring + t * STAGE + TILEB, wave);
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NSLOT - 2) * LPS));
  __builtin_amdgcn_s_barrier();
  // Only the last tile can lie wholly after a wave's queries (waves 0 and 1 under the mask): it is peeled so
  // that the loop body has a single path.
  for (int j = 0; j < last; j++) {
    const size_t o = (size_t)min(j + NSLOT - 1, last) * step;
    char* fill = ring + ((j + NSLOT - 1) & (NSLOT - 1)) * STAGE;
    const char* cur = ring + (j & (NSLOT - 1)) * STAGE;
    fwd_step<D, CAUSAL, false>(kp + o, vp + o, off, fill, fill + TILEB, cur, cur + TILEB, st, j * 64, q, qw0, sc2, wave, lane);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NSLOT - 2) * LPS));
    __builtin_amdgcn_s_barrier();
  }
  {
    const size_t o = (size_t)last * step;
    char* fill = ring + ((last + NSLOT - 1) & (NSLOT - 1)) * STAGE;
    const char* cur = ring + (last & (NSLOT - 1)) * STAGE;
    fwd_step<D, CAUSAL, true>(kp + o, vp + o, off, fill, fill + TILEB, cur, cur + TILEB, st, last * 64, q, qw0, sc2, wave, lane);
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));  // drain the redundant tail loads

  const float l = st.l + __shfl_xor(st.l, 32, 64);
  const float inv = 1.f / l;
  bf16* op = o + ((size_t)b * S + q) * (nh * D) + head * D;
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int g = 0; g < 4; g++) {
      bf16x4 v;
#pragma unroll
      for (int i = 0; i < 4; i++) v[i] = f2bf(st.oacc[dt][4 * g + i] * inv);
      *(bf16x4*)(op + dt * 32 + 8 * g + 4 * hf) = v;
    }
  if (hf == 0) lse[((size_t)b * nh + head) * S + q] = (st.m + __log2f(l)) * LN2;
}

// =========================================================================== forward for launches that cannot fill the chip
// With at most one 128-query block per CU a wave sits alone on its SIMD and the launch lasts as long as the block
// with the most key tiles.  Here a block takes 64 queries and its four waves split the work two ways: wave w
// owns queries 32 * (w & 1) .. + 31 and, of every 64-key tile, the keys 32 * (w >> 1) .. + 31.  There are twice as
// many blocks (two per CU, heavy ones paired with light ones) and every wave walks half the keys of its queries;
// the two partial results per query (running maximum, sum and output accumulator) meet in LDS at the end.
template <int D>
__device__ __forceinline__ void fwd_half_tile(const char* __restrict__ cK, const char* __restrict__ cV, FwdState<D>& st, int kbase,
                                              int kh, int q, bool diag, float sc2, int lane) {
  constexpr int NK = D / 16, ND = D / 32;
  const int hf = lane >> 5;
  bf16x8 fk[NK];
#pragma unroll
  for (int ks = 0; ks < NK; ks++) fk[ks] = frag_rowmajor<D>(cK, 32 * kh + (lane & 31), ks, hf);
  AH_SCHED_FENCE();
  f32x16 s;
#pragma unroll
  for (int r = 0; r < 16; r++) s[r] = 0.f;
#pragma unroll
  for (int ks = 0; ks < NK; ks++) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[ks], st.qf[ks], s, 0, 0, 0);
  bf16x8 v[2][ND];
#pragma unroll
  for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
    for (int dt = 0; dt < ND; dt++) v[s2][dt] = frag_transposed<D>(cV, 32 * kh + 16 * s2 + 4 * hf, dt, lane);
  AH_SCHED_FENCE();
  if (diag) {
    // element r is key kbase + 8*(r/4) + 4*hf + r%4: masked iff that exceeds q
    const int lim = q - kbase - 4 * hf;
#pragma unroll
    for (int r = 0; r < 16; r++)
      if (8 * (r >> 2) + (r & 3) > lim) s[r] = -INFINITY;
  }
  float mx = s[0];
#pragma unroll
  for (int r = 1; r < 16; r++) mx = fmaxf(mx, s[r]);
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * sc2;
  if (__any(mx > st.m + RESCALE_SLACK)) {  // wave-uniform branch
    const float m_new = fmaxf(st.m, mx);
    const float alpha = fexp2(st.m - m_new);
    st.m = m_new;
    st.l *= alpha;
#pragma unroll
    for (int dt = 0; dt < ND; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) st.oacc[dt][r] *= alpha;
  }
  const float nm = -st.m;
  float ls = 0.f;
#pragma unroll
  for (int r = 0; r < 16; r++) {
    s[r] = fexp2(__builtin_fmaf(s[r], sc2, nm));
    ls += s[r];
  }
  st.l += ls;
  AH_SCHED_FENCE();
#pragma unroll
  for (int s2 = 0; s2 < 2; s2++) {
    const bf16x8 pf = pack8(s, s2);
#pragma unroll
    for (int dt = 0; dt < ND; dt++) st.oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v[s2][dt], pf, st.oacc[dt], 0, 0, 0);
  }
  AH_SCHED_FENCE();
}

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void attn_fwd64_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ o, float* __restrict__ lse,
                                                         int S, int nh, float sc2) {
  constexpr int TILEB = 64 * 2 * D, STAGE = 2 * TILEB, ND = D / 32;
  __shared__ __attribute__((aligned(1024))) char ring[NSLOT * STAGE];
  static_assert(2 * (ND * 16 + 2) * 64 * 4 <= NSLOT * STAGE, "the partial results of two waves fit in the ring");
  const int lane = threadIdx.x & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qt = wave & 1, kh = wave >> 1;
  const int nq = S / 64;
  const int nbh = gridDim.x / nq;
  const int bh = blockIdx.x % nbh;
  const int qb = CAUSAL ? causal_query_block(blockIdx.x / nbh, nq) : blockIdx.x / nbh;
  const int b = bh / nh, head = bh % nh;
  const int ld = 3 * nh * D;
  const bf16* qp = qkv + (size_t)b * S * ld + head * D;
  const bf16* kp = qp + nh * D;
  const bf16* vp = qp + 2 * nh * D;
  const int qw0 = qb * 64 + qt * 32, q = qw0 + (lane & 31);

  FwdState<D> st;
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++) st.qf[ks] = *(const bf16x8*)(qp + (size_t)q * ld + ks * 16 + hf * 8);
#pragma unroll
  for (int dt = 0; dt < ND; dt++)
#pragma unroll
    for (int r = 0; r < 16; r++) st.oacc[dt][r] = 0.f;
  st.m = -INFINITY;
  st.l = 0.f;

  uint32_t off[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++) off[i] = tile_src_offset<D>(wave + 4 * i, lane, ld);

  // key tiles of 64 up to and including the one that holds the block's own keys; tile t lives in ring slot t % 2
  // and is fetched during step t - 1 (past the end the last tile again, into a slot nobody reads)
  const int ntile = CAUSAL ? qb + 1 : nq, last = ntile - 1;
  const size_t step = (size_t)64 * ld;
  issue_tile<D>(kp, off, ring, wave);
  issue_tile<D>(vp, off, ring + TILEB, wave);
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
  __builtin_amdgcn_s_barrier();
  for (int j = 0; j < ntile; j++) {
    const size_t o2 = (size_t)min(j + 1, last) * step;
    char* fill = ring + ((j + 1) & 1) * STAGE;
    const char* cur = ring + (j & 1) * STAGE;
    issue_tile<D>(kp + o2, off, fill, wave);
    issue_tile<D>(vp + o2, off, fill + TILEB, wave);
    // In the block's own tile the wave's keys lie before (kh < qt), on (kh == qt) or after (kh > qt) its queries.
    const bool own = CAUSAL && j == last;
    if (!(own && kh > qt)) fwd_half_tile<D>(cur, cur + TILEB, st, j * 64 + 32 * kh, kh, q, own && kh == qt, sc2, lane);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
    __builtin_amdgcn_s_barrier();
  }

  // merge: the waves of the second key half leave (m, l, O) in LDS, lane by lane; the others fold them in
  float* mg = (float*)ring + (size_t)qt * (ND * 16 + 2) * 64;
  if (kh == 1) {
#pragma unroll
    for (int dt = 0; dt < ND; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) mg[(dt * 16 + r) * 64 + lane] = st.oacc[dt][r];
    mg[(ND * 16) * 64 + lane] = st.m;
    mg[(ND * 16 + 1) * 64 + lane] = st.l;
  }
  __syncthreads();
  if (kh == 1) return;
  const float m2 = mg[(ND * 16) * 64 + lane], l2 = mg[(ND * 16 + 1) * 64 + lane];
  const float m = fmaxf(st.m, m2);
  const float a1 = fexp2(st.m - m), a2 = fexp2(m2 - m);  // m2 = -inf (nothing visible in that half) gives a2 = 0
  const float lsum = a1 * st.l + a2 * l2;
  const float l = lsum + __shfl_xor(lsum, 32, 64);
  const float inv = 1.f / l;
  bf16* op = o + ((size_t)b * S + q) * (nh * D) + head * D;
#pragma unroll
  for (int dt = 0; dt < ND; dt++)
#pragma unroll
    for (int g = 0; g < 4; g++) {
      bf16x4 v;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int r = 4 * g + i;
        v[i] = f2bf((a1 * st.oacc[dt][r] + a2 * mg[(dt * 16 + r) * 64 + lane]) * inv);
      }
      *(bf16x4*)(op + dt * 32 + 8 * g + 4 * hf) = v;
    }
  if (hf == 0) lse[((size_t)b * nh + head) * S + q] = (m + __log2f(l)) * LN2;
}

// =========================================================================== backward: dQ (one block per 128 queries)
// delta_q = sum_c dO[q, c] O[q, c] for the lane's query: the lane holds half of the row of dO as MFMA fragments
// (columns ks * 16 + hf * 8 ..), reads the same columns of O, and the two lanes of a query add their halves.
// The dQ kernels compute it for their own queries and leave it in `delta` for the dK/dV kernel, which runs after them.
template <int D>
__device__ __forceinline__ float row_delta(const bf16x8 (&dof)[D / 16], const bf16* __restrict__ orow, int hf) {
  float s = 0.f;
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++) {
    const bf16x8 ov = *(const bf16x8*)(orow + ks * 16 + hf * 8);
#pragma unroll
    for (int j = 0; j < 8; j++) s = __builtin_fmaf(bf2f(dof[ks][j]), bf2f(ov[j]), s);
  }
  return s + __shfl_xor(s, 32, 64);
}

template <int D>
struct DqState {
  bf16x8 qf[D / 16], dof[D / 16];
  f32x16 acc[D / 32];
  float lse2, delta;
};

// One key tile of 64 for the wave's 32 queries.  With head_dim 64 the LDS reads run a phase ahead of their
// use as in dkv_tile; with head_dim 128 the 256 registers of a wave (two blocks share a CU) leave no room
// for fragments in flight, so they are fetched where they are used and the other block covers the wait.
template <int D>
__device__ __forceinline__ void dq_tile(const char* __restrict__ cK, const char* __restrict__ cV, DqState<D>& st, int k0, int q,
                                        bool diag, float sc2, int lane) {
  constexpr int NK = D / 16, ND = D / 32;
  constexpr bool AHEAD = D == 64;
  const int hf = lane >> 5;
  const int lim = q - k0 - 4 * hf;  // element r of half t is masked iff t*32 + 8*(r/4) + r%4 > lim
  bf16x8 fk[NK], fv[NK];
  if (AHEAD) {
#pragma unroll
    for (int ks = 0; ks < NK; ks++) {
      fk[ks] = frag_rowmajor<D>(cK, lane & 31, ks, hf);
      fv[ks] = frag_rowmajor<D>(cV, lane & 31, ks, hf);
    }
  }
#pragma unroll
  for (int t = 0; t < 2; t++) {
    if (AHEAD) AH_SCHED_FENCE();
    f32x16 s, dp;
#pragma unroll
    for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = -st.delta; }   // the product dO V^T lands on -delta: dP - delta for free
    bf16x8 kt[2][ND];
#pragma unroll
    for (int ks = 0; ks < NK; ks++) {
      if (!AHEAD) {
        fk[ks] = frag_rowmajor<D>(cK, t * 32 + (lane & 31), ks, hf);
        fv[ks] = frag_rowmajor<D>(cV, t * 32 + (lane & 31), ks, hf);
      }
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[ks], st.qf[ks], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[ks], st.dof[ks], dp, 0, 0, 0);
    }
    if (AHEAD) {
#pragma unroll
      for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
        for (int dt = 0; dt < ND; dt++) kt[s2][dt] = frag_transposed<D>(cK, t * 32 + 16 * s2 + 4 * hf, dt, lane);
      AH_SCHED_FENCE();
    }
    const float nl = -st.lse2;
#pragma unroll
    for (int r = 0; r < 16; r++) s[r] = fexp2(__builtin_fmaf(s[r], sc2, nl));
    if (diag) {  // wave-uniform
#pragma unroll
      for (int r = 0; r < 16; r++)
        if (t * 32 + 8 * (r >> 2) + (r & 3) > lim) s[r] = 0.f;
    }
#pragma unroll
    for (int r = 0; r < 16; r++) s[r] *= dp[r];  // dS^T
    if (AHEAD && t == 0) {
#pragma unroll
      for (int ks = 0; ks < NK; ks++) {
        fk[ks] = frag_rowmajor<D>(cK, 32 + (lane & 31), ks, hf);
        fv[ks] = frag_rowmajor<D>(cV, 32 + (lane & 31), ks, hf);
      }
    }
    if (AHEAD) AH_SCHED_FENCE();
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++) {
      const bf16x8 dsf = pack8(s, s2);
#pragma unroll
      for (int dt = 0; dt < ND; dt++) {
        if (!AHEAD) kt[s2][dt] = frag_transposed<D>(cK, t * 32 + 16 * s2 + 4 * hf, dt, lane);
        st.acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt[s2][dt], dsf, st.acc[dt], 0, 0, 0);
      }
    }
  }
  if (AHEAD) AH_SCHED_FENCE();
}

template <int D, bool CAUSAL, bool MAY_SKIP>
__device__ __forceinline__ void dq_step(const bf16* gK, const bf16* gV, const uint32_t* off, char* __restrict__ nK,
                                        char* __restrict__ nV, const char* __restrict__ cK, const char* __restrict__ cV,
                                        DqState<D>& st, int k0, int q, int qw0, float sc2, int wave, int lane) {
  issue_tile<D>(gK, off, nK, wave);
  issue_tile<D>(gV, off, nV, wave);
  if (CAUSAL && MAY_SKIP && k0 > qw0 + 31) return;
  dq_tile<D>(cK, cV, st, k0, q, CAUSAL && k0 + 63 > qw0, sc2, lane);
}

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void attn_dq_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ o,
                                                      const bf16* __restrict__ d_o, const float* __restrict__ lse,
                                                      float* __restrict__ delta, bf16* __restrict__ dqkv, int S, int nh,
                                                      float sc2, float scale) {
  constexpr int TILEB = 64 * 2 * D, STAGE = 2 * TILEB, LPS = 2 * (D / 32);  // ring slot = K tile then V tile
  __shared__ __attribute__((aligned(1024))) char ring[NSLOT * STAGE];
  const int lane = threadIdx.x & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform: LDS bases stay scalar
  const int nbh = gridDim.x / (S / 128);
  const int bh = blockIdx.x % nbh;
  const int qb = CAUSAL ? causal_query_block(blockIdx.x / nbh, S / 128) : blockIdx.x / nbh;
  const int b = bh / nh, head = bh % nh;
  const int ld = 3 * nh * D;
  const bf16* qp = qkv + (size_t)b * S * ld + head * D;
  const bf16* kp = qp + nh * D;
  const bf16* vp = qp + 2 * nh * D;
  const int qw0 = qb * 128 + wave * 32, q = qw0 + (lane & 31);

  DqState<D> st;
  const bf16* dop = d_o + ((size_t)b * S + q) * (nh * D) + head * D;
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++) {
    st.qf[ks] = *(const bf16x8*)(qp + (size_t)q * ld + ks * 16 + hf * 8);
    st.dof[ks] = *(const bf16x8*)(dop + ks * 16 + hf * 8);
  }
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int r = 0; r < 16; r++) st.acc[dt][r] = 0.f;
  st.lse2 = lse[((size_t)b * nh + head) * S + q] * LOG2E;
  st.delta = row_delta<D>(st.dof, o + ((size_t)b * S + q) * (nh * D) + head * D, hf);
  if (hf == 0) delta[((size_t)b * nh + head) * S + q] = st.delta;

  uint32_t off[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++) off[i] = tile_src_offset<D>(wave + 4 * i, lane, ld);

  // key tiles of 64 up to and including the diagonal (all of them without the mask).  Tile t lives in ring
  // slot t % NSLOT; the tile loaded during step j is min(j + NSLOT - 1, last): past the end the last tile is
  // fetched again into a dead slot, which keeps the number of loads in flight uniform for the counted wait.
  const int ntile = CAUSAL ? 2 * qb + 2 : S / 64, last = ntile - 1;
  const size_t step = (size_t)64 * ld;
#pragma unroll
  for (int t = 0; t < NSLOT - 1; t++) {
    const size_t o = (size_t)min(t, last) * step;
    issue_tile<D>(kp + o, off, ring + t * STAGE, wave);
    issue_tile<D>(vp + o, off, ring + t * STAGE + TILEB, wave);
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NSLOT - 2) * LPS));
  __builtin_amdgcn_s_barrier();
  for (int j = 0; j < last; j++) {
    const size_t o = (size_t)min(j + NSLOT - 1, last) * step;
    char* fill = ring + ((j + NSLOT - 1) & (NSLOT - 1)) * STAGE;
    const char* cur = ring + (j & (NSLOT - 1)) * STAGE;
    dq_step<D, CAUSAL, false>(kp + o, vp + o, off, fill, fill + TILEB, cur, cur + TILEB, st, j * 64, q, qw0, sc2, wave, lane);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NSLOT - 2) * LPS));
    __builtin_amdgcn_s_barrier();
  }
  {  // the last tile, peeled as in the forward kernel
    const size_t o = (size_t)last * step;
    char* fill = ring + ((last + NSLOT - 1) & (NSLOT - 1)) * STAGE;
    const char* cur = ring + (last & (NSLOT - 1)) * STAGE;
    dq_step<D, CAUSAL, true>(kp + o, vp + o, off, fill, fill + TILEB, cur, cur + TILEB, st, last * 64, q, qw0, sc2, wave, lane);
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));  // drain the redundant tail loads

  bf16* out = dqkv + ((size_t)b * S + q) * ld + head * D;
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int g = 0; g < 4; g++) {
      bf16x4 v;
#pragma unroll
      for (int i = 0; i < 4; i++) v[i] = f2bf(st.acc[dt][4 * g + i] * scale);
      *(bf16x4*)(out + dt * 32 + 8 * g + 4 * hf) = v;
    }
}

// =========================================================================== backward: dQ for launches that cannot fill the chip
// The split of attn_fwd64_kernel applied to dQ: 64 queries per block, wave w owns queries 32 * (w & 1) .. + 31 and
// keys 32 * (w >> 1) .. + 31 of every 64-key tile; the two partial dQ per query are added in LDS at the end.
template <int D>
__device__ __forceinline__ void dq_half_tile(const char* __restrict__ cK, const char* __restrict__ cV, DqState<D>& st, int kbase,
                                             int kh, int q, bool diag, float sc2, int lane) {
  constexpr int NK = D / 16, ND = D / 32;
  const int hf = lane >> 5;
  // with head_dim 128 the 256 registers of a wave (two blocks share a CU) leave no room for all fragments at once:
  // they are fetched where they are used and the other block covers the wait
  constexpr bool AHEAD = D == 64;
  bf16x8 fk[NK], fv[NK];
  if (AHEAD) {
#pragma unroll
    for (int ks = 0; ks < NK; ks++) {
      fk[ks] = frag_rowmajor<D>(cK, 32 * kh + (lane & 31), ks, hf);
      fv[ks] = frag_rowmajor<D>(cV, 32 * kh + (lane & 31), ks, hf);
    }
    AH_SCHED_FENCE();
  }
  f32x16 s, dp;
#pragma unroll
  for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = -st.delta; }   // dP - delta for free
#pragma unroll
  for (int ks = 0; ks < NK; ks++) {
    if (!AHEAD) {
      fk[ks] = frag_rowmajor<D>(cK, 32 * kh + (lane & 31), ks, hf);
      fv[ks] = frag_rowmajor<D>(cV, 32 * kh + (lane & 31), ks, hf);
    }
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[ks], st.qf[ks], s, 0, 0, 0);
    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[ks], st.dof[ks], dp, 0, 0, 0);
  }
  bf16x8 kt[2][ND];
  if (AHEAD) {
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
      for (int dt = 0; dt < ND; dt++) kt[s2][dt] = frag_transposed<D>(cK, 32 * kh + 16 * s2 + 4 * hf, dt, lane);
    AH_SCHED_FENCE();
  }
  const float nl = -st.lse2;
#pragma unroll
  for (int r = 0; r < 16; r++) s[r] = fexp2(__builtin_fmaf(s[r], sc2, nl));
  if (diag) {  // wave-uniform; element r is key kbase + 8*(r/4) + 4*hf + r%4
    const int lim = q - kbase - 4 * hf;
#pragma unroll
    for (int r = 0; r < 16; r++)
      if (8 * (r >> 2) + (r & 3) > lim) s[r] = 0.f;
  }
#pragma unroll
  for (int r = 0; r < 16; r++) s[r] *= dp[r];  // dS^T
  if (AHEAD) AH_SCHED_FENCE();
#pragma unroll
  for (int s2 = 0; s2 < 2; s2++) {
    const bf16x8 dsf = pack8(s, s2);
#pragma unroll
    for (int dt = 0; dt < ND; dt++) {
      if (!AHEAD) kt[s2][dt] = frag_transposed<D>(cK, 32 * kh + 16 * s2 + 4 * hf, dt, lane);
      st.acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt[s2][dt], dsf, st.acc[dt], 0, 0, 0);
    }
  }
  if (AHEAD) AH_SCHED_FENCE();
}

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void attn_dq64_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ o,
                                                        const bf16* __restrict__ d_o, const float* __restrict__ lse,
                                                        float* __restrict__ delta, bf16* __restrict__ dqkv, int S, int nh,
                                                        float sc2, float scale) {
  constexpr int TILEB = 64 * 2 * D, STAGE = 2 * TILEB, ND = D / 32;
  __shared__ __attribute__((aligned(1024))) char ring[NSLOT * STAGE];
  static_assert(2 * ND * 16 * 64 * 4 <= NSLOT * STAGE, "the partial results of two waves fit in the ring");
  const int lane = threadIdx.x & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qt = wave & 1, kh = wave >> 1;
  const int nq = S / 64;
  const int nbh = gridDim.x / nq;
  const int bh = blockIdx.x % nbh;
  const int qb = CAUSAL ? causal_query_block(blockIdx.x / nbh, nq) : blockIdx.x / nbh;
  const int b = bh / nh, head = bh % nh;
  const int ld = 3 * nh * D;
  const bf16* qp = qkv + (size_t)b * S * ld + head * D;
  const bf16* kp = qp + nh * D;
  const bf16* vp = qp + 2 * nh * D;
  const int qw0 = qb * 64 + qt * 32, q = qw0 + (lane & 31);

  DqState<D> st;
  const bf16* dop = d_o + ((size_t)b * S + q) * (nh * D) + head * D;
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++) {
    st.qf[ks] = *(const bf16x8*)(qp + (size_t)q * ld + ks * 16 + hf * 8);
    st.dof[ks] = *(const bf16x8*)(dop + ks * 16 + hf * 8);
  }
#pragma unroll
  for (int dt = 0; dt < ND; dt++)
#pragma unroll
    for (int r = 0; r < 16; r++) st.acc[dt][r] = 0.f;
  st.lse2 = lse[((size_t)b * nh + head) * S + q] * LOG2E;
  st.delta = row_delta<D>(st.dof, o + ((size_t)b * S + q) * (nh * D) + head * D, hf);   // both key halves compute it, one writes
  if (hf == 0 && kh == 0) delta[((size_t)b * nh + head) * S + q] = st.delta;

  uint32_t off[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++) off[i] = tile_src_offset<D>(wave + 4 * i, lane, ld);

  const int ntile = CAUSAL ? qb + 1 : nq, last = ntile - 1;
  const size_t step = (size_t)64 * ld;
  issue_tile<D>(kp, off, ring, wave);
  issue_tile<D>(vp, off, ring + TILEB, wave);
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
  __builtin_amdgcn_s_barrier();
  for (int j = 0; j < ntile; j++) {
    const size_t o2 = (size_t)min(j + 1, last) * step;
    char* fill = ring + ((j + 1) & 1) * STAGE;
    const char* cur = ring + (j & 1) * STAGE;
    issue_tile<D>(kp + o2, off, fill, wave);
    issue_tile<D>(vp + o2, off, fill + TILEB, wave);
    const bool own = CAUSAL && j == last;
    if (!(own && kh > qt)) dq_half_tile<D>(cur, cur + TILEB, st, j * 64 + 32 * kh, kh, q, own && kh == qt, sc2, lane);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
    __builtin_amdgcn_s_barrier();
  }

  float* mg = (float*)ring + (size_t)qt * ND * 16 * 64;
  if (kh == 1) {
#pragma unroll
    for (int dt = 0; dt < ND; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) mg[(dt * 16 + r) * 64 + lane] = st.acc[dt][r];
  }
  __syncthreads();
  if (kh == 1) return;
  bf16* out = dqkv + ((size_t)b * S + q) * ld + head * D;
#pragma unroll
  for (int dt = 0; dt < ND; dt++)
#pragma unroll
    for (int g = 0; g < 4; g++) {
      bf16x4 v;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int r = 4 * g + i;
        v[i] = f2bf((st.acc[dt][r] + mg[(dt * 16 + r) * 64 + lane]) * scale);
      }
      *(bf16x4*)(out + dt * 32 + 8 * g + 4 * hf) = v;
    }
}

// =========================================================================== backward: dK, dV (one block per 128 keys)
template <int D>
struct DkvState {
  bf16x8 kf[D / 16], vf[D / 16];
  f32x16 dk[D / 32], dv[D / 32];
};

// One query tile of 64 for the wave's 32 keys.  Every fragment comes out of LDS, which all four waves
// share and which is the busiest unit of this kernel, so the reads are issued one phase ahead of their
// use (scheduling fences keep the compiler from sinking them back to the point of use): the transposed
// fragments of the second pair of products are requested while the first pair runs and while the
// probabilities are rebuilt, the row-major fragments of the next half while the second pair runs.
template <int D>
__device__ __forceinline__ void dkv_tile(const char* __restrict__ cQ, const char* __restrict__ cO, DkvState<D>& st,
                                         const float* __restrict__ lse_tile, const float* __restrict__ delta_tile, int q0, int key,
                                         bool diag, float sc2, int lane) {
  constexpr int NK = D / 16, ND = D / 32;
  const int hf = lane >> 5;
  const int lim = key - q0 - 4 * hf;  // query offset ql (without the 4*hf term) is masked iff ql < lim
  bf16x8 fq[NK], fo[NK];
#pragma unroll
  for (int ks = 0; ks < NK; ks++) {
    fq[ks] = frag_rowmajor<D>(cQ, lane & 31, ks, hf);
    fo[ks] = frag_rowmajor<D>(cO, lane & 31, ks, hf);
  }
  // delta of the lane's queries (q0 + t*32 + 8g + 4hf + i), read ahead with the fragments: the product dO V^T is
  // accumulated onto -delta, which gives dP - delta without a subtraction per element
  f32x4 dl[2][4];
#pragma unroll
  for (int t = 0; t < 2; t++)
#pragma unroll
    for (int g = 0; g < 4; g++) dl[t][g] = *(const f32x4*)(delta_tile + t * 32 + 8 * g + 4 * hf);
#pragma unroll
  for (int t = 0; t < 2; t++) {
    AH_SCHED_FENCE();
    f32x16 s, dp;
#pragma unroll
    for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = -dl[t][r >> 2][r & 3]; }
    bf16x8 tq0[ND], to0[ND], tq1[ND], to1[ND];
#pragma unroll
    for (int ks = 0; ks < NK; ks++) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[ks], st.kf[ks], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo[ks], st.vf[ks], dp, 0, 0, 0);
    }
#pragma unroll
    for (int dt = 0; dt < ND; dt++) {
      to0[dt] = frag_transposed<D>(cO, t * 32 + 4 * hf, dt, lane);
      tq0[dt] = frag_transposed<D>(cQ, t * 32 + 4 * hf, dt, lane);
    }
    AH_SCHED_FENCE();
    // lane holds queries q0 + t*32 + 8g + 4hf + i of its key
#pragma unroll
    for (int g = 0; g < 4; g++) {
      const int ql = t * 32 + 8 * g + 4 * hf;
      const f32x4 l4 = *(const f32x4*)(lse_tile + ql);
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int r = 4 * g + i;
        s[r] = fexp2(__builtin_fmaf(s[r], sc2, -l4[i] * LOG2E));
      }
    }
    if (diag) {  // wave-uniform: only tiles that straddle the diagonal pay for the mask
#pragma unroll
      for (int r = 0; r < 16; r++)
        if (t * 32 + 8 * (r >> 2) + (r & 3) < lim) s[r] = 0.f;
    }
#pragma unroll
    for (int r = 0; r < 16; r++) dp[r] *= s[r];
    AH_SCHED_FENCE();
    const bf16x8 pf0 = pack8(s, 0), dsf0 = pack8(dp, 0), pf1 = pack8(s, 1), dsf1 = pack8(dp, 1);
#pragma unroll
    for (int dt = 0; dt < ND; dt++) {
      to1[dt] = frag_transposed<D>(cO, t * 32 + 16 + 4 * hf, dt, lane);
      tq1[dt] = frag_transposed<D>(cQ, t * 32 + 16 + 4 * hf, dt, lane);
    }
#pragma unroll
    for (int dt = 0; dt < ND; dt++) {
      st.dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(to0[dt], pf0, st.dv[dt], 0, 0, 0);
      st.dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tq0[dt], dsf0, st.dk[dt], 0, 0, 0);
    }
    AH_SCHED_FENCE();
#pragma unroll
    for (int dt = 0; dt < ND; dt++) {
      st.dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(to1[dt], pf1, st.dv[dt], 0, 0, 0);
      st.dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tq1[dt], dsf1, st.dk[dt], 0, 0, 0);
    }
    if (t == 0) {
#pragma unroll
      for (int ks = 0; ks < NK; ks++) {
        fq[ks] = frag_rowmajor<D>(cQ, 32 + (lane & 31), ks, hf);
        fo[ks] = frag_rowmajor<D>(cO, 32 + (lane & 31), ks, hf);
      }
    }
  }
  AH_SCHED_FENCE();
}

// ring slot of the dK/dV kernel: Q tile, dO tile, then 64 log-sum-exps, 64 deltas and 512 spare bytes
template <int D>
__device__ __forceinline__ void dkv_issue(const bf16* gQ, const bf16* gO, const float* gL, const float* gD, const uint32_t* offq,
                                          const uint32_t* offo, char* __restrict__ slot, int wave, int lane) {
  constexpr int TILEB = 64 * 2 * D;
  issue_tile<D>(gQ, offq, slot, wave);
  issue_tile<D>(gO, offo, slot + TILEB, wave);
  // one 4-byte load per lane: waves 0 and 1 bring the statistics, waves 2 and 3 repeat them into the
  // spare bytes so that every wave has the same number of loads in flight
  const float* src = ((wave & 1) ? gD : gL) + lane;
  __builtin_amdgcn_global_load_lds(src, AH_LDS(slot + 2 * TILEB + wave * 256), 4, 0, 0);
}

template <int D, bool CAUSAL, bool MAY_SKIP>
__device__ __forceinline__ void dkv_step(const bf16* gQ, const bf16* gO, const float* gL, const float* gD, const uint32_t* offq,
                                         const uint32_t* offo, char* __restrict__ fill, const char* __restrict__ cur, DkvState<D>& st,
                                         int q0, int key, int kw0, float sc2, int wave, int lane) {
  constexpr int TILEB = 64 * 2 * D;
  dkv_issue<D>(gQ, gO, gL, gD, offq, offo, fill, wave, lane);
  const float* lse_tile = (const float*)(cur + 2 * TILEB);
  if (CAUSAL && MAY_SKIP && q0 + 63 < kw0) return;  // every query of this tile is before every key of the wave
  // diag: the tile straddles the diagonal of this wave's keys (wave-uniform)
  dkv_tile<D>(cur, cur + TILEB, st, lse_tile, lse_tile + 64, q0, key, CAUSAL && q0 < kw0 + 31, sc2, lane);
}

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_dkv_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ d_o,
                                                       const float* __restrict__ lse, const float* __restrict__ delta,
                                                       bf16* __restrict__ dqkv, int S, int nh, float sc2, float scale) {
  constexpr int TILEB = 64 * 2 * D, STAGE = 2 * TILEB + 1024, LPS = 2 * (D / 32) + 1;
  __shared__ __attribute__((aligned(1024))) char ring[4 * STAGE];
  const int lane = threadIdx.x & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform: LDS bases stay scalar
  const int nbh = gridDim.x / (S / 128);
  const int bh = blockIdx.x % nbh;
  const int kb = blockIdx.x / nbh;  // key block 0 sees every query tile: heaviest first
  const int b = bh / nh, head = bh % nh;
  const int ld = 3 * nh * D, ldo = nh * D;
  const bf16* qp = qkv + (size_t)b * S * ld + head * D;
  const bf16* kp = qp + nh * D;
  const bf16* vp = qp + 2 * nh * D;
  const bf16* dop = d_o + (size_t)b * S * ldo + head * D;
  const int kw0 = kb * 128 + wave * 32, key = kw0 + (lane & 31);
  const float* lse_row = lse + ((size_t)b * nh + head) * S;
  const float* delta_row = delta + ((size_t)b * nh + head) * S;

  DkvState<D> st;
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++) {
    st.kf[ks] = *(const bf16x8*)(kp + (size_t)key * ld + ks * 16 + hf * 8);
    st.vf[ks] = *(const bf16x8*)(vp + (size_t)key * ld + ks * 16 + hf * 8);
  }
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int r = 0; r < 16; r++) { st.dk[dt][r] = 0.f; st.dv[dt][r] = 0.f; }

  uint32_t offq[D / 32], offo[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++) {
    offq[i] = tile_src_offset<D>(wave + 4 * i, lane, ld);
    offo[i] = tile_src_offset<D>(wave + 4 * i, lane, ldo);
  }

  // query tiles of 64 from the diagonal on (from 0 without the mask).  Tile t lives in ring slot t % 4; past the
  // end the last tile is fetched again into a dead slot (uniform number of loads in flight for the counted wait).
  const int j0 = CAUSAL ? 2 * kb : 0, ntile = S / 64 - j0, last = ntile - 1;
  qp += (size_t)j0 * 64 * ld;
  dop += (size_t)j0 * 64 * ldo;
  lse_row += j0 * 64;
  delta_row += j0 * 64;
  const size_t stepq = (size_t)64 * ld, stepo = (size_t)64 * ldo;
#pragma unroll
  for (int t = 0; t < 3; t++) {
    const int tt = min(t, last);
    dkv_issue<D>(qp + tt * stepq, dop + tt * stepo, lse_row + tt * 64, delta_row + tt * 64, offq, offo, ring + t * STAGE, wave, lane);
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(2 * LPS));
  __builtin_amdgcn_s_barrier();
  // Only the block's first tile can lie wholly before a wave's keys (waves 2 and 3 under the mask); it is
  // peeled so that the loop body has a single path and the accumulators stay where the MFMAs want them.
  {
    const int tf = min(3, last);
    dkv_step<D, CAUSAL, true>(qp + tf * stepq, dop + tf * stepo, lse_row + tf * 64, delta_row + tf * 64, offq, offo, ring + 3 * STAGE, ring,
                              st, j0 * 64, key, kw0, sc2, wave, lane);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(2 * LPS));
    __builtin_amdgcn_s_barrier();
  }
  for (int j = 1; j < ntile; j++) {
    const int tf = min(j + 3, last);
    dkv_step<D, CAUSAL, false>(qp + tf * stepq, dop + tf * stepo, lse_row + tf * 64, delta_row + tf * 64, offq, offo,
                               ring + ((j + 3) & 3) * STAGE, ring + (j & 3) * STAGE, st, (j0 + j) * 64, key, kw0, sc2, wave, lane);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(2 * LPS));
    __builtin_amdgcn_s_barrier();
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));  // drain the redundant tail loads

  bf16* outk = dqkv + ((size_t)b * S + key) * ld + nh * D + head * D;
  bf16* outv = outk + nh * D;
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int g = 0; g < 4; g++) {
      bf16x4 a, c;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        a[i] = f2bf(st.dk[dt][4 * g + i] * scale);
        c[i] = f2bf(st.dv[dt][4 * g + i]);
      }
      *(bf16x4*)(outk + dt * 32 + 8 * g + 4 * hf) = a;
      *(bf16x4*)(outv + dt * 32 + 8 * g + 4 * hf) = c;
    }
}

// =========================================================================== backward: dK, dV for launches that cannot fill the chip
// 64 keys per block instead of 128 (twice the blocks, dispatched heaviest first, so that the CUs even out): wave w
// owns keys 32 * (w & 1) .. + 31 of the block and, of every 64-query tile, the queries 32 * (w >> 1) .. + 31; the two
// partial dK, dV per key are added in LDS at the end.
template <int D>
__device__ __forceinline__ void dkv_half_tile(const char* __restrict__ cQ, const char* __restrict__ cO, DkvState<D>& st,
                                              const float* __restrict__ lse_tile, const float* __restrict__ delta_tile, int q0, int key,
                                              int t, bool diag, float sc2, int lane) {
  constexpr int NK = D / 16, ND = D / 32;
  const int hf = lane >> 5;
  const int lim = key - q0 - 4 * hf;  // query offset ql (without the 4*hf term) is masked iff ql < lim
  bf16x8 fq[NK], fo[NK];
#pragma unroll
  for (int ks = 0; ks < NK; ks++) {
    fq[ks] = frag_rowmajor<D>(cQ, 32 * t + (lane & 31), ks, hf);
    fo[ks] = frag_rowmajor<D>(cO, 32 * t + (lane & 31), ks, hf);
  }
  f32x4 dl[4];   // delta of the lane's queries: dO V^T is accumulated onto -delta
#pragma unroll
  for (int g = 0; g < 4; g++) dl[g] = *(const f32x4*)(delta_tile + t * 32 + 8 * g + 4 * hf);
  AH_SCHED_FENCE();
  f32x16 s, dp;
#pragma unroll
  for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = -dl[r >> 2][r & 3]; }
  bf16x8 tq0[ND], to0[ND], tq1[ND], to1[ND];
#pragma unroll
  for (int ks = 0; ks < NK; ks++) {
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[ks], st.kf[ks], s, 0, 0, 0);
    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo[ks], st.vf[ks], dp, 0, 0, 0);
  }
#pragma unroll
  for (int dt = 0; dt < ND; dt++) {
    to0[dt] = frag_transposed<D>(cO, t * 32 + 4 * hf, dt, lane);
    tq0[dt] = frag_transposed<D>(cQ, t * 32 + 4 * hf, dt, lane);
  }
  AH_SCHED_FENCE();
  // lane holds queries q0 + t*32 + 8g + 4hf + i of its key
#pragma unroll
  for (int g = 0; g < 4; g++) {
    const int ql = t * 32 + 8 * g + 4 * hf;
    const f32x4 l4 = *(const f32x4*)(lse_tile + ql);
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int r = 4 * g + i;
      s[r] = fexp2(__builtin_fmaf(s[r], sc2, -l4[i] * LOG2E));
    }
  }
  if (diag) {  // wave-uniform
#pragma unroll
    for (int r = 0; r < 16; r++)
      if (t * 32 + 8 * (r >> 2) + (r & 3) < lim) s[r] = 0.f;
  }
#pragma unroll
  for (int r = 0; r < 16; r++) dp[r] *= s[r];
  AH_SCHED_FENCE();
  const bf16x8 pf0 = pack8(s, 0), dsf0 = pack8(dp, 0), pf1 = pack8(s, 1), dsf1 = pack8(dp, 1);
#pragma unroll
  for (int dt = 0; dt < ND; dt++) {
    to1[dt] = frag_transposed<D>(cO, t * 32 + 16 + 4 * hf, dt, lane);
    tq1[dt] = frag_transposed<D>(cQ, t * 32 + 16 + 4 * hf, dt, lane);
  }
#pragma unroll
  for (int dt = 0; dt < ND; dt++) {
    st.dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(to0[dt], pf0, st.dv[dt], 0, 0, 0);
    st.dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tq0[dt], dsf0, st.dk[dt], 0, 0, 0);
  }
  AH_SCHED_FENCE();
#pragma unroll
  for (int dt = 0; dt < ND; dt++) {
    st.dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(to1[dt], pf1, st.dv[dt], 0, 0, 0);
    st.dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tq1[dt], dsf1, st.dk[dt], 0, 0, 0);
  }
  AH_SCHED_FENCE();
}

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_dkv64_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ d_o,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         bf16* __restrict__ dqkv, int S, int nh, float sc2, float scale) {
  constexpr int TILEB = 64 * 2 * D, STAGE = 2 * TILEB + 1024, LPS = 2 * (D / 32) + 1, ND = D / 32;
  __shared__ __attribute__((aligned(1024))) char ring[4 * STAGE];
  static_assert(2 * 2 * ND * 16 * 64 * 4 <= 4 * STAGE, "the partial results of two waves fit in the ring");
  const int lane = threadIdx.x & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kt = wave & 1, qh = wave >> 1;
  const int nkb = S / 64;
  const int nbh = gridDim.x / nkb;
  const int bh = blockIdx.x % nbh;
  const int kb = blockIdx.x / nbh;  // key block 0 sees every query tile: heaviest first
  const int b = bh / nh, head = bh % nh;
  const int ld = 3 * nh * D, ldo = nh * D;
  const bf16* qp = qkv + (size_t)b * S * ld + head * D;
  const bf16* kp = qp + nh * D;
  const bf16* vp = qp + 2 * nh * D;
  const bf16* dop = d_o + (size_t)b * S * ldo + head * D;
  const int kw0 = kb * 64 + kt * 32, key = kw0 + (lane & 31);
  const float* lse_row = lse + ((size_t)b * nh + head) * S;
  const float* delta_row = delta + ((size_t)b * nh + head) * S;

  DkvState<D> st;
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++) {
    st.kf[ks] = *(const bf16x8*)(kp + (size_t)key * ld + ks * 16 + hf * 8);
    st.vf[ks] = *(const bf16x8*)(vp + (size_t)key * ld + ks * 16 + hf * 8);
  }
#pragma unroll
  for (int dt = 0; dt < ND; dt++)
#pragma unroll
    for (int r = 0; r < 16; r++) { st.dk[dt][r] = 0.f; st.dv[dt][r] = 0.f; }

  uint32_t offq[D / 32], offo[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++) {
    offq[i] = tile_src_offset<D>(wave + 4 * i, lane, ld);
    offo[i] = tile_src_offset<D>(wave + 4 * i, lane, ldo);
  }

  // query tiles of 64 from the one that holds the block's own positions on (from 0 without the mask); ring and
  // counted waits as in attn_dkv_kernel
  const int j0 = CAUSAL ? kb : 0, ntile = S / 64 - j0, last = ntile - 1;
  qp += (size_t)j0 * 64 * ld;
  dop += (size_t)j0 * 64 * ldo;
  lse_row += j0 * 64;
  delta_row += j0 * 64;
  const size_t stepq = (size_t)64 * ld, stepo = (size_t)64 * ldo;
#pragma unroll
  for (int t = 0; t < 3; t++) {
    const int tt = min(t, last);
    dkv_issue<D>(qp + tt * stepq, dop + tt * stepo, lse_row + tt * 64, delta_row + tt * 64, offq, offo, ring + t * STAGE, wave, lane);
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(2 * LPS));
  __builtin_amdgcn_s_barrier();
  for (int j = 0; j < ntile; j++) {
    const int tf = min(j + 3, last);
    dkv_issue<D>(qp + tf * stepq, dop + tf * stepo, lse_row + tf * 64, delta_row + tf * 64, offq, offo, ring + ((j + 3) & 3) * STAGE, wave,
                 lane);
    const char* cur = ring + (j & 3) * STAGE;
    const float* lse_tile = (const float*)(cur + 2 * TILEB);
    // in the block's own tile the wave's queries lie before (qh < kt), on (qh == kt) or after (qh > kt) its keys
    const bool own = CAUSAL && j == 0;
    if (!(own && qh < kt))
      dkv_half_tile<D>(cur, cur + TILEB, st, lse_tile, lse_tile + 64, (j0 + j) * 64, key, qh, own && qh == kt, sc2, lane);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(2 * LPS));
    __builtin_amdgcn_s_barrier();
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));  // drain the redundant tail loads
  __syncthreads();

  float* mg = (float*)ring + (size_t)kt * 2 * ND * 16 * 64;
  if (qh == 1) {
#pragma unroll
    for (int dt = 0; dt < ND; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        mg[(dt * 16 + r) * 64 + lane] = st.dk[dt][r];
        mg[((ND + dt) * 16 + r) * 64 + lane] = st.dv[dt][r];
      }
  }
  __syncthreads();
  if (qh == 1) return;
  bf16* outk = dqkv + ((size_t)b * S + key) * ld + nh * D + head * D;
  bf16* outv = outk + nh * D;
#pragma unroll
  for (int dt = 0; dt < ND; dt++)
#pragma unroll
    for (int g = 0; g < 4; g++) {
      bf16x4 a, c;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int r = 4 * g + i;
        a[i] = f2bf((st.dk[dt][r] + mg[(dt * 16 + r) * 64 + lane]) * scale);
        c[i] = f2bf(st.dv[dt][r] + mg[((ND + dt) * 16 + r) * 64 + lane]);
      }
      *(bf16x4*)(outk + dt * 32 + 8 * g + 4 * hf) = a;
      *(bf16x4*)(outv + dt * 32 + 8 * g + 4 * hf) = c;
    }
}

}  // namespace

// Launches of at most this many 128-row blocks (one per CU) take the 64-row kernels, which split every block's work
// between wave pairs: twice the blocks, so that the CUs even out under the causal mask and a SIMD has two waves
// (gpt1p3b stage, 1 x 16 heads x 2048: forward 48 -> 36 us, backward 144 -> 114 us); larger launches fill the chip
// with 128-row blocks and are 8 % faster with them.
static int small_grid_blocks() {
  static const int v = getenv("AH_ATTN_SMALL_GRID") ? atoi(getenv("AH_ATTN_SMALL_GRID")) : 256;  // tuning aid
  return v;
}

static bool attn_shape_ok(int B, int S, int nh, int d) { return B > 0 && nh > 0 && S > 0 && S % 128 == 0 && (d == 64 || d == 128); }

template <int D, bool CAUSAL>
static void launch_fwd_t(dim3 grid, hipStream_t s, const void* qkv, void* o, float* lse, int S, int nh, float sc2) {
  if ((int)grid.x <= small_grid_blocks())  // at most one 128-query block per CU: 64-query blocks with the keys split between wave pairs
    hipLaunchKernelGGL((attn_fwd64_kernel<D, CAUSAL>), dim3(2 * grid.x), dim3(256), 0, s, (const bf16*)qkv, (bf16*)o, lse, S, nh, sc2);
  else
    hipLaunchKernelGGL((attn_fwd_kernel<D, CAUSAL>), grid, dim3(256), 0, s, (const bf16*)qkv, (bf16*)o, lse, S, nh, sc2);
}

hipError_t launch_attention_fwd(const void* qkv, void* o, float* lse, int B, int S, int nh, int d, bool causal, hipStream_t s) {
  if (!attn_shape_ok(B, S, nh, d)) return hipErrorInvalidValue;
  const float sc2 = LOG2E / sqrtf((float)d);
  const dim3 grid(B * nh * (S / 128));
  if (d == 128) {
    if (causal) launch_fwd_t<128, true>(grid, s, qkv, o, lse, S, nh, sc2);
    else launch_fwd_t<128, false>(grid, s, qkv, o, lse, S, nh, sc2);
  } else {
    if (causal) launch_fwd_t<64, true>(grid, s, qkv, o, lse, S, nh, sc2);
    else launch_fwd_t<64, false>(grid, s, qkv, o, lse, S, nh, sc2);
  }
  return hipGetLastError();
}

// dQ first: it leaves the row sums delta = rowsum(dO * O) of its queries behind for the dK/dV kernel
template <int D, bool CAUSAL>
static void launch_bwd_t(dim3 grid, hipStream_t s, const void* qkv, const void* o, const float* lse, const void* d_o,
                         void* dqkv, float* delta, int S, int nh, float sc2, float scale) {
  if ((int)grid.x <= small_grid_blocks())  // at most one 128-query block per CU: 64-query blocks with the keys split between wave pairs
    hipLaunchKernelGGL((attn_dq64_kernel<D, CAUSAL>), dim3(2 * grid.x), dim3(256), 0, s, (const bf16*)qkv, (const bf16*)o, (const bf16*)d_o, lse,
                       delta, (bf16*)dqkv, S, nh, sc2, scale);
  else
    hipLaunchKernelGGL((attn_dq_kernel<D, CAUSAL>), grid, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)o, (const bf16*)d_o, lse, delta,
                       (bf16*)dqkv, S, nh, sc2, scale);
  if ((int)grid.x <= small_grid_blocks())  // at most one 128-key block per CU: 64-key blocks with the queries split between wave pairs
    hipLaunchKernelGGL((attn_dkv64_kernel<D, CAUSAL>), dim3(2 * grid.x), dim3(256), 0, s, (const bf16*)qkv, (const bf16*)d_o, lse, delta,
                       (bf16*)dqkv, S, nh, sc2, scale);
  else
    hipLaunchKernelGGL((attn_dkv_kernel<D, CAUSAL>), grid, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)d_o, lse, delta, (bf16*)dqkv,
                       S, nh, sc2, scale);
}

hipError_t launch_attention_bwd(const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv, float* delta,
                                int B, int S, int nh, int d, bool causal, hipStream_t s) {
  if (!attn_shape_ok(B, S, nh, d)) return hipErrorInvalidValue;
  const float scale = 1.f / sqrtf((float)d), sc2 = LOG2E * scale;
  const dim3 grid(B * nh * (S / 128));
  if (d == 128) {
    if (causal) launch_bwd_t<128, true>(grid, s, qkv, o, lse, d_o, dqkv, delta, S, nh, sc2, scale);
    else launch_bwd_t<128, false>(grid, s, qkv, o, lse, d_o, dqkv, delta, S, nh, sc2, scale);
  } else {
    if (causal) launch_bwd_t<64, true>(grid, s, qkv, o, lse, d_o, dqkv, delta, S, nh, sc2, scale);
    else launch_bwd_t<64, false>(grid, s, qkv, o, lse, d_o, dqkv, delta, S, nh, sc2, scale);
  }
  return hipGetLastError();
}

}  // namespace ah
