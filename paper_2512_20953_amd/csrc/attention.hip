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
// Backward is two deterministic kernels (no atomics): one block per 128 keys
// accumulates dK and dV over the query tiles at or after it, one block per 128
// queries accumulates dQ over the key tiles at or before it (causal; without the
// mask both walk every tile of the sequence).
#include "common.h"
#include "kernels.h"

namespace ah {
namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr int NSLOT = 2;  // ring slots of the forward and dQ kernels (two blocks share a CU)

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

// =========================================================================== forward
template <int D>
struct FwdState {
  bf16x8 qf[D / 16];
  f32x16 oacc[D / 32];
  float m, l;
};

template <int D, bool CAUSAL>
__device__ __forceinline__ void fwd_tile(const char* __restrict__ cK, const char* __restrict__ cV, FwdState<D>& st, int k0,
                                         int q, int qw0, float sc2, int lane) {
  const int hf = lane >> 5;
  if (CAUSAL && k0 > qw0 + 31) return;  // every key of this tile is after every query of the wave
  f32x16 s[2];
#pragma unroll
  for (int t = 0; t < 2; t++) {
#pragma unroll
    for (int r = 0; r < 16; r++) s[t][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++)
      s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rowmajor<D>(cK, t * 32 + (lane & 31), ks, hf), st.qf[ks], s[t], 0, 0, 0);
  }
  const bool diag = CAUSAL && k0 + 63 > qw0;
  float mx = -INFINITY;
#pragma unroll
  for (int t = 0; t < 2; t++)
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int key = k0 + t * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
      float v = s[t][r] * sc2;
      if (diag && key > q) v = -INFINITY;
      s[t][r] = v;
      mx = fmaxf(mx, v);
    }
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  const float m_new = fmaxf(st.m, mx);
  const float alpha = fexp2(st.m - m_new);
  st.m = m_new;
  float ls = 0.f;
#pragma unroll
  for (int t = 0; t < 2; t++)
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const float p = fexp2(s[t][r] - m_new);
      s[t][r] = p;
      ls += p;
    }
  st.l = st.l * alpha + ls;
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int r = 0; r < 16; r++) st.oacc[dt][r] *= alpha;
#pragma unroll
  for (int t = 0; t < 2; t++)
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++) {
      const bf16x8 pf = pack8(s[t], s2);
#pragma unroll
      for (int dt = 0; dt < D / 32; dt++)
        st.oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_transposed<D>(cV, t * 32 + 16 * s2 + 4 * hf, dt, lane), pf,
                                                             st.oacc[dt], 0, 0, 0);
    }
}

template <int D, bool CAUSAL>
__device__ __forceinline__ void fwd_step(const bf16* gK, const bf16* gV, const uint32_t* off, char* __restrict__ nK,
                                         char* __restrict__ nV, const char* __restrict__ cK, const char* __restrict__ cV,
                                         FwdState<D>& st, int k0, int q, int qw0, float sc2, int wave, int lane) {
  issue_tile<D>(gK, off, nK, wave);
  issue_tile<D>(gV, off, nV, wave);
  fwd_tile<D, CAUSAL>(cK, cV, st, k0, q, qw0, sc2, lane);
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
  const int qb = S / 128 - 1 - blockIdx.x / nbh;  // heaviest query blocks first
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
  for (int j = 0; j < ntile; j++) {
    const size_t o = (size_t)min(j + NSLOT - 1, last) * step;
    char* fill = ring + ((j + NSLOT - 1) & (NSLOT - 1)) * STAGE;
    const char* cur = ring + (j & (NSLOT - 1)) * STAGE;
    fwd_step<D, CAUSAL>(kp + o, vp + o, off, fill, fill + TILEB, cur, cur + TILEB, st, j * 64, q, qw0, sc2, wave, lane);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NSLOT - 2) * LPS));
    __builtin_amdgcn_s_barrier();
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

// =========================================================================== backward: delta = rowsum(dO * O)
template <int D>
__global__ __launch_bounds__(256) void attn_delta_kernel(const bf16* __restrict__ o, const bf16* __restrict__ d_o,
                                                         float* __restrict__ delta, int T, int S, int nh) {
  constexpr int LPR = D / 8;  // lanes per (token, head)
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  const long row = idx / LPR;  // token * nh + head
  const int piece = idx % LPR;
  float s = 0.f;
  if (row < (long)T * nh) {
    bf16x8 a = *(const bf16x8*)(o + row * D + piece * 8), b = *(const bf16x8*)(d_o + row * D + piece * 8);
#pragma unroll
    for (int j = 0; j < 8; j++) s += bf2f(a[j]) * bf2f(b[j]);
  }
#pragma unroll
  for (int w = LPR / 2; w > 0; w >>= 1) s += __shfl_xor(s, w, 64);
  if (piece == 0 && row < (long)T * nh) {
    const long t = row / nh;
    const int head = row % nh;
    delta[((t / S) * nh + head) * S + (t % S)] = s;
  }
}

// =========================================================================== backward: dQ (one block per 128 queries)
template <int D>
struct DqState {
  bf16x8 qf[D / 16], dof[D / 16];
  f32x16 acc[D / 32];
  float lse2, delta;
};

template <int D, bool CAUSAL>
__device__ __forceinline__ void dq_tile(const char* __restrict__ cK, const char* __restrict__ cV, DqState<D>& st, int k0, int q,
                                        int qw0, float sc2, int lane) {
  const int hf = lane >> 5;
  if (CAUSAL && k0 > qw0 + 31) return;
  const bool diag = CAUSAL && k0 + 63 > qw0;
#pragma unroll
  for (int t = 0; t < 2; t++) {
    f32x16 s, dp;
#pragma unroll
    for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
    const int row = t * 32 + (lane & 31);
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rowmajor<D>(cK, row, ks, hf), st.qf[ks], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rowmajor<D>(cV, row, ks, hf), st.dof[ks], dp, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int key = k0 + t * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
      float p = fexp2(s[r] * sc2 - st.lse2);
      if (diag && key > q) p = 0.f;
      s[r] = p * (dp[r] - st.delta);  // dS^T
    }
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++) {
      const bf16x8 dsf = pack8(s, s2);
#pragma unroll
      for (int dt = 0; dt < D / 32; dt++)
        st.acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_transposed<D>(cK, t * 32 + 16 * s2 + 4 * hf, dt, lane), dsf,
                                                            st.acc[dt], 0, 0, 0);
    }
  }
}

template <int D, bool CAUSAL>
__device__ __forceinline__ void dq_step(const bf16* gK, const bf16* gV, const uint32_t* off, char* __restrict__ nK,
                                        char* __restrict__ nV, const char* __restrict__ cK, const char* __restrict__ cV,
                                        DqState<D>& st, int k0, int q, int qw0, float sc2, int wave, int lane) {
  issue_tile<D>(gK, off, nK, wave);
  issue_tile<D>(gV, off, nV, wave);
  dq_tile<D, CAUSAL>(cK, cV, st, k0, q, qw0, sc2, lane);
}

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void attn_dq_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ d_o,
                                                      const float* __restrict__ lse, const float* __restrict__ delta,
                                                      bf16* __restrict__ dqkv, int S, int nh, float sc2, float scale) {
  constexpr int TILEB = 64 * 2 * D, STAGE = 2 * TILEB, LPS = 2 * (D / 32);  // ring slot = K tile then V tile
  __shared__ __attribute__((aligned(1024))) char ring[NSLOT * STAGE];
  const int lane = threadIdx.x & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform: LDS bases stay scalar
  const int nbh = gridDim.x / (S / 128);
  const int bh = blockIdx.x % nbh;
  const int qb = S / 128 - 1 - blockIdx.x / nbh;
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
  st.delta = delta[((size_t)b * nh + head) * S + q];

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
  for (int j = 0; j < ntile; j++) {
    const size_t o = (size_t)min(j + NSLOT - 1, last) * step;
    char* fill = ring + ((j + NSLOT - 1) & (NSLOT - 1)) * STAGE;
    const char* cur = ring + (j & (NSLOT - 1)) * STAGE;
    dq_step<D, CAUSAL>(kp + o, vp + o, off, fill, fill + TILEB, cur, cur + TILEB, st, j * 64, q, qw0, sc2, wave, lane);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NSLOT - 2) * LPS));
    __builtin_amdgcn_s_barrier();
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

// =========================================================================== backward: dK, dV (one block per 128 keys)
template <int D>
struct DkvState {
  bf16x8 kf[D / 16], vf[D / 16];
  f32x16 dk[D / 32], dv[D / 32];
};

template <int D, bool CAUSAL>
__device__ __forceinline__ void dkv_tile(const char* __restrict__ cQ, const char* __restrict__ cO, DkvState<D>& st,
                                         const float* __restrict__ lse_tile, const float* __restrict__ delta_tile, int q0, int key,
                                         int kw0, float sc2, int lane) {
  const int hf = lane >> 5;
  if (CAUSAL && q0 + 63 < kw0) return;  // every query of this tile is before every key of the wave
  const bool diag = CAUSAL && q0 < kw0 + 31;
#pragma unroll
  for (int t = 0; t < 2; t++) {
    f32x16 s, dp;
#pragma unroll
    for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
    const int row = t * 32 + (lane & 31);
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rowmajor<D>(cQ, row, ks, hf), st.kf[ks], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rowmajor<D>(cO, row, ks, hf), st.vf[ks], dp, 0, 0, 0);
    }
    // lane holds queries q0 + t*32 + 8g + 4hf + i of its key
#pragma unroll
    for (int g = 0; g < 4; g++) {
      const int ql = t * 32 + 8 * g + 4 * hf, qq = q0 + ql;
      const f32x4 l4 = *(const f32x4*)(lse_tile + ql);
      const f32x4 d4 = *(const f32x4*)(delta_tile + ql);
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int r = 4 * g + i;
        float p = fexp2(s[r] * sc2 - l4[i] * LOG2E);
        if (diag && key > qq + i) p = 0.f;
        s[r] = p;
        dp[r] = p * (dp[r] - d4[i]);
      }
    }
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++) {
      const bf16x8 pf = pack8(s, s2), dsf = pack8(dp, s2);
      const int rbase = t * 32 + 16 * s2 + 4 * hf;
#pragma unroll
      for (int dt = 0; dt < D / 32; dt++) {
        st.dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_transposed<D>(cO, rbase, dt, lane), pf, st.dv[dt], 0, 0, 0);
        st.dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_transposed<D>(cQ, rbase, dt, lane), dsf, st.dk[dt], 0, 0, 0);
      }
    }
  }
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

template <int D, bool CAUSAL>
__device__ __forceinline__ void dkv_step(const bf16* gQ, const bf16* gO, const float* gL, const float* gD, const uint32_t* offq,
                                         const uint32_t* offo, char* __restrict__ fill, const char* __restrict__ cur, DkvState<D>& st,
                                         int q0, int key, int kw0, float sc2, int wave, int lane) {
  constexpr int TILEB = 64 * 2 * D;
  dkv_issue<D>(gQ, gO, gL, gD, offq, offo, fill, wave, lane);
  dkv_tile<D, CAUSAL>(cur, cur + TILEB, st, (const float*)(cur + 2 * TILEB), (const float*)(cur + 2 * TILEB + 256), q0, key, kw0, sc2, lane);
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
  for (int j = 0; j < ntile; j++) {
    const int tf = min(j + 3, last);
    dkv_step<D, CAUSAL>(qp + tf * stepq, dop + tf * stepo, lse_row + tf * 64, delta_row + tf * 64, offq, offo, ring + ((j + 3) & 3) * STAGE,
                ring + (j & 3) * STAGE, st, (j0 + j) * 64, key, kw0, sc2, wave, lane);
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

}  // namespace

static bool attn_shape_ok(int B, int S, int nh, int d) { return B > 0 && nh > 0 && S > 0 && S % 128 == 0 && (d == 64 || d == 128); }

template <int D, bool CAUSAL>
static void launch_fwd_t(dim3 grid, hipStream_t s, const void* qkv, void* o, float* lse, int S, int nh, float sc2) {
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

template <int D, bool CAUSAL>
static void launch_bwd_t(dim3 grid, dim3 dgrid, hipStream_t s, const void* qkv, const void* o, const float* lse, const void* d_o,
                         void* dqkv, float* delta, int T, int S, int nh, float sc2, float scale) {
  hipLaunchKernelGGL(attn_delta_kernel<D>, dgrid, dim3(256), 0, s, (const bf16*)o, (const bf16*)d_o, delta, T, S, nh);
  hipLaunchKernelGGL((attn_dkv_kernel<D, CAUSAL>), grid, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)d_o, lse, delta, (bf16*)dqkv,
                     S, nh, sc2, scale);
  hipLaunchKernelGGL((attn_dq_kernel<D, CAUSAL>), grid, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)d_o, lse, delta, (bf16*)dqkv,
                     S, nh, sc2, scale);
}

hipError_t launch_attention_bwd(const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv, float* delta,
                                int B, int S, int nh, int d, bool causal, hipStream_t s) {
  if (!attn_shape_ok(B, S, nh, d)) return hipErrorInvalidValue;
  const float scale = 1.f / sqrtf((float)d), sc2 = LOG2E * scale;
  const int T = B * S;
  const dim3 grid(B * nh * (S / 128));
  const long nthreads = (long)T * nh * (d / 8);
  const dim3 dgrid((unsigned)((nthreads + 255) / 256));
  if (d == 128) {
    if (causal) launch_bwd_t<128, true>(grid, dgrid, s, qkv, o, lse, d_o, dqkv, delta, T, S, nh, sc2, scale);
    else launch_bwd_t<128, false>(grid, dgrid, s, qkv, o, lse, d_o, dqkv, delta, T, S, nh, sc2, scale);
  } else {
    if (causal) launch_bwd_t<64, true>(grid, dgrid, s, qkv, o, lse, d_o, dqkv, delta, T, S, nh, sc2, scale);
    else launch_bwd_t<64, false>(grid, dgrid, s, qkv, o, lse, d_o, dqkv, delta, T, S, nh, sc2, scale);
  }
  return hipGetLastError();
}

}  // namespace ah
