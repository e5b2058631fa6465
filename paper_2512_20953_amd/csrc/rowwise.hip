// Row-wise and element-wise kernels of the decoder layer: LayerNorm / RMSNorm
// forward and backward (fused with the residual add and the column sums that
// give the gains', offsets' and biases' gradients), column sums, rotary
// embedding.  All are bound by HBM bandwidth: every tensor is read and
// written once, 16 bytes per lane, statistics and sums in fp32.
#include "common.h"
#include "kernels.h"
#include <cstdlib>

namespace ah {

namespace {

constexpr int NT = 256;      // threads per block
// MAXC (template): 16-byte chunks per thread per row, ceil(hidden / 2048), at most 8 (hidden <= 16384)

__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();  // red may still be read from the previous call
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// Eight consecutive values of a tensor of the residual stream, which is bf16 or (residual_fp32) fp32.
template <bool F32> struct XVec;
template <> struct XVec<false> {
  bf16x8 v;
  __device__ __forceinline__ void load(const void* base, size_t elem) { v = *(const bf16x8*)((const bf16*)base + elem); }
  __device__ __forceinline__ float get(int j) const { return bf2f(v[j]); }
};
template <> struct XVec<true> {
  f32x4 a, b;
  __device__ __forceinline__ void load(const void* base, size_t elem) {
    a = *(const f32x4*)((const float*)base + elem);
    b = *(const f32x4*)((const float*)base + elem + 4);
  }
  __device__ __forceinline__ float get(int j) const { return j < 4 ? a[j] : b[j - 4]; }
};

// ---------------------------------------------------------------- norm forward: one block per row
template <bool RMS, int MAXC, bool XF32>
__global__ __launch_bounds__(NT) void norm_fwd_kernel(const void* __restrict__ x, const bf16* __restrict__ gamma,
                                                      const bf16* __restrict__ beta, bf16* __restrict__ a,
                                                      float* __restrict__ stats, int h, float eps) {
  __shared__ float red[8];
  const int row = blockIdx.x, nchunk = h >> 3;
  float v[MAXC][8];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < MAXC; i++) {
    const int c = threadIdx.x + i * NT;
    if (c < nchunk) {
      XVec<XF32> t;
      t.load(x, (size_t)row * h + c * 8);
#pragma unroll
      for (int j = 0; j < 8; j++) { v[i][j] = t.get(j); s += RMS ? v[i][j] * v[i][j] : v[i][j]; }
    }
  }
  float mean = 0.f, rstd;
  if (RMS) {
    rstd = rsqrtf(block_sum(s, red) / h + eps);
  } else {
    mean = block_sum(s, red) / h;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; i++)
      if (threadIdx.x + i * NT < nchunk)
#pragma unroll
        for (int j = 0; j < 8; j++) { float d = v[i][j] - mean; q += d * d; }
    rstd = rsqrtf(block_sum(q, red) / h + eps);
  }
  if (threadIdx.x == 0) { stats[2 * row] = mean; stats[2 * row + 1] = rstd; }
#pragma unroll
  for (int i = 0; i < MAXC; i++) {
    const int c = threadIdx.x + i * NT;
    if (c < nchunk) {
      bf16x8 g = *(const bf16x8*)(gamma + c * 8), o;
      bf16x8 b;
      if (!RMS) b = *(const bf16x8*)(beta + c * 8);
#pragma unroll
      for (int j = 0; j < 8; j++) {
        float r = (v[i][j] - mean) * rstd * bf2f(g[j]);
        if (!RMS) r += bf2f(b[j]);
        o[j] = f2bf(r);
      }
      *(bf16x8*)(a + (size_t)row * h + c * 8) = o;
    }
  }
}

// ---------------------------------------------------------------- norm forward, rows up to 8192 wide: one wave per row
// A wave keeps a whole row in registers (MAXI chunks of 8 values per lane), so both statistics are wave
// reductions with no block barrier, and it walks rows w, w + (waves in the grid), ... with the next row's loads
// issued before the current one is reduced: loads, arithmetic and stores of different rows overlap inside a wave
// as well as across the waves of a CU.  The gain and offset stay packed in registers for all rows.
template <bool RMS, int MAXI, bool XF32>
__global__ __launch_bounds__(NT) void norm_fwd_wave_kernel(const void* __restrict__ x, const bf16* __restrict__ gamma,
                                                           const bf16* __restrict__ beta, bf16* __restrict__ a,
                                                           float* __restrict__ stats, int T, int h, float eps) {
  const int lane = threadIdx.x & 63, nchunk = h >> 3;
  const int nw = gridDim.x * (NT / 64);
  int row = blockIdx.x * (NT / 64) + (threadIdx.x >> 6);
  if (row >= T) return;
  const float inv_h = 1.f / h;
  bf16x8 gam[MAXI], bet[RMS ? 1 : MAXI];
  XVec<XF32> cur[MAXI], nxt[MAXI];
#pragma unroll
  for (int i = 0; i < MAXI; i++) {
    const int c = lane + 64 * i;
    if (c < nchunk) {
      gam[i] = *(const bf16x8*)(gamma + c * 8);
      if (!RMS) bet[i] = *(const bf16x8*)(beta + c * 8);
      cur[i].load(x, (size_t)row * h + c * 8);
    }
  }
  for (; row < T; row += nw) {
    const int nr = row + nw;
    if (nr < T) {
#pragma unroll
      for (int i = 0; i < MAXI; i++)
        if (lane + 64 * i < nchunk) nxt[i].load(x, (size_t)nr * h + (lane + 64 * i) * 8);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MAXI; i++)
      if (lane + 64 * i < nchunk)
#pragma unroll
        for (int j = 0; j < 8; j++) { const float v = cur[i].get(j); s += RMS ? v * v : v; }
    s = wave_sum(s);
    float mean = 0.f, rstd;
    if (RMS) {
      rstd = rsqrtf(s * inv_h + eps);
    } else {
      mean = s * inv_h;
      float q = 0.f;
#pragma unroll
      for (int i = 0; i < MAXI; i++)
        if (lane + 64 * i < nchunk)
#pragma unroll
          for (int j = 0; j < 8; j++) { const float d = cur[i].get(j) - mean; q += d * d; }
      rstd = rsqrtf(wave_sum(q) * inv_h + eps);
    }
    if (lane == 0) { stats[2 * row] = mean; stats[2 * row + 1] = rstd; }
#pragma unroll
    for (int i = 0; i < MAXI; i++) {
      const int c = lane + 64 * i;
      if (c < nchunk) {
        bf16x8 o;
#pragma unroll
        for (int j = 0; j < 8; j++) {
          float r = (cur[i].get(j) - mean) * rstd * bf2f(gam[i][j]);
          if (!RMS) r += bf2f(bet[i][j]);
          o[j] = f2bf(r);
        }
        *(bf16x8*)(a + (size_t)row * h + c * 8) = o;
      }
    }
#pragma unroll
    for (int i = 0; i < MAXI; i++) cur[i] = nxt[i];
  }
}

// ---------------------------------------------------------------- norm backward
// Block b handles rows b, b + nblk, b + 2*nblk, ... (so that the blocks, which advance together, read one
// contiguous stretch of memory at a time and spread over all HBM channels); a thread keeps its columns for
// all of them, so the three column sums accumulate in registers and leave the block once.  512 threads (two waves per
// SIMD), rows in batches of RB; the loads of the next batch are issued before the current one is
// reduced, so that memory latency, the block reduction and the arithmetic overlap.
constexpr int NTB = 512;  // threads per block of the norm backward; MAXC here = ceil(hidden / 4096)

template <bool RMS, int MAXC, bool XF32>
__global__ __launch_bounds__(NTB) void norm_bwd_kernel(const bf16* __restrict__ da, const void* __restrict__ x,
                                                       const float* __restrict__ stats, const bf16* __restrict__ gamma,
                                                       const bf16* __restrict__ dres, bf16* __restrict__ dx,
                                                       float* __restrict__ part, int T, int h, int rpb, int acc) {
  constexpr int RB = MAXC <= 1 ? 2 : 1;  // rows per batch: two keep a 4096-wide row kernel at 125 registers (36.8 us; four rows 39.6, one 38.4)
  constexpr int NWV = NTB / 64;
  constexpr bool PIPE = MAXC <= 2;  // wider rows (hidden > 8192) leave no registers for a second batch, and spill a few
  __shared__ float red[2][NWV][2 * RB];                     // double-buffered: one block barrier per batch
  const int nchunk = h >> 3, nblk = gridDim.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float inv_h = 1.f / h;
  // the gain stays packed (bf16x8 per chunk: a quarter of the registers of a float copy; rows wider than 8192 need the room)
  bf16x8 gam[MAXC];
  float s_g[MAXC][8], s_b[MAXC][8], s_r[MAXC][8];
#pragma unroll
  for (int i = 0; i < MAXC; i++) {
    const int c = threadIdx.x + i * NTB;
    if (c < nchunk) {
      gam[i] = *(const bf16x8*)(gamma + c * 8);
#pragma unroll
      for (int j = 0; j < 8; j++) { s_g[i][j] = 0.f; s_b[i][j] = 0.f; s_r[i][j] = 0.f; }
    }
  }
  // the block's rows are j * nblk + blockIdx.x for j in [r0, r1)
  const int r0 = 0, r1 = (T - (int)blockIdx.x + nblk - 1) / nblk;
  XVec<XF32> tx[RB][MAXC];
  bf16x8 td[RB][MAXC], tr[RB][MAXC];   // current batch
  XVec<XF32> nx[PIPE ? RB : 1][PIPE ? MAXC : 1];
  bf16x8 nd[PIPE ? RB : 1][PIPE ? MAXC : 1], nr[PIPE ? RB : 1][PIPE ? MAXC : 1];  // next batch
  float mean[RB], rstd[RB], nmean[PIPE ? RB : 1], nrstd[PIPE ? RB : 1];
  // a short last batch repeats its last row; the copies are computed but neither summed nor stored
  auto fetch = [&](int rb, auto& fx, auto& fd, auto& fr, auto& fm, auto& fs) {
#pragma unroll
    for (int k = 0; k < RB; k++) {
      const int row = min(rb + k, r1 - 1) * nblk + blockIdx.x;
#pragma unroll
      for (int i = 0; i < MAXC; i++) {
        const int c = threadIdx.x + i * NTB;
        if (c < nchunk) {
          fx[k][i].load(x, (size_t)row * h + c * 8);
          fd[k][i] = *(const bf16x8*)(da + (size_t)row * h + c * 8);
          fr[k][i] = *(const bf16x8*)(dres + (size_t)row * h + c * 8);
        }
      }
      fm[k] = RMS ? 0.f : stats[2 * row];
      fs[k] = stats[2 * row + 1];
    }
  };
  if (PIPE && r0 < r1) fetch(r0, tx, td, tr, mean, rstd);
  int buf = 0;
  for (int rb = r0; rb < r1; rb += RB, buf ^= 1) {
    if constexpr (PIPE) {
      if (rb + RB < r1) fetch(rb + RB, nx, nd, nr, nmean, nrstd);
    } else {
      fetch(rb, tx, td, tr, mean, rstd);
    }
    float sums[2 * RB];
#pragma unroll
    for (int k = 0; k < RB; k++) {
      const bool live = rb + k < r1;
      const float nm = -mean[k] * rstd[k];
      float sw = 0.f, swx = 0.f;
#pragma unroll
      for (int i = 0; i < MAXC; i++) {
        if (threadIdx.x + i * NTB < nchunk) {
#pragma unroll
          for (int j = 0; j < 8; j++) {
            const float d = bf2f(td[k][i][j]);
            const float xh = __builtin_fmaf(tx[k][i].get(j), rstd[k], nm);
            const float w = d * bf2f(gam[i][j]);
            sw += w;
            swx = __builtin_fmaf(w, xh, swx);
            if (live) { s_g[i][j] = __builtin_fmaf(d, xh, s_g[i][j]); s_b[i][j] += d; }
          }
        }
      }
      sums[2 * k] = wave_sum(sw);
      sums[2 * k + 1] = wave_sum(swx);
    }
    if (lane == 0) {
#pragma unroll
      for (int k = 0; k < 2 * RB; k++) red[buf][wave][k] = sums[k];
    }
    __syncthreads();  // the other half of red was last read before the previous barrier
#pragma unroll
    for (int k = 0; k < RB; k++) {
      if (rb + k >= r1) break;
      const int row = (rb + k) * nblk + blockIdx.x;
      float c1 = 0.f, c2 = 0.f;
#pragma unroll
      for (int w8 = 0; w8 < NWV; w8++) { c1 += red[buf][w8][2 * k]; c2 += red[buf][w8][2 * k + 1]; }
      c1 = RMS ? 0.f : c1 * inv_h;
      c2 *= inv_h;
      const float nm = -mean[k] * rstd[k];
#pragma unroll
      for (int i = 0; i < MAXC; i++) {
        const int c = threadIdx.x + i * NTB;
        if (c < nchunk) {
          bf16x8 o;
#pragma unroll
          for (int j = 0; j < 8; j++) {
            const float r = bf2f(tr[k][i][j]);
            const float xh = __builtin_fmaf(tx[k][i].get(j), rstd[k], nm);
            const float w = bf2f(td[k][i][j]) * bf2f(gam[i][j]);
            s_r[i][j] += r;
            o[j] = f2bf(r + rstd[k] * (w - c1 - xh * c2));
          }
          *(bf16x8*)(dx + (size_t)row * h + c * 8) = o;
        }
      }
    }
    if constexpr (PIPE) {
#pragma unroll
      for (int k = 0; k < RB; k++) {
        mean[k] = nmean[k];
        rstd[k] = nrstd[k];
#pragma unroll
        for (int i = 0; i < MAXC; i++) { tx[k][i] = nx[k][i]; td[k][i] = nd[k][i]; tr[k][i] = nr[k][i]; }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < MAXC; i++) {
    const int c = threadIdx.x + i * NTB;
    if (c < nchunk) {
      float* p0 = part + ((size_t)0 * nblk + blockIdx.x) * h + c * 8;
      float* p1 = part + ((size_t)1 * nblk + blockIdx.x) * h + c * 8;
      float* p2 = part + ((size_t)2 * nblk + blockIdx.x) * h + c * 8;
#pragma unroll
      for (int j = 0; j < 8; j++) {
        if (acc) { p0[j] += s_g[i][j]; p1[j] += s_b[i][j]; p2[j] += s_r[i][j]; }  // on top of earlier micro-batches' partial sums
        else { p0[j] = s_g[i][j]; p1[j] = s_b[i][j]; p2[j] = s_r[i][j]; }
      }
    }
  }
}

// ---------------------------------------------------------------- column sums
// Partial sums: grid (ceil(n / 512), nblk).  A wave owns 512 columns (16 bytes per lane, one
// contiguous kilobyte per row) and every fourth row of the block's slab; the four waves' sums
// meet in LDS and leave as one row of part[nblk][n].
constexpr int CS_ROWS = 64;  // rows per block
__global__ __launch_bounds__(NT) void colsum_partial_kernel(const bf16* __restrict__ m, int T, int n, int ld,
                                                            float* __restrict__ part, int acc) {
  __shared__ float red[3][512];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = blockIdx.x * 512 + lane * 8;
  const int r0 = blockIdx.y * CS_ROWS, r1 = min(T, r0 + CS_ROWS);
  float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (col < n) {
#pragma unroll 4
    for (int r = r0 + wave; r < r1; r += 4) {
      bf16x8 t = *(const bf16x8*)(m + (size_t)r * ld + col);
#pragma unroll
      for (int j = 0; j < 8; j++) s[j] += bf2f(t[j]);
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int j = 0; j < 8; j++) red[wave - 1][lane * 8 + j] = s[j];
  }
  __syncthreads();
  if (wave == 0 && col < n) {
    float* p = part + (size_t)blockIdx.y * n + col;
#pragma unroll
    for (int j = 0; j < 8; j++) {
      const float v = s[j] + red[0][lane * 8 + j] + red[1][lane * 8 + j] + red[2][lane * 8 + j];
      p[j] = acc ? p[j] + v : v;
    }
  }
}

// g[c] = beta * g[c] + sum_b part[b][c] for up to three (part, g) pairs that share n and nblk.
// A block takes 64 columns; its four waves each sum a quarter of the partial rows.
struct FinishArgs { const float* part[3]; float* g[3]; };
__global__ __launch_bounds__(NT) void colsum_finish_kernel(FinishArgs a, int nblk, int n, int beta) {
  __shared__ float red[3][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  const float* part = a.part[blockIdx.y];
  float s0 = 0.f, s1 = 0.f;
  if (c < n) {
    int b = wave;
    for (; b + 4 < nblk; b += 8) {
      s0 += part[(size_t)b * n + c];
      s1 += part[(size_t)(b + 4) * n + c];
    }
    if (b < nblk) s0 += part[(size_t)b * n + c];
  }
  if (wave > 0) red[wave - 1][lane] = s0 + s1;
  __syncthreads();
  if (wave == 0 && c < n) {
    const float s = (s0 + s1) + red[0][lane] + red[1][lane] + red[2][lane];
    float* g = a.g[blockIdx.y];
    g[c] = beta ? g[c] + s : s;
  }
}

// ---------------------------------------------------------------- rotary embedding
// thread: one token, one head of Q or K, 8 pairs (i .. i+7, i + d/2 ..)
__global__ __launch_bounds__(NT) void rope_kernel(bf16* __restrict__ qkv, const float* __restrict__ cs, int T, int S, int nh,
                                                  int d, float sign) {
  const int half = d >> 1, per_head = half >> 3;
  const long idx = (long)blockIdx.x * NT + threadIdx.x;
  const long total = (long)T * 2 * nh * per_head;
  if (idx >= total) return;
  const int piece = idx % per_head;
  const int head = (idx / per_head) % (2 * nh);   // heads of Q then heads of K: contiguous in the packed row
  const int t = idx / ((long)per_head * 2 * nh);
  const int pos = t % S;
  bf16* p = qkv + (size_t)t * 3 * nh * d + (size_t)head * d + piece * 8;
  bf16x8 a = *(bf16x8*)p, b = *(bf16x8*)(p + half), oa, ob;
  const float* c = cs + ((size_t)pos * half + piece * 8) * 2;
#pragma unroll
  for (int j = 0; j < 8; j++) {
    const float co = c[2 * j], si = c[2 * j + 1] * sign;
    const float fa = bf2f(a[j]), fb = bf2f(b[j]);
    oa[j] = f2bf(fa * co - fb * si);
    ob[j] = f2bf(fb * co + fa * si);
  }
  *(bf16x8*)p = oa;
  *(bf16x8*)(p + half) = ob;
}

// ---------------------------------------------------------------- plain copy, 16 bytes per lane
__global__ __launch_bounds__(NT) void copy16_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t i = (size_t)blockIdx.x * NT + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

// bf16 -> fp32, 8 elements per lane (the stage input entering an fp32 residual stream)
__global__ __launch_bounds__(NT) void widen_kernel(const bf16* __restrict__ src, float* __restrict__ dst, size_t n8) {
  const size_t i = (size_t)blockIdx.x * NT + threadIdx.x;
  if (i >= n8) return;
  const bf16x8 t = *(const bf16x8*)(src + i * 8);
  *(f32x4*)(dst + i * 8) = f32x4{bf2f(t[0]), bf2f(t[1]), bf2f(t[2]), bf2f(t[3])};
  *(f32x4*)(dst + i * 8 + 4) = f32x4{bf2f(t[4]), bf2f(t[5]), bf2f(t[6]), bf2f(t[7])};
}

}  // namespace

namespace {
// one wave per row; MAXI = chunks of 8 values per lane
template <bool RMS, int MAXI>
void norm_fwd_wave_go(const void* x, bool x_f32, const void* gamma, const void* beta, void* a, float* stats, int T, int h, float eps, hipStream_t s) {
  // two rows per wave where the rows suffice (the second row's loads run under the first row's arithmetic), at most 8 waves per CU
  const int waves = T >= 4096 ? 2048 : (T + 1) / 2 > 0 ? (T + 1) / 2 : 1;
  const dim3 grid((waves + NT / 64 - 1) / (NT / 64));
  if (x_f32)
    hipLaunchKernelGGL((norm_fwd_wave_kernel<RMS, MAXI, true>), grid, dim3(NT), 0, s, x, (const bf16*)gamma, (const bf16*)beta, (bf16*)a, stats, T, h, eps);
  else
    hipLaunchKernelGGL((norm_fwd_wave_kernel<RMS, MAXI, false>), grid, dim3(NT), 0, s, x, (const bf16*)gamma, (const bf16*)beta, (bf16*)a, stats, T, h, eps);
}

template <bool RMS, int MAXC>
void norm_fwd_go(const void* x, bool x_f32, const void* gamma, const void* beta, void* a, float* stats, int T, int h, float eps, hipStream_t s) {
  if (x_f32)
    hipLaunchKernelGGL((norm_fwd_kernel<RMS, MAXC, true>), dim3(T), dim3(NT), 0, s, x, (const bf16*)gamma, (const bf16*)beta, (bf16*)a, stats, h, eps);
  else
    hipLaunchKernelGGL((norm_fwd_kernel<RMS, MAXC, false>), dim3(T), dim3(NT), 0, s, x, (const bf16*)gamma, (const bf16*)beta, (bf16*)a, stats, h, eps);
}
template <bool RMS, int MAXC>
void norm_bwd_go(const void* da, const void* x, bool x_f32, const float* stats, const void* gamma, const void* dres, void* dx, float* part,
                 int T, int h, int acc, hipStream_t s) {
  const int nblk = norm_bwd_blocks(T);
  const int rpb = (T + nblk - 1) / nblk;
  if (x_f32)
    hipLaunchKernelGGL((norm_bwd_kernel<RMS, MAXC, true>), dim3(nblk), dim3(NTB), 0, s, (const bf16*)da, x, stats,
                       (const bf16*)gamma, (const bf16*)dres, (bf16*)dx, part, T, h, rpb, acc);
  else
    hipLaunchKernelGGL((norm_bwd_kernel<RMS, MAXC, false>), dim3(nblk), dim3(NTB), 0, s, (const bf16*)da, x, stats,
                       (const bf16*)gamma, (const bf16*)dres, (bf16*)dx, part, T, h, rpb, acc);
}
}  // namespace

int norm_bwd_blocks(int T) {
  static int cap = -1;
  if (cap < 0) cap = getenv("AH_NORM_NBLK") ? atoi(getenv("AH_NORM_NBLK")) : 256;  // tuning aid
  return T / 4 < cap ? (T / 4 > 0 ? T / 4 : 1) : cap;
}

#define AH_BY_CHUNKS(FN, RMS, ...)                                   \
  do {                                                               \
    const int nc = (h + 2047) / 2048;                                \
    if (nc <= 1) FN<RMS, 1>(__VA_ARGS__);                            \
    else if (nc == 2) FN<RMS, 2>(__VA_ARGS__);                       \
    else if (nc == 3) FN<RMS, 3>(__VA_ARGS__);                       \
    else if (nc == 4) FN<RMS, 4>(__VA_ARGS__);                       \
    else FN<RMS, 8>(__VA_ARGS__);                                    \
  } while (0)

hipError_t launch_norm_fwd(bool rms, const void* x, const void* gamma, const void* beta, void* a, float* stats, int T,
                           int h, float eps, hipStream_t s, bool x_f32) {
  if (h % 8 || h > 16384) return hipErrorInvalidValue;
  static int wave_rows = -1;
  if (wave_rows < 0) wave_rows = getenv("AH_NORM_FWD_BLOCK_PER_ROW") ? 0 : 1;  // tuning aid
  const int per_lane = (h / 8 + 63) / 64;   // chunks per lane with one wave per row
  if (wave_rows && per_lane <= 16) {
#define AH_WAVE_ROWS(RMS)                                                                                     \
    do {                                                                                                      \
      if (per_lane <= 2) norm_fwd_wave_go<RMS, 2>(x, x_f32, gamma, beta, a, stats, T, h, eps, s);             \
      else if (per_lane <= 4) norm_fwd_wave_go<RMS, 4>(x, x_f32, gamma, beta, a, stats, T, h, eps, s);        \
      else if (per_lane <= 8) norm_fwd_wave_go<RMS, 8>(x, x_f32, gamma, beta, a, stats, T, h, eps, s);        \
      else if (per_lane <= 12) norm_fwd_wave_go<RMS, 12>(x, x_f32, gamma, beta, a, stats, T, h, eps, s);      \
      else norm_fwd_wave_go<RMS, 16>(x, x_f32, gamma, beta, a, stats, T, h, eps, s);                          \
    } while (0)
    if (rms) AH_WAVE_ROWS(true);
    else AH_WAVE_ROWS(false);
#undef AH_WAVE_ROWS
    return hipGetLastError();
  }
  if (rms) AH_BY_CHUNKS(norm_fwd_go, true, x, x_f32, gamma, beta, a, stats, T, h, eps, s);
  else AH_BY_CHUNKS(norm_fwd_go, false, x, x_f32, gamma, beta, a, stats, T, h, eps, s);
  return hipGetLastError();
}

#define AH_BWD_BY_CHUNKS(RMS)                                                                        \
  do {                                                                                               \
    const int nc = (h + 4095) / 4096;                                                                \
    if (nc <= 1) norm_bwd_go<RMS, 1>(da, x, x_f32, stats, gamma, dres, dx, part, T, h, acc, s);      \
    else if (nc == 2) norm_bwd_go<RMS, 2>(da, x, x_f32, stats, gamma, dres, dx, part, T, h, acc, s); \
    else norm_bwd_go<RMS, 4>(da, x, x_f32, stats, gamma, dres, dx, part, T, h, acc, s);              \
  } while (0)

hipError_t launch_norm_bwd(bool rms, const void* da, const void* x, const float* stats, const void* gamma, const void* dres,
                           void* dx, float* part, int T, int h, hipStream_t s, int acc, bool x_f32) {
  if (h % 8 || h > 16384) return hipErrorInvalidValue;
  if (rms) AH_BWD_BY_CHUNKS(true);
  else AH_BWD_BY_CHUNKS(false);
  return hipGetLastError();
}

hipError_t launch_colsum_finish(const float* part, int nblk, int n, float* g, int beta, hipStream_t s) {
  FinishArgs a = {{part, nullptr, nullptr}, {g, nullptr, nullptr}};
  hipLaunchKernelGGL(colsum_finish_kernel, dim3((n + 63) / 64, 1), dim3(NT), 0, s, a, nblk, n, beta);
  return hipGetLastError();
}

hipError_t launch_colsum_finish3(const float* part, int nblk, int n, float* g0, float* g1, float* g2, int beta, hipStream_t s) {
  FinishArgs a = {{part, part + (size_t)nblk * n, part + (size_t)2 * nblk * n}, {g0, g1, g2}};
  hipLaunchKernelGGL(colsum_finish_kernel, dim3((n + 63) / 64, 3), dim3(NT), 0, s, a, nblk, n, beta);
  return hipGetLastError();
}

int colsum_blocks(int T) { return (T + CS_ROWS - 1) / CS_ROWS; }

hipError_t launch_colsum_partial(const void* m, int T, int n, int ld, float* part, hipStream_t s, int acc) {
  if (n % 8) return hipErrorInvalidValue;
  hipLaunchKernelGGL(colsum_partial_kernel, dim3((n + 511) / 512, colsum_blocks(T)), dim3(NT), 0, s, (const bf16*)m, T, n, ld, part, acc);
  return hipGetLastError();
}

hipError_t launch_rope(void* qkv, const float* cos_sin, int T, int S, int nh, int d, float sign, hipStream_t s) {
  const long total = (long)T * 2 * nh * (d / 16);
  hipLaunchKernelGGL(rope_kernel, dim3((unsigned)((total + NT - 1) / NT)), dim3(NT), 0, s, (bf16*)qkv, cos_sin, T, S, nh, d, sign);
  return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
  if (bytes % 16) return hipErrorInvalidValue;
  const size_t n16 = bytes / 16;
  hipLaunchKernelGGL(copy16_kernel, dim3((unsigned)((n16 + NT - 1) / NT)), dim3(NT), 0, s, (const uint4*)src, (uint4*)dst, n16);
  return hipGetLastError();
}

hipError_t launch_widen(void* dst_f32, const void* src_bf16, size_t n, hipStream_t s) {
  if (n % 8) return hipErrorInvalidValue;
  const size_t n8 = n / 8;
  hipLaunchKernelGGL(widen_kernel, dim3((unsigned)((n8 + NT - 1) / NT)), dim3(NT), 0, s, (const bf16*)src_bf16, (float*)dst_f32, n8);
  return hipGetLastError();
}

}  // namespace ah
