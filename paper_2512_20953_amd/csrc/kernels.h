// Internal launch interface between the stage orchestration and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ah {

enum GemmLayout { GEMM_NN = 0, GEMM_NT = 1, GEMM_TN = 2 };
enum GemmEpilogue {
  EPI_BF16 = 0,      // C = acc (+ bias[n])
  EPI_GELU = 1,      // C = u = acc + bias[n];  C2 = gelu(u)
  EPI_RESID = 2,     // C = acc (+ bias[n]) + aux[m, n]
  EPI_GELU_BWD = 3,  // C = acc * gelu'(aux[m, n])
  EPI_F32_ACC = 4,   // C (fp32) = beta * C + acc  (callers use this one; beta selects the kernel)
  EPI_F32_SET = 5,   // C (fp32) = acc            (internal: EPI_F32_ACC with beta == 0)
  EPI_RESID_F32 = 6,        // C (fp32) = acc (+ bias[n]) + aux[m, n] (fp32): the residual stream kept in fp32
  EPI_RESID_F32_OUT16 = 7,  // C (bf16) = acc (+ bias[n]) + aux[m, n] (fp32): the last layer's output
  // NN only, B = [K, 2F] holding gate | up: the launch's N is 2F, every tile pairs gate columns with their up
  // columns; C[M, 2F] (ldc) = gate | up as bf16 (kept for backward), C2[M, F] (ldc2) = silu(gate) * up taken from
  // the fp32 accumulators.  No bias.  F = swiglu_F, a multiple of 128.
  EPI_SWIGLU = 8,
  // NT only, the input gradient of the SwiGLU block's second matrix with the activation's backward fused: with
  // dm = acc [M, F] and aux = gate | up [M, 2F] (ld_aux), C[M, 2F] (ldc) = dm up silu'(gate) | dm silu(gate).
  // N = F = swiglu_F; dm itself is not stored.
  EPI_SWIGLU_BWD = 9,
  // NN only, no bias: C = acc with the rotary embedding applied to columns [0, rope_cols) on the fp32 sums (heads of
  // rope_d columns, pairs (i, i + rope_d / 2), position = row % rope_S, table rope_cs[pos][i] = (cos, sin)).  Every
  // tile's wave strip must hold whole heads: gemm_min_wave_cols(M, N) % rope_d == 0.
  EPI_ROPE = 10
};

constexpr int kMaxGemmSegments = 16;

struct GemmArgs {
  const void* A;     // NN/NT: [M, K] row-major;  TN: [K, M] row-major
  const void* B;     // NN/TN: [K, N] row-major;  NT: [N, K] row-major
  void* C;           // [M, N]
  void* C2;          // EPI_GELU second output
  const void* bias;  // [N] bf16 or NULL
  const void* aux;   // [M, N] bf16 (residual, or the pre-activation for EPI_GELU_BWD); fp32 for the _F32 residual epilogues
  int lda, ldb, ldc, ld_aux;
  int ldc2, swiglu_F;  // EPI_SWIGLU, EPI_SWIGLU_BWD
  const float* rope_cs;  // EPI_ROPE only
  int rope_S, rope_d, rope_cols;
  int M, N, K;
  int beta;
  int group, xcd_remap;  // tile rasterisation (set by launch_gemm)
  // TN only: the k axis may be the concatenation of n_seg pieces of seg_k rows each (K = n_seg * seg_k), piece i
  // of A starting at segA[i] and of B at segB[i] (same leading dimensions).  n_seg == 0: one piece, A and B.
  int seg_k, n_seg;
  // EPI_GELU_BWD only, optional: column sums of the (bf16-rounded) output over each slab of 64 rows are written
  // to colsum_part[m / 64][n] (leading dimension ld_colsum), for the bias gradient.  Needs M % 64 == 0 (it is).
  float* colsum_part;
  int ld_colsum, colsum_acc;  // colsum_acc != 0: added to what is there
  const void* segA[kMaxGemmSegments];
  const void* segB[kMaxGemmSegments];
};

// M, N, K multiples of 128, all leading dimensions multiples of 8.
hipError_t launch_gemm(GemmLayout layout, GemmEpilogue epi, const GemmArgs& a, hipStream_t s);
bool gemm_shape_ok(int M, int N, int K);
int gemm_min_wave_cols(int M, int N, GemmLayout layout);  // columns of a wave's sub-tile, the smallest over the launches that cover the output
int gemm_tile_area(int M, int N, GemmLayout layout);  // rows x columns of the tile launch_gemm would pick for an M x N output
bool gemm_segments_ok(int seg_k, int n_seg);  // seg_k a positive multiple of 128, 1 <= n_seg <= kMaxGemmSegments

// ---- attention (d = 64 or 128, S multiple of 128) ----
// causal: query i attends to keys 0..i of its sequence; otherwise to all S keys
hipError_t launch_attention_fwd(const void* qkv, void* o, float* lse, int B, int S, int nh, int d, bool causal, hipStream_t s);
hipError_t launch_attention_bwd(const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv,
                                float* delta, int B, int S, int nh, int d, bool causal, hipStream_t s);

// ---- row-wise / element-wise kernels (bf16 I/O, fp32 math) ----
// a = norm(x) * gamma (+ beta); stats[2*T] = (mean, rstd) per row (RMS: mean slot unused = 0)
// x_f32: x is fp32 (the residual stream kept in fp32) instead of bf16
hipError_t launch_norm_fwd(bool rms, const void* x, const void* gamma, const void* beta, void* a, float* stats,
                           int T, int h, float eps, hipStream_t s, bool x_f32 = false);
// dx = dres + norm_bwd(da);  partial column sums of (da*xhat, da, dres) go to `part` ([3][nblk][h] fp32),
// written, or with acc != 0 added to what is there (a group of micro-batches sharing one set of partial sums)
hipError_t launch_norm_bwd(bool rms, const void* da, const void* x, const float* stats, const void* gamma,
                           const void* dres, void* dx, float* part, int T, int h, hipStream_t s, int acc = 0, bool x_f32 = false);
int norm_bwd_blocks(int T);
// g[c] = beta * g[c] + sum_b part[b][c]
hipError_t launch_colsum_finish(const float* part, int nblk, int n, float* g, int beta, hipStream_t s);
// the three partial arrays a norm backward leaves in `part` -> three gradient vectors in one launch
hipError_t launch_colsum_finish3(const float* part, int nblk, int n, float* g0, float* g1, float* g2, int beta, hipStream_t s);
// partial column sums of a bf16 matrix [T, n] -> part[nblk][n] (acc != 0: added to what is there)
hipError_t launch_colsum_partial(const void* m, int T, int n, int ld, float* part, hipStream_t s, int acc = 0);
int colsum_blocks(int T);
// rotary embedding in place on the Q and K blocks of qkv[T, 3*nh*d]; sign = +1 forward, -1 backward
hipError_t launch_rope(void* qkv, const float* cos_sin, int T, int S, int nh, int d, float sign, hipStream_t s);
// device-to-device copy of a multiple of 16 bytes
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
// n bf16 values (a multiple of 8) -> fp32
hipError_t launch_widen(void* dst_f32, const void* src_bf16, size_t n, hipStream_t s);

}  // namespace ah
