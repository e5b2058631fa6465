// C ABI: single-GEMM entry points (declared in include/ah_stage.h).
#include "ah_stage.h"
#include "capi_util.h"
#include "kernels.h"

using namespace ah;

static const char* kShapeMsg = "M, N, K must be positive multiples of 128";

extern "C" int ah_gemm_nn(const void* A, const void* B, const void* bias, void* C, int M, int N, int K, void* stream) {
  discard_stale_hip_error();
  if (!A || !B || !C) return set_error(AH_EINVAL, "ah_gemm_nn: NULL pointer");
  if (!gemm_shape_ok(M, N, K)) return set_error(AH_EUNSUPPORTED, "ah_gemm_nn: %s", kShapeMsg);
  GemmArgs g = {};
  g.A = A; g.B = B; g.C = C; g.bias = bias;
  g.lda = K; g.ldb = N; g.ldc = N; g.M = M; g.N = N; g.K = K;
  return hip_status(launch_gemm(GEMM_NN, EPI_BF16, g, (hipStream_t)stream), "ah_gemm_nn");
}

extern "C" int ah_gemm_nn_swiglu(const void* A, const void* B, void* U, void* Mout, int M, int F, int K, void* stream) {
  discard_stale_hip_error();
  if (!A || !B || !U || !Mout) return set_error(AH_EINVAL, "ah_gemm_nn_swiglu: NULL pointer");
  if (F <= 0 || F > (1 << 29) || !gemm_shape_ok(M, 2 * F, K) || F % 128) return set_error(AH_EUNSUPPORTED, "ah_gemm_nn_swiglu: M, F, K must be positive multiples of 128");
  GemmArgs g = {};
  g.A = A; g.B = B; g.C = U; g.C2 = Mout;
  g.lda = K; g.ldb = 2 * F; g.ldc = 2 * F; g.ldc2 = F; g.swiglu_F = F; g.M = M; g.N = 2 * F; g.K = K;
  return hip_status(launch_gemm(GEMM_NN, EPI_SWIGLU, g, (hipStream_t)stream), "ah_gemm_nn_swiglu");
}

extern "C" int ah_gemm_nt(const void* A, const void* B, void* C, int M, int N, int K, void* stream) {
  discard_stale_hip_error();
  if (!A || !B || !C) return set_error(AH_EINVAL, "ah_gemm_nt: NULL pointer");
  if (!gemm_shape_ok(M, N, K)) return set_error(AH_EUNSUPPORTED, "ah_gemm_nt: %s", kShapeMsg);
  GemmArgs g = {};
  g.A = A; g.B = B; g.C = C;
  g.lda = K; g.ldb = K; g.ldc = N; g.M = M; g.N = N; g.K = K;
  return hip_status(launch_gemm(GEMM_NT, EPI_BF16, g, (hipStream_t)stream), "ah_gemm_nt");
}

extern "C" int ah_gemm_tn(const void* A, const void* B, float* C, int M, int N, int K, int beta, void* stream) {
  discard_stale_hip_error();
  if (!A || !B || !C) return set_error(AH_EINVAL, "ah_gemm_tn: NULL pointer");
  if (beta != 0 && beta != 1) return set_error(AH_EINVAL, "ah_gemm_tn: beta must be 0 or 1");
  if (!gemm_shape_ok(M, N, K)) return set_error(AH_EUNSUPPORTED, "ah_gemm_tn: %s", kShapeMsg);
  GemmArgs g = {};
  g.A = A; g.B = B; g.C = C;
  g.lda = M; g.ldb = N; g.ldc = N; g.M = M; g.N = N; g.K = K; g.beta = beta;
  return hip_status(launch_gemm(GEMM_TN, EPI_F32_ACC, g, (hipStream_t)stream), "ah_gemm_tn");
}

extern "C" int ah_gemm_tn_segmented(const void* const* A_seg, const void* const* B_seg, int n_seg, float* C, int M, int N, int seg_k,
                                    int beta, void* stream) {
  discard_stale_hip_error();
  if (!A_seg || !B_seg || !C) return set_error(AH_EINVAL, "ah_gemm_tn_segmented: NULL pointer");
  if (beta != 0 && beta != 1) return set_error(AH_EINVAL, "ah_gemm_tn_segmented: beta must be 0 or 1");
  if (!gemm_segments_ok(seg_k, n_seg)) return set_error(AH_EUNSUPPORTED, "ah_gemm_tn_segmented: need 1 <= n_seg <= %d pieces of seg_k %% 128 == 0 rows", kMaxGemmSegments);
  if (!gemm_shape_ok(M, N, seg_k * n_seg)) return set_error(AH_EUNSUPPORTED, "ah_gemm_tn_segmented: %s", kShapeMsg);
  GemmArgs g = {};
  for (int i = 0; i < n_seg; i++) {
    if (!A_seg[i] || !B_seg[i]) return set_error(AH_EINVAL, "ah_gemm_tn_segmented: piece %d is NULL", i);
    g.segA[i] = A_seg[i];
    g.segB[i] = B_seg[i];
  }
  g.A = A_seg[0]; g.B = B_seg[0]; g.C = C;
  g.seg_k = seg_k; g.n_seg = n_seg;
  g.lda = M; g.ldb = N; g.ldc = N; g.M = M; g.N = N; g.K = seg_k * n_seg; g.beta = beta;
  return hip_status(launch_gemm(GEMM_TN, EPI_F32_ACC, g, (hipStream_t)stream), "ah_gemm_tn_segmented");
}
