// Shared device helpers for the gfx950 kernels of the stage library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ah {

typedef __bf16 bf16;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define AH_LDS(p) ((__attribute__((address_space(3))) void*)(p))

// 16 bytes per lane, global memory straight into LDS: lane i of the wave lands
// at lds_base + 16*i (lds_base must be wave-uniform).
__device__ __forceinline__ void load16_to_lds(const void* gsrc, void* lds_base) {
  __builtin_amdgcn_global_load_lds(gsrc, AH_LDS(lds_base), 16, 0, 0);
}

// Transposing LDS read: within each group of 16 lanes, lane j supplies the
// address of 4 consecutive 16-bit elements; lane i receives element (i % 4) of
// the data addressed by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4.  With lane j
// pointing at row j/4, columns 4*(j%4).. of a row-major block, lane i ends up
// with 4 consecutive rows of column i.
__device__ __forceinline__ bf16x4 lds_read_tr4(const void* p) {
  s16x4 t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
  return __builtin_bit_cast(bf16x4, t);
}

__device__ __forceinline__ bf16x8 cat4(bf16x4 a, bf16x4 b) {
  return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ float bf2f(bf16 v) { return (float)v; }
__device__ __forceinline__ bf16 f2bf(float v) { return (bf16)v; }  // round to nearest even

// tanh-form GeLU written through the logistic function: with z = kappa (u + 0.044715 u^3),
// 0.5 (1 + tanh z) = sigma(2 z), so gelu(u) = u sigma(2z) and
// gelu'(u) = sigma(2z) (1 + 2 u (1 - sigma(2z)) kappa (1 + 0.134145 u^2)).
// sigma uses the hardware exp2 and reciprocal (1 ulp each); exp2 overflow gives sigma = 0 exactly.
#define AH_KAPPA 0.7978845608028654f
__device__ __forceinline__ float sigmoid2z(float u) {
  const float z2 = (2.0f * AH_KAPPA) * __builtin_fmaf(0.044715f * u * u, u, u);
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z2));
}
__device__ __forceinline__ float gelu_f(float u) { return u * sigmoid2z(u); }
__device__ __forceinline__ float gelu_grad_f(float u) {
  const float s = sigmoid2z(u);
  return s * __builtin_fmaf(2.0f * u * (1.0f - s), AH_KAPPA * __builtin_fmaf(0.134145f, u * u, 1.0f), 1.0f);
}

// silu(x) = x sigma(x) through the hardware exp2 and reciprocal
__device__ __forceinline__ float silu_f(float x) {
  return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}

// s_waitcnt immediate (gfx9 encoding): vmcnt = n (6 bits, split), lgkmcnt = 0, expcnt untouched
constexpr int waitcnt_vm_lgkm0(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

}  // namespace ah
