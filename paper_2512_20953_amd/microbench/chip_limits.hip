// Two ceilings of one MI355X that bound every kernel of the stage library, measured rather than quoted:
//   1. the rate of a register-resident MFMA 32x32x16 bf16 loop (no memory traffic at all) on zero,
//      constant and random operands: the board's power limit makes the matrix rate depend on how many
//      operand bits toggle, so random data -- what a training step multiplies -- runs well below the
//      2.5 PFLOP/s that zero data reaches;
//   2. the rate at which a CU's LDS serves wave-wide reads (16-byte reads, transposing 8-byte reads):
//      the operands of an LDS-fed GEMM tile pass through this pipe.
// Prints a markdown table.  Every access is in bounds of its own buffers; kernels take no input sizes.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

constexpr int NSET = 3;  // operand sets cycled through, so that consecutive MFMAs see different data

// src: [NSET][8][256] fragments of 16 bytes (4 A-side and 4 B-side per set), one per thread
__global__ __launch_bounds__(256) void mfma_loop(const bf16x8* __restrict__ src, float* __restrict__ out, int iters) {
  bf16x8 f[NSET][8];
#pragma unroll
  for (int s = 0; s < NSET; s++)
#pragma unroll
    for (int i = 0; i < 8; i++) f[s][i] = src[(s * 8 + i) * 256 + threadIdx.x];
  f32x16 acc[16];
#pragma unroll
  for (int i = 0; i < 16; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) acc[i][r] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int s = 0; s < NSET; s++)
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++)
          acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[s][i], f[s][4 + j], acc[i * 4 + j], 0, 0, 0);
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 16; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) t += acc[i][r];
  out[blockIdx.x * 256 + threadIdx.x] = t;
}

// KIND 0: 16-byte reads, lane i at byte 16 i; KIND 1: transposing 8-byte reads in the pattern of a k-strided GEMM tile
template <int KIND>
__global__ __launch_bounds__(512) void lds_loop(int* out, int iters) {
  __shared__ __attribute__((aligned(1024))) char lds[65536];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < 65536 / 4; i += blockDim.x) ((int*)lds)[i] = i;
  __syncthreads();
  const char* p;
  if (KIND == 0) {
    p = lds + (wave & 3) * 1024 + lane * 16;  // < 4 KB
  } else {
    const int k = (lane >> 5) * 8 + ((lane & 15) >> 2), c = (wave & 1) * 128 + ((lane >> 4) & 1) * 16 + 4 * (lane & 3);
    p = lds + k * 512 + (((c >> 5) ^ (k & 3)) << 6) + ((c * 2) & 63);  // < 8.5 KB
  }
  int s0 = 0, s1 = 0;
  for (int it = 0; it < iters; it++) {
    asm volatile("" : "+v"(p));
#pragma unroll
    for (int t = 0; t < 16; t++) {
      const int off = (t % 12) * 4096;  // <= 45056: every address stays below 54 KB
      if (KIND == 0) {
        i32x4 v = *(const i32x4*)(p + off);
        s0 ^= v[0] ^ v[2];
        s1 ^= v[1] ^ v[3];
      } else {
        s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + off));
        s0 ^= v[0];
        s1 ^= v[2];
      }
    }
  }
  out[blockIdx.x * blockDim.x + threadIdx.x] = s0 ^ s1;
}

static unsigned short to_bf16(float x) {
  unsigned u;
  memcpy(&u, &x, 4);
  u += 0x7fff + ((u >> 16) & 1);
  return (unsigned short)(u >> 16);
}

int main() {
  hipDeviceProp_t prop;
  CK(hipGetDeviceProperties(&prop, 0));
  const int ncu = prop.multiProcessorCount;
  printf("device: %s, %d CUs\n\n", prop.gcnArchName, ncu);
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));

  // ---- 1. MFMA loop
  const int iters = 4096, reps = 120;
  const size_t n = (size_t)NSET * 8 * 256 * 8;
  std::vector<unsigned short> h(n);
  unsigned short* d;
  float* o;
  CK(hipMalloc(&d, n * 2));
  CK(hipMalloc(&o, (size_t)ncu * 256 * 4));
  std::mt19937 rng(20953);
  std::normal_distribution<float> N01(0.f, 1.f);
  const char* names[] = {"zero", "constant (1.0 x 0.02)", "random N(0,1) x N(0,0.02)"};
  printf("| MFMA 32x32x16 bf16, registers only, one wave per SIMD | ms per launch | PFLOP/s | %% of 2.5 |\n|---|---|---|---|\n");
  for (int mode = 0; mode < 3; mode++) {
    for (int s = 0; s < NSET; s++)
      for (int i = 0; i < 8; i++)
        for (int t = 0; t < 256 * 8; t++) {
          float v = 0.f;
          if (mode == 1) v = i < 4 ? 1.0f : 0.02f;
          if (mode == 2) v = N01(rng) * (i < 4 ? 1.0f : 0.02f);
          h[((size_t)s * 8 + i) * 2048 + t] = to_bf16(v);
        }
    CK(hipMemcpy(d, h.data(), n * 2, hipMemcpyHostToDevice));
    double sum = 0;
    for (int r = 0; r < reps; r++) {
      CK(hipEventRecord(e0, 0));
      mfma_loop<<<ncu, 256>>>((const bf16x8*)d, o, iters);
      CK(hipEventRecord(e1, 0));
      CK(hipEventSynchronize(e1));
      float ms;
      CK(hipEventElapsedTime(&ms, e0, e1));
      if (r >= reps / 2) sum += ms;  // steady state: the board has settled at its power limit
    }
    CK(hipGetLastError());
    const double ms = sum / (reps - reps / 2);
    const double pf = (double)ncu * 4 * iters * NSET * 16 * 32768.0 / ms * 1e-12;
    printf("| %s | %.3f | %.3f | %.1f |\n", names[mode], ms, pf, pf / 2.5 * 100);
    fflush(stdout);
  }

  // ---- 2. LDS reads
  int* oi;
  CK(hipMalloc(&oi, (size_t)ncu * 512 * 4));
  printf("\n| LDS read, 8 waves per CU, 16 in flight per wave | ns per wave instruction per CU | GB/s per CU | bytes per clock at 2.4 GHz |\n|---|---|---|---|\n");
  for (int kind = 0; kind < 2; kind++) {
    const int it2 = 10000;
    auto launch = [&](int its) {
      if (kind == 0) lds_loop<0><<<ncu, 512>>>(oi, its);
      else lds_loop<1><<<ncu, 512>>>(oi, its);
    };
    launch(100);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0, 0));
    launch(it2);
    CK(hipEventRecord(e1, 0));
    CK(hipEventSynchronize(e1));
    CK(hipGetLastError());
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double ninstr = 16.0 * it2 * 8, bytes = kind == 0 ? 1024 : 512;
    printf("| %s | %.2f | %.0f | %.0f |\n", kind == 0 ? "ds_read_b128 (1 KB per instruction)" : "ds_read_b64_tr_b16 (512 B per instruction)",
           ms * 1e6 / ninstr, ninstr * bytes / ms * 1e-6, ninstr * bytes / ms * 1e-6 / 2.4);
    fflush(stdout);
  }
  return 0;
}
