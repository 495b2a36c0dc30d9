// Matrix-pipe rate probes for bench.py (a separate small library, not part of the C ABI of the layer):
// a loop of independent MFMAs on register operands, two waves per SIMD on every CU.  The achieved rate on
// random operand bits is what the chip sustains under its power limit; on all-zero operands the shader
// clock stays near its maximum.  kind 0: bf16 32x32x16, 1: bf16 16x16x32, 2: fp8 32x32x64.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

template <int KIND>
__global__ __launch_bounds__(512, 1) void mfma_rate_kernel(const uint32_t* __restrict__ seed, float* __restrict__ sink,
                                                           int iters) {
  const int t = threadIdx.x;
  // operand bits from memory (the compiler cannot fold them); finite bf16 / fp8 numbers of moderate size
  uint32_t w[8];
#pragma unroll
  for (int e = 0; e < 8; e++) w[e] = seed[(blockIdx.x * 512 + t) * 8 + e];
  float s = 0.0f;
  if constexpr (KIND == 2) {
    i32x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; e++) {
      a[e] = (int)(w[e] & 0x3F3F3F3Fu);                  // fp8 e4m3 bytes below 2
      b[e] = (int)((w[e] >> 1) & 0x3F3F3F3Fu);
    }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][v] = 0.0f;
    for (int it = 0; it < iters; it++) {
#pragma unroll
      for (int i = 0; i < 4; i++) acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i], 0, 0, 0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; i++) s += acc[i][0];
  } else {
    bf16x8 a, b;
    uint32_t wa[4], wb[4];
#pragma unroll
    for (int e = 0; e < 4; e++) {
      wa[e] = (w[e] & 0x807F807Fu) | 0x3F003F00u;        // bf16 pairs with magnitude in [0.5, 1)
      wb[e] = (w[4 + e] & 0x807F807Fu) | 0x3F003F00u;
      if (w[e] == 0) wa[e] = wb[e] = 0;                   // all-zero seed: all-zero operands
    }
    a = __builtin_bit_cast(bf16x8, wa);
    b = __builtin_bit_cast(bf16x8, wb);
    if constexpr (KIND == 0) {
      f32x16 acc[4];
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int v = 0; v < 16; v++) acc[i][v] = 0.0f;
      for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int i = 0; i < 4; i++) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < 4; i++) s += acc[i][0];
    } else {
      f32x4 acc[8];
#pragma unroll
      for (int i = 0; i < 8; i++)
#pragma unroll
        for (int v = 0; v < 4; v++) acc[i][v] = 0.0f;
      for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int i = 0; i < 8; i++) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < 8; i++) s += acc[i][0];
    }
  }
  sink[blockIdx.x * 512 + t] = s;
}

extern "C" {
// Flops of one launch: blocks * 8 waves * iters * (per-iteration flops of a wave).  seed: blocks * 512 * 8 dwords
// (device), sink: blocks * 512 floats (device).  Returns the flop count, or -1 for an unknown kind.
double dirotq_probe_mfma_rate(int kind, int blocks, int iters, const uint32_t* seed, float* sink, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  const double per_wave_iter = kind == 0 ? 4.0 * 2 * 32 * 32 * 16 : kind == 1 ? 8.0 * 2 * 16 * 16 * 32 : 4.0 * 2 * 32 * 32 * 64;
  if (kind == 0) hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(blocks), dim3(512), 0, s, seed, sink, iters);
  else if (kind == 1) hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(blocks), dim3(512), 0, s, seed, sink, iters);
  else if (kind == 2) hipLaunchKernelGGL(mfma_rate_kernel<2>, dim3(blocks), dim3(512), 0, s, seed, sink, iters);
  else return -1.0;
  if (hipGetLastError() != hipSuccess) return -1.0;
  return (double)blocks * 8.0 * iters * per_wave_iter;
}
}
