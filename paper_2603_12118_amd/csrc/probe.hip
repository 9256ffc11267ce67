// Measurement aid: the rate a bare MFMA loop sustains on this chip, which is what the GEMM's
// roofline fraction is to be read against.  No memory traffic: every wave keeps eight 32x32
// accumulator blocks and feeds them from six operand registers, the same shape of inner loop as
// the GEMM's k-steps.  With zero operands the loop runs at the nominal clock; with random operands
// the board reaches its power limit and the clock drops, which is the regime the encoder runs in.
#include "common.h"

namespace cs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(512) void mfma_loop_kernel(float* out, int iters, int random_operands) {
  unsigned s = threadIdx.x * 2654435761u + blockIdx.x * 97u + 12345u;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      s = s * 1664525u + 1013904223u;
      const float u = random_operands ? (float)((int)(s >> 8) % 2001 - 1000) * 1e-3f : 0.f;
      a[q][i] = (__bf16)u;
      b[q][i] = (__bf16)(u * 0.05f);
    }
  f32x16 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int n = 0; n < 8; ++n)
        acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[(n & 1) + 2 * (ks & 1)], a[n >> 1], acc[n], 0, 0, 0);
  }
  float tot = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) tot += acc[j][r];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = tot;
}

cs_status launch_mfma_loop(float* out, int blocks, int iters, int random_operands, hipStream_t stream) {
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(blocks), dim3(512), 0, stream, out, iters, random_operands);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

}  // namespace cs
