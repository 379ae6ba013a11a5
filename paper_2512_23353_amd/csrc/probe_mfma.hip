// Diagnostic, not a step of the method: the rate the matrix cores sustain when they do nothing but multiply.
// One wave per SIMD (256 workgroups of 256 threads), 256 accumulator registers per lane, eight + eight
// operand fragments held in registers, no memory traffic inside the loop.  The benchmark times it on random
// and on all-zero operands for both bf16 MFMA shapes: the ceiling a contraction kernel of this register shape
// can reach on this board at its power limit, which is what the contraction's rate is to be read against.
#include "common.h"
#include "kernels.h"

namespace isopo {
namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// SHAPE 32: v_mfma_f32_32x32x16_bf16, 4 x 4 blocks, two K halves per trip; SHAPE 16: v_mfma_f32_16x16x32_bf16,
// 8 x 8 blocks.  Either way a trip is 2 * 128 * 128 * 32 flop per wave.
template <int SHAPE>
__global__ __launch_bounds__(256) void mfma_loop_kernel(const u32x4* __restrict__ operands, float* __restrict__ sink,
                                                        int iters) {
  const size_t tid = (size_t)blockIdx.x * 256 + threadIdx.x;
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = __builtin_bit_cast(bf16x8, operands[tid * 16 + i]);
    b[i] = __builtin_bit_cast(bf16x8, operands[tid * 16 + 8 + i]);
  }
  float s = 0.f;
  if constexpr (SHAPE == 32) {
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i + 4 * h], b[j + 4 * h], acc[i][j], 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][j][v];
  } else {
    f32x4 acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) s += acc[i][j][v];
  }
  sink[tid] = s;       // keeps the loop alive
}

}  // namespace

hipError_t launch_mfma_loop(int shape, const void* operands, float* sink, int iters, hipStream_t s) {
  if (shape == 32)
    hipLaunchKernelGGL(mfma_loop_kernel<32>, dim3(kProbeWorkgroups), dim3(256), 0, s,
                       static_cast<const u32x4*>(operands), sink, iters);
  else if (shape == 16)
    hipLaunchKernelGGL(mfma_loop_kernel<16>, dim3(kProbeWorkgroups), dim3(256), 0, s,
                       static_cast<const u32x4*>(operands), sink, iters);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace isopo
