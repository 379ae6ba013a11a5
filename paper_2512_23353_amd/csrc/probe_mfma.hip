// Diagnostics, not steps of the method.  First: the rate the matrix cores sustain when they do nothing but multiply.
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

// Second diagnostic: the rate at which one workgroup streams global memory into LDS with the DMA loads the
// contraction kernels use (16 bytes per lane, 1 KiB per wave instruction), as a function of how many waves
// issue them.  A ring of STAGES stages of 32 KiB, refilled without a pause: before stage k + STAGES - 1 is
// requested every wave waits until its part of stage k has arrived, and the workgroup meets (what a consumer
// of stage k would need).  Workgroup b reads the (b mod 8)-th eighth of the buffer, round and round, so a
// buffer of 16 MiB stays in the eight L2s.  Nothing is computed; sink keeps the stores alive.
typedef void __attribute__((address_space(3)))* lds_void_ptr;

__device__ __forceinline__ void probe_load_lds16(const void* gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(gptr) : "memory");
}

template <int STAGES, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void lds_dma_ring_kernel(const char* __restrict__ buf, size_t span, int iters,
                                                                  float* __restrict__ sink) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr int kStage = 32768, LPW = kStage / 1024 / WAVES;      // wave-loads per wave and stage
  const unsigned base = (unsigned)(size_t)(lds_void_ptr)smem;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const char* src = buf + (size_t)(blockIdx.x & 7) * span;
  const size_t off = ((size_t)(blockIdx.x >> 3) * kStage) % span;
  auto issue = [&](int k) {
#pragma unroll
    for (int q = 0; q < LPW; ++q) {
      const size_t o = (off + (size_t)k * kStage + (size_t)(wave * LPW + q) * 1024 + (size_t)lane * 16) % span;
      probe_load_lds16(src + o, base + (unsigned)((k % STAGES) * kStage + (wave * LPW + q) * 1024));
    }
  };
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s) issue(s);
  for (int k = 0; k < iters; ++k) {
    constexpr int allowed = (STAGES - 2) * LPW;
    __builtin_amdgcn_s_waitcnt(0x0f70 | (allowed & 15) | ((allowed >> 4) << 14));
    __builtin_amdgcn_s_barrier();
    issue(k + STAGES - 1);
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = *reinterpret_cast<const float*>(smem);
}

template <int STAGES, int WAVES>
hipError_t launch_lds_dma_ring_t(const void* buf, size_t span, int workgroups, int iters, float* sink, hipStream_t s) {
  auto kern = lds_dma_ring_kernel<STAGES, WAVES>;
  constexpr int smem = STAGES * 32768;
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3(workgroups), dim3(64 * WAVES), smem, s, static_cast<const char*>(buf), span, iters, sink);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_lds_dma_ring(const void* buf, size_t bytes, int waves, int stages, int workgroups, int iters,
                               float* sink, hipStream_t s) {
  const size_t span = bytes / 8;                 // one eighth per XCD; the caller has checked the sizes
  if (stages == 2) {
    if (waves == 2) return launch_lds_dma_ring_t<2, 2>(buf, span, workgroups, iters, sink, s);
    if (waves == 4) return launch_lds_dma_ring_t<2, 4>(buf, span, workgroups, iters, sink, s);
    if (waves == 8) return launch_lds_dma_ring_t<2, 8>(buf, span, workgroups, iters, sink, s);
    if (waves == 16) return launch_lds_dma_ring_t<2, 16>(buf, span, workgroups, iters, sink, s);
  } else if (stages == 4) {
    if (waves == 2) return launch_lds_dma_ring_t<4, 2>(buf, span, workgroups, iters, sink, s);
    if (waves == 4) return launch_lds_dma_ring_t<4, 4>(buf, span, workgroups, iters, sink, s);
    if (waves == 8) return launch_lds_dma_ring_t<4, 8>(buf, span, workgroups, iters, sink, s);
    if (waves == 16) return launch_lds_dma_ring_t<4, 16>(buf, span, workgroups, iters, sink, s);
  }
  return hipErrorInvalidValue;
}

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
