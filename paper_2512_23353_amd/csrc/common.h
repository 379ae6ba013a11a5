// Device-side helpers shared by the gfx950 kernels of the ISOPO layer step.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace isopo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kWave = 64;
constexpr int kXcds = 8;   // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

// Workgroups are dispatched to the XCDs round-robin by linear id.  This maps a
// linear id to a work index so that each XCD (and its private L2) walks one
// contiguous range of the work list.  Bijective for any n.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned b, unsigned n) {
  const unsigned q = n / kXcds, r = n % kXcds;
  const unsigned x = b % kXcds, idx = b / kXcds;
  return x * q + (x < r ? x : r) + idx;
}

// fp32 accumulator tile of a 32x32 MFMA: element v of lane l is
//   row = 8*(v/4) + 4*(l/32) + v%4,  col = l%32.
__device__ __forceinline__ int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

__device__ __forceinline__ float bf16_bits_to_f32(unsigned short b) {
  return __builtin_bit_cast(float, (unsigned)b << 16);
}

// Round-to-nearest-even fp32 -> bf16 bits (NaN kept quiet).
__device__ __forceinline__ unsigned short f32_to_bf16_bits(float f) {
  return __builtin_bit_cast(unsigned short, (__bf16)f);
}

// 8 bf16 packed in a uint4, each multiplied by s in fp32 and rounded back.
__device__ __forceinline__ uint4 scale_bf16x8(uint4 v, float s) {
  unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = __builtin_bit_cast(float, w[i] << 16) * s;
    const float hi = __builtin_bit_cast(float, w[i] & 0xffff0000u) * s;
    w[i] = (unsigned)f32_to_bf16_bits(lo) | ((unsigned)f32_to_bf16_bits(hi) << 16);
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}

}  // namespace isopo
