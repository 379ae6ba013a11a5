// dst[t][:] = c[seq(t)] * src[t][:], rounded to the storage type.  Scaling the narrower of X and Delta
// by the per-sequence coefficients turns the weighted contraction dW = Delta^T diag(c_tok) X
// (`grad += advantages[i] * scale_i * seq_logprob_grad`) into the unweighted streaming one; bound by HBM.
#include "common.h"
#include "kernels.h"

namespace isopo {
namespace {

template <bool BF16>
__global__ __launch_bounds__(256) void scale_rows_kernel(const void* __restrict__ src, long long n_tokens, int d,
                                                         const int32_t* __restrict__ off, int n_seq,
                                                         const float* __restrict__ c, void* __restrict__ dst) {
  constexpr int kV = BF16 ? 8 : 4;
  const int vpr = d / kV;
  const long long n_vec = n_tokens * vpr;
  for (long long vi = (long long)blockIdx.x * blockDim.x + threadIdx.x; vi < n_vec;
       vi += (long long)gridDim.x * blockDim.x) {
    const int t = (int)(vi / vpr);
    int lo = 0, hi = n_seq;                       // largest i with off[i] <= t
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (off[mid] <= t) lo = mid; else hi = mid;
    }
    const float s = c[lo];
    uint4 v = reinterpret_cast<const uint4*>(src)[vi];
    if constexpr (BF16) {
      v = scale_bf16x8(v, s);
    } else {
      float4 f = __builtin_bit_cast(float4, v);
      f.x *= s; f.y *= s; f.z *= s; f.w *= s;
      v = __builtin_bit_cast(uint4, f);
    }
    reinterpret_cast<uint4*>(dst)[vi] = v;
  }
}

}  // namespace

hipError_t launch_scale_rows(const void* src, bool bf16, long long n_tokens, int d, const int32_t* off, int n_seq,
                             const float* c, void* dst, hipStream_t s) {
  const long long n_vec = n_tokens * (d / (bf16 ? 8 : 4));
  if (n_vec <= 0) return hipSuccess;
  long long blocks = (n_vec + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (bf16)
    hipLaunchKernelGGL((scale_rows_kernel<true>), dim3((unsigned)blocks), dim3(256), 0, s, src, n_tokens, d, off, n_seq,
                       c, dst);
  else
    hipLaunchKernelGGL((scale_rows_kernel<false>), dim3((unsigned)blocks), dim3(256), 0, s, src, n_tokens, d, off,
                       n_seq, c, dst);
  return hipGetLastError();
}

}  // namespace isopo
