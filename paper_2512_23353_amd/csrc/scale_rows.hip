// dst[t][:] = c[seq(t)] * src[t][:], rounded to the storage type.  Scaling the narrower of X and Delta
// by the per-sequence coefficients turns the weighted contraction dW = Delta^T diag(c_tok) X
// (`grad += advantages[i] * scale_i * seq_logprob_grad`) into the unweighted streaming one; bound by HBM.
#include "common.h"
#include "kernels.h"

namespace isopo {
namespace {

// A workgroup takes a contiguous range of token rows: one binary search in the offsets for its first
// row, then every thread walks forward from there (rows and offsets are both ascending), so the
// per-vector cost is one short scan in cached offsets instead of a full search.
template <bool BF16>
__global__ __launch_bounds__(256) void scale_rows_kernel(const void* __restrict__ src, long long n_tokens, int d,
                                                         const int32_t* __restrict__ off, int n_seq,
                                                         const float* __restrict__ c, void* __restrict__ dst,
                                                         int rows_per_wg) {
  constexpr int kV = BF16 ? 8 : 4;
  __shared__ int s_base;
  const int vpr = d / kV;
  for (long long r0 = (long long)blockIdx.x * rows_per_wg; r0 < n_tokens; r0 += (long long)gridDim.x * rows_per_wg) {
    const int rows = (int)(n_tokens - r0 < rows_per_wg ? n_tokens - r0 : rows_per_wg);
    __syncthreads();                              // the previous range's readers are done with s_base
    if (threadIdx.x == 0) {
      const int t = (int)r0;
      int lo = 0, hi = n_seq;                     // largest i with off[i] <= t
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= t) lo = mid; else hi = mid;
      }
      s_base = lo;
    }
    __syncthreads();
    const int base = s_base;
    const uint4* in = reinterpret_cast<const uint4*>(src) + r0 * vpr;
    uint4* out = reinterpret_cast<uint4*>(dst) + r0 * vpr;
    const int n_vec = rows * vpr;
    for (int vi = threadIdx.x; vi < n_vec; vi += 256) {
      const int t = (int)r0 + vi / vpr;
      int seq = base;
      while (seq + 1 < n_seq && off[seq + 1] <= t) ++seq;
      const float sc = c[seq];
      uint4 v = in[vi];
      if constexpr (BF16) {
        v = scale_bf16x8(v, sc);
      } else {
        float4 f = __builtin_bit_cast(float4, v);
        f.x *= sc; f.y *= sc; f.z *= sc; f.w *= sc;
        v = __builtin_bit_cast(uint4, f);
      }
      out[vi] = v;
    }
  }
}

}  // namespace

hipError_t launch_scale_rows(const void* src, bool bf16, long long n_tokens, int d, const int32_t* off, int n_seq,
                             const float* c, void* dst, hipStream_t s) {
  if (n_tokens <= 0) return hipSuccess;
  // about 64 KiB per range
  const long long row_bytes = (long long)d * (bf16 ? 2 : 4);
  int rows_per_wg = (int)(65536 / row_bytes);
  if (rows_per_wg < 1) rows_per_wg = 1;
  long long blocks = (n_tokens + rows_per_wg - 1) / rows_per_wg;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (bf16)
    hipLaunchKernelGGL((scale_rows_kernel<true>), dim3((unsigned)blocks), dim3(256), 0, s, src, n_tokens, d, off, n_seq,
                       c, dst, rows_per_wg);
  else
    hipLaunchKernelGGL((scale_rows_kernel<false>), dim3((unsigned)blocks), dim3(256), 0, s, src, n_tokens, d, off,
                       n_seq, c, dst, rows_per_wg);
  return hipGetLastError();
}

}  // namespace isopo
