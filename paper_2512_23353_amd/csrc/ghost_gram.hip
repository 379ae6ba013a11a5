// Ghost form of the layer's Gram matrix.  Each token gradient is the rank-one
// matrix delta_t x_t^T (efficient-implementation paragraph), so
//     <g^(t), g^(s)> = (x_t . x_s)(delta_t . delta_s)
// (its t = s case is eq. (two)), and summing over the tokens of two sequences
//     K_ij = sum_{t in i} sum_{s in j} (x_t . x_s)(delta_t . delta_s)
// without ever forming a per-sequence gradient.
//
// One workgroup takes a 64x64 block of token pairs (bt <= bs); each of its four
// waves forms a 32x32 block of P = X X^T and Q = Delta Delta^T on the matrix
// cores (here the reduction index is the fast index of both operands, so
// fragments are plain 16-byte loads), multiplies them element-wise in
// registers and reduces the products by (sequence of t, sequence of s).  Only
// token pairs t <= s are used; a pair t < s inside one sequence counts twice.
// Segment sums go to an fp64 upper-triangular accumulator with atomics (the
// accumulation order varies from run to run, but in fp64, so that the fp32 K
// changes by at most one rounding of the final conversion).
#include "common.h"
#include "kernels.h"

namespace isopo {
namespace {

__global__ void token_seq_kernel(const int32_t* __restrict__ off, int n_seq, int n_tokens,
                                 int32_t* __restrict__ tok_seq) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_tokens) return;
  int lo = 0, hi = n_seq;   // largest i with off[i] <= t (empty sequences are skipped by the <=)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off[mid] <= t) lo = mid; else hi = mid;
  }
  tok_seq[t] = lo;
}

__global__ void fill_f64_kernel(double* p, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.0;
}

template <bool BF16>
__device__ __forceinline__ void gram_block(const void* __restrict__ M, int d, int t_row, int s_row, bool t_ok,
                                           bool s_ok, int half, f32x16& acc) {
  constexpr int kV = BF16 ? 8 : 4;
  constexpr int kEs = BF16 ? 2 : 4;
  const char* a = static_cast<const char*>(M) + (size_t)t_row * d * kEs;
  const char* b = static_cast<const char*>(M) + (size_t)s_row * d * kEs;
  // The trip count is the same for every lane: an MFMA must be issued by the whole wave.
  for (int k0 = 0; k0 < d; k0 += 2 * kV) {
    const int k = k0 + half * kV;
    const bool k_ok = k < d;
    const uint4 va = (t_ok && k_ok) ? *reinterpret_cast<const uint4*>(a + (size_t)k * kEs) : make_uint4(0, 0, 0, 0);
    const uint4 vb = (s_ok && k_ok) ? *reinterpret_cast<const uint4*>(b + (size_t)k * kEs) : make_uint4(0, 0, 0, 0);
    if constexpr (BF16) {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va), __builtin_bit_cast(bf16x8, vb),
                                                    acc, 0, 0, 0);
    } else {
      const float4 fa = __builtin_bit_cast(float4, va), fb = __builtin_bit_cast(float4, vb);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.x, fb.x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.y, fb.y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.z, fb.z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.w, fb.w, acc, 0, 0, 0);
    }
  }
}

template <bool BF16>
__global__ __launch_bounds__(256) void ghost_gram_kernel(const void* __restrict__ X, const void* __restrict__ Delta,
                                                         const int32_t* __restrict__ tok_seq, int n_tokens, int d_in,
                                                         int d_out, int n_seq, int n_tiles, double* __restrict__ K64) {
  // blockIdx.x enumerates tile pairs (bt <= bs) row by row.
  int bt = 0, rem = blockIdx.x;
  while (rem >= n_tiles - bt) { rem -= n_tiles - bt; ++bt; }
  const int bs = bt + rem;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t0 = bt * 64 + (wave >> 1) * 32, s0 = bs * 64 + (wave & 1) * 32;
  if (t0 >= n_tokens || s0 >= n_tokens) return;
  if (t0 > s0) return;                       // lower-left wave of a diagonal tile: all pairs have t > s
  const int r32 = lane & 31, half = lane >> 5;
  const int t_row = t0 + r32, s_row = s0 + r32;
  const bool t_ok = t_row < n_tokens, s_ok = s_row < n_tokens;

  f32x16 P, Q;
#pragma unroll
  for (int v = 0; v < 16; ++v) { P[v] = 0.f; Q[v] = 0.f; }
  gram_block<BF16>(X, d_in, t_ok ? t_row : 0, s_ok ? s_row : 0, t_ok, s_ok, half, P);
  gram_block<BF16>(Delta, d_out, t_ok ? t_row : 0, s_ok ? s_row : 0, t_ok, s_ok, half, Q);

  // Lane holds column s = s0 + lane%32 and rows t = t0 + acc_row(v, lane).
  const int s = s0 + r32;
  const int q = s_ok ? tok_seq[s] : -1;
  const int t_last = min(t0 + 31, n_tokens - 1), s_last = min(s0 + 31, n_tokens - 1);
  const int r_first = tok_seq[t0], r_last = tok_seq[t_last];
  const int q_first = tok_seq[s0], q_last = tok_seq[s_last];
  const bool uniform = (r_first == r_last) && (q_first == q_last);   // same for the whole wave

  double run = 0.0;
  int run_r = -1;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int t = t0 + acc_row(v, lane);
    if (t >= n_tokens || !s_ok || t > s) continue;
    const int r = uniform ? r_first : tok_seq[t];
    const double w = (t == s) ? 1.0 : ((r == q) ? 2.0 : 1.0);
    const double h = w * (double)P[v] * (double)Q[v];
    if (uniform) {
      run += h;
    } else {
      if (r != run_r) {
        if (run_r >= 0) atomicAdd(&K64[(size_t)run_r * n_seq + q], run);
        run_r = r;
        run = 0.0;
      }
      run += h;
    }
  }
  if (uniform) {
    run = wave_sum(run);
    if (lane == 0) atomicAdd(&K64[(size_t)r_first * n_seq + q_first], run);
  } else if (run_r >= 0) {
    atomicAdd(&K64[(size_t)run_r * n_seq + q], run);
  }
}

__global__ void ghost_finish_kernel(const double* __restrict__ K64, int n_seq, float* __restrict__ K) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_seq * n_seq) return;
  const int i = idx / n_seq, j = idx % n_seq;
  if (i > j) return;
  const float v = (float)K64[(size_t)i * n_seq + j];
  K[(size_t)i * n_seq + j] = v;
  K[(size_t)j * n_seq + i] = v;
}

}  // namespace

hipError_t launch_ghost_gram(const GhostArgs& a, hipStream_t s) {
  const long long kk = (long long)a.n_seq * a.n_seq;
  hipLaunchKernelGGL(fill_f64_kernel, dim3((unsigned)((kk + 255) / 256)), dim3(256), 0, s, a.K64, kk);
  if (a.n_tokens > 0) {
    hipLaunchKernelGGL(token_seq_kernel, dim3((a.n_tokens + 255) / 256), dim3(256), 0, s, a.off, a.n_seq, a.n_tokens,
                       a.tok_seq);
    const long long n_tiles = (a.n_tokens + 63) / 64;
    const long long pairs = n_tiles * (n_tiles + 1) / 2;
    if (pairs > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.bf16)
      hipLaunchKernelGGL((ghost_gram_kernel<true>), dim3((unsigned)pairs), dim3(256), 0, s, a.X, a.Delta, a.tok_seq,
                         a.n_tokens, a.d_in, a.d_out, a.n_seq, (int)n_tiles, a.K64);
    else
      hipLaunchKernelGGL((ghost_gram_kernel<false>), dim3((unsigned)pairs), dim3(256), 0, s, a.X, a.Delta, a.tok_seq,
                         a.n_tokens, a.d_in, a.d_out, a.n_seq, (int)n_tiles, a.K64);
  }
  hipLaunchKernelGGL(ghost_finish_kernel, dim3((unsigned)((kk + 255) / 256)), dim3(256), 0, s, a.K64, a.n_seq, a.K);
  return hipGetLastError();
}

}  // namespace isopo
