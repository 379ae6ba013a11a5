// Generalised per-sequence re-scaling (alternative re-scalings listing):
//
//     rel_F_norm = F_norm / ||G||
//     scaling    = reg2(F_norm)^p * reg2(||G||)^q * reg2(rel_F_norm)^r,   c_i = A_i * scaling_i
//     reg2(val)  = sqrt(val^2 + regularization * E[val^2] + 1e-8)
//
// p = -1 is the KL-bounding re-scaling, r = -2 the closest-to-natural-gradient
// one, q = -1 with r = -2 the setting of the headline experiment.  The inputs
// are per-sequence squares: F_norm^2 (from the Gram matrix, or from the
// token-position samples) and ||G_i||^2 = K_ii.  E[val^2] is the caller's
// trailing mean, or this batch's mean when the caller passes none; the batch
// means are returned so the caller can carry the trailing mean forward.
// m values: one workgroup, fp64, fixed summation order.
#include "common.h"
#include "kernels.h"

namespace isopo {
namespace {

constexpr int kThreads = 256;
constexpr double kEps = 1e-8;

__device__ double block_sum(double x, double* red) {
  x = wave_sum(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  double s = 0.0;
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) s += red[w];
  return s;
}

__device__ __forceinline__ double rel_sq(double f2, double g2) { return g2 > 0.0 ? f2 / g2 : 0.0; }

__global__ __launch_bounds__(kThreads) void rescale_kernel(RescaleArgs a) {
  __shared__ double red[kThreads / 64];
  const int tid = threadIdx.x, m = a.n_seq;
  double sf = 0.0, sg = 0.0, sr = 0.0;
  for (int i = tid; i < m; i += kThreads) {
    const double f2 = (double)a.fisher_sq[i], g2 = (double)a.grad_sq[(size_t)i * a.grad_sq_stride];
    sf += f2;
    sg += g2;
    sr += rel_sq(f2, g2);
  }
  const double mean_f = block_sum(sf, red) / m, mean_g = block_sum(sg, red) / m, mean_r = block_sum(sr, red) / m;
  const double ef = a.expectation[0] >= 0.f ? (double)a.expectation[0] : mean_f;
  const double eg = a.expectation[1] >= 0.f ? (double)a.expectation[1] : mean_g;
  const double er = a.expectation[2] >= 0.f ? (double)a.expectation[2] : mean_r;
  for (int i = tid; i < m; i += kThreads) {
    const double f2 = (double)a.fisher_sq[i], g2 = (double)a.grad_sq[(size_t)i * a.grad_sq_stride];
    const double rf = f2 + (double)a.reg[0] * ef + kEps;          // reg2(.)^2 of the three quantities
    const double rg = g2 + (double)a.reg[1] * eg + kEps;
    const double rr = rel_sq(f2, g2) + (double)a.reg[2] * er + kEps;
    // reg2^p = (reg2^2)^(p/2)
    const double scaling = pow(rf, 0.5 * (double)a.p) * pow(rg, 0.5 * (double)a.q) * pow(rr, 0.5 * (double)a.r);
    a.c[i] = (float)((double)a.A[i] * scaling);
  }
  if (a.batch_means && tid == 0) {
    a.batch_means[0] = (float)mean_f;
    a.batch_means[1] = (float)mean_g;
    a.batch_means[2] = (float)mean_r;
  }
}

// fisher_sq[i] = (1/m) sum_j K_ij^2 (eq. F-norm-basic over the batch's reduced gradients), grad_sq[i] = K_ii.
__global__ __launch_bounds__(kThreads) void gram_norms_kernel(const float* __restrict__ K, int m,
                                                              float* __restrict__ fisher_sq,
                                                              float* __restrict__ grad_sq) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i >= m) return;
  double s = 0.0;
  for (int j = 0; j < m; ++j) {
    const double k = (double)K[(size_t)i * m + j];
    s += k * k;
  }
  if (fisher_sq) fisher_sq[i] = (float)(s / (double)m);
  if (grad_sq) grad_sq[i] = K[(size_t)i * m + i];
}

}  // namespace

hipError_t launch_rescale(const RescaleArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(rescale_kernel, dim3(1), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_gram_norms(const float* K, int m, float* fisher_sq, float* grad_sq, hipStream_t s) {
  hipLaunchKernelGGL(gram_norms_kernel, dim3((m + kThreads - 1) / kThreads), dim3(kThreads), 0, s, K, m, fisher_sq,
                     grad_sq);
  return hipGetLastError();
}

}  // namespace isopo
