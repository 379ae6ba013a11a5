// Per-sequence coefficients from the layer's Gram matrix K and the advantages A.
//
//   FISHER       c_i = A_i / sqrt(||g_i||_F^2 + reg),  ||g_i||_F^2 = (1/m) sum_j K_ij^2
//                (non-interacting update u_l, with the Fisher norm of eq.
//                F-norm-basic taken over the batch's reduced gradients, j = i
//                included)
//   INTERACTING  c = (K + reg I)^-1 A          (v = J^T (K + cI)^-1 A)
//
// reg = lambda, or lambda times this batch's typical value of the quantity reg is
// added to, or lambda times the trailing mean over minibatches of that value.  For
// INTERACTING the value is tr(K)/m (the interacting experiment's regulariser,
// factor * E[mean(D)]: the mean eigenvalue is the trace over m, so no
// decomposition is needed for it); for FISHER it is mean_i ||g_i||_F^2 (the
// non-interacting derivation compares reg_l with the typical ||.||_F^2).
// The m x m problem is tiny next to the
// contractions around it, so one workgroup per problem works in fp64: a
// right-looking Cholesky factorisation in LDS (m <= 128) or in a caller-provided
// global scratch (larger m), then two triangular solves.  The result is the
// unique solution; the eigendecomposition the interacting listing uses reaches
// the same vector.  A non-positive pivot is reported, never clamped.
#include "common.h"
#include "kernels.h"

namespace isopo {
namespace {

constexpr int ISOPO_MAX_SEQ_TRANSFORM = 1024;     // the header's ISOPO_MAX_SEQ

template <int kThreads>
__device__ double block_sum(double x, double* red /* [kThreads/64] */) {
  x = wave_sum(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  double s = 0.0;
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) s += red[w];
  return s;
}

template <int kThreads>
__global__ __launch_bounds__(kThreads) void transform_kernel(const float* __restrict__ Kb, const float* __restrict__ Ab,
                                                             int m, int variant, int reg_mode, float lambda,
                                                             float* __restrict__ cb, int32_t* __restrict__ info,
                                                             double* __restrict__ gws, float* __restrict__ ema_state,
                                                             float ema_decay) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ double red[kThreads / 64];
  const int prob = blockIdx.x, tid = threadIdx.x;
  const float* K = Kb + (size_t)prob * m * m;
  const float* A = Ab + (size_t)prob * m;
  float* c = cb + (size_t)prob * m;

  // FISHER: the norms first; the relative regulariser is measured against their mean
  __shared__ double f2s[ISOPO_MAX_SEQ_TRANSFORM];
  if (variant == 0) {
    for (int i = tid; i < m; i += kThreads) {
      double s = 0.0;
      for (int j = 0; j < m; ++j) {
        const double k = (double)K[(size_t)i * m + j];
        s += k * k;
      }
      f2s[i] = s / (double)m;
    }
    __syncthreads();
  }

  double reg = (double)lambda;
  if (reg_mode != 0) {
    // this batch's typical value of what reg is added to: the mean eigenvalue tr(K)/m of K (INTERACTING),
    // the mean of the Fisher norms (FISHER)
    double part = 0.0;
    for (int i = tid; i < m; i += kThreads) part += variant == 0 ? f2s[i] : (double)K[(size_t)i * m + i];
    double scale = block_sum<kThreads>(part, red) / (double)m;
    if (reg_mode == 2) {
      // trailing mean over minibatches, this one included; every thread forms the same value from the
      // state as it was, then one thread stores the new state
      float* st = ema_state + (size_t)prob * 2;
      const double prev = (double)st[0];
      const bool first = st[1] == 0.f;
      scale = first ? scale : (double)ema_decay * prev + (1.0 - (double)ema_decay) * scale;
      __syncthreads();                                                  // everyone has read the old state
      if (tid == 0) { st[0] = (float)scale; st[1] = st[1] + 1.f; }
    }
    reg = (double)lambda * scale;
  }

  if (variant == 0) {
    for (int i = tid; i < m; i += kThreads) {
      const double den = f2s[i] + reg;
      c[i] = den > 0.0 ? (float)((double)A[i] / sqrt(den)) : 0.f;
    }
    if (info && tid == 0) info[prob] = 0;
    return;
  }

  // M = K + reg I (lower triangle), y, in LDS or global scratch.
  double* M = gws ? gws + (size_t)prob * ((size_t)m * m + m) : reinterpret_cast<double*>(smem);
  double* y = M + (size_t)m * m;
  for (int e = tid; e < m * m; e += kThreads) {
    const int r = e / m, q = e % m;
    if (q <= r) M[e] = (double)K[e] + (r == q ? reg : 0.0);
  }
  for (int i = tid; i < m; i += kThreads) y[i] = (double)A[i];
  __syncthreads();

  // Right-looking Cholesky in panels of kPanel columns: the panel is factored column by column (updates
  // confined to the panel), then the trailing matrix takes one rank-kPanel update, so the large matrix is
  // swept m/kPanel times instead of m times.
  constexpr int kPanel = 8;
  for (int k0 = 0; k0 < m; k0 += kPanel) {
    const int nb = m - k0 < kPanel ? m - k0 : kPanel;
    for (int kk = 0; kk < nb; ++kk) {
      const int k = k0 + kk;
      const double d = M[(size_t)k * m + k];
      if (!(d > 0.0)) {                       // uniform: every thread reads the same value
        for (int i = tid; i < m; i += kThreads) c[i] = __builtin_nanf("");
        if (info && tid == 0) info[prob] = k + 1;
        return;
      }
      const double inv = 1.0 / sqrt(d);
      __syncthreads();                        // everyone has read the pivot
      for (int r = k + tid; r < m; r += kThreads) M[(size_t)r * m + k] *= inv;   // column k of L (M[k][k] -> sqrt(d))
      __syncthreads();
      const int ncol = k0 + nb - 1 - k;       // panel columns right of k
      const int nrow = m - k - 1;
      for (int e = tid; e < nrow * ncol; e += kThreads) {
        const int r = k + 1 + e / ncol, q = k + 1 + e % ncol;
        if (q <= r) M[(size_t)r * m + q] -= M[(size_t)r * m + k] * M[(size_t)q * m + k];
      }
      __syncthreads();
    }
    const int t0 = k0 + nb, rem = m - t0;     // trailing lower triangle, rows/cols t0..m-1
    for (int e = tid; e < rem * rem; e += kThreads) {
      const int r = t0 + e / rem, q = t0 + e % rem;
      if (q <= r) {
        double s = 0.0;
        for (int kk = 0; kk < nb; ++kk) s += M[(size_t)r * m + k0 + kk] * M[(size_t)q * m + k0 + kk];
        M[(size_t)r * m + q] -= s;
      }
    }
    __syncthreads();
  }
  // forward: L y = A
  for (int k = 0; k < m; ++k) {
    const double yk = y[k] / M[(size_t)k * m + k];
    __syncthreads();
    if (tid == 0) y[k] = yk;
    for (int r = k + 1 + tid; r < m; r += kThreads) y[r] -= M[(size_t)r * m + k] * yk;
    __syncthreads();
  }
  // backward: L^T c = y
  for (int k = m - 1; k >= 0; --k) {
    const double ck = y[k] / M[(size_t)k * m + k];
    __syncthreads();
    if (tid == 0) y[k] = ck;
    for (int r = tid; r < k; r += kThreads) y[r] -= M[(size_t)k * m + r] * ck;
    __syncthreads();
  }
  for (int i = tid; i < m; i += kThreads) c[i] = (float)y[i];
  if (info && tid == 0) info[prob] = 0;
}

}  // namespace

template <int THREADS>
hipError_t launch_transform_t(const TransformArgs& a, size_t smem, double* gws, hipStream_t s) {
  auto kern = transform_kernel<THREADS>;
  // once per process and instantiation (static initialisation is thread-safe); a failure is returned by every call
  constexpr int max_smem = (int)(((size_t)kTransformLdsMax * kTransformLdsMax + kTransformLdsMax) * sizeof(double));
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, max_smem);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3(a.batch), dim3(THREADS), smem, s, a.K, a.A, a.n_seq, a.variant, a.reg_mode, a.lambda,
                     a.c, a.info, gws, a.ema_state, a.ema_decay);
  return hipGetLastError();
}

hipError_t launch_transform(const TransformArgs& a, hipStream_t s) {
  const bool lds = a.n_seq <= kTransformLdsMax;
  size_t smem = 0;
  if (a.variant == 1 && lds) smem = ((size_t)a.n_seq * a.n_seq + a.n_seq) * sizeof(double);
  double* gws = (a.variant == 1 && !lds) ? a.workspace : nullptr;
  // the trailing update of column k has (m-k)^2/2 independent elements: more threads for larger problems
  if (a.n_seq <= 48) return launch_transform_t<256>(a, smem, gws, s);
  if (a.n_seq <= 96) return launch_transform_t<512>(a, smem, gws, s);
  return launch_transform_t<1024>(a, smem, gws, s);
}

}  // namespace isopo
