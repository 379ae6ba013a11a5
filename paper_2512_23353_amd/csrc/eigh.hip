// Eigendecomposition route of the interacting variant (interacting listing:
// D, U = eigh(ntk); c = U ((1 / (D + regularization)) * (U^T A))).
//
// One decomposition serves any number of regularisers, so a sweep over lambda
// costs one factorisation instead of one Cholesky per value.  K is m x m with
// m the number of sequences (tens to a few hundred), so one workgroup per problem
// (a block's projections go in one launch) runs a cyclic two-sided Jacobi iteration
// in fp64: each round applies m/2 disjoint
// plane rotations (round-robin pairing), first to the rows, then to the columns
// of the work matrix and to the accumulated eigenvector matrix.  The matrices
// live in LDS when they fit, else in a caller-provided global scratch that stays
// in L2.  Eigenvalues come out ascending, eigenvectors as columns.
#include "common.h"
#include "kernels.h"

namespace isopo {
namespace {

constexpr int kMaxPairs = kEighMaxSeq / 2;
constexpr int kMaxSweeps = 40;
constexpr double kOffTol = 1e-14;      // stop when ||off(A)||_F <= kOffTol * ||A||_F

template <int THREADS>
__device__ double block_sum(double x, double* red) {
  x = wave_sum(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  double s = 0.0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) s += red[w];
  return s;
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void jacobi_eigh_kernel(const float* __restrict__ Kb, int m,
                                                              double* __restrict__ Db, double* __restrict__ Ub,
                                                              int32_t* __restrict__ infob, double* __restrict__ gAb,
                                                              double* __restrict__ gVb, size_t ws_stride) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  __shared__ double rot_c[kMaxPairs], rot_s[kMaxPairs];
  __shared__ short rot_p[kMaxPairs], rot_q[kMaxPairs];
  __shared__ double red[THREADS / 64];
  __shared__ short rank_of[kEighMaxSeq];
  const int tid = threadIdx.x;
  const size_t prob = blockIdx.x;        // one problem per workgroup
  const float* K = Kb + prob * m * m;
  double* D = Db + prob * m;
  double* U = Ub + prob * m * m;
  int32_t* info = infob ? infob + prob : nullptr;
  double* gA = gAb ? gAb + prob * ws_stride : nullptr;
  double* gV = gVb ? gVb + prob * ws_stride : nullptr;
  const int n = (m + 1) & ~1;            // even: an odd m gets one idle index
  const int ld = n + 1;                  // odd pitch: column walks spread over the LDS banks
  // work matrix and eigenvectors: each in LDS when the caller passes no global buffer for it
  double* Aw = gA ? gA : reinterpret_cast<double*>(smem_raw);
  double* V = gV ? gV : reinterpret_cast<double*>(smem_raw) + (gA ? 0 : (size_t)n * ld);
  const int half = n / 2;

  for (int e = tid; e < n * n; e += THREADS) {
    const int i = e / n, j = e % n;
    double v = 0.0;
    if (i < m && j < m) v = 0.5 * ((double)K[(size_t)i * m + j] + (double)K[(size_t)j * m + i]);
    Aw[(size_t)i * ld + j] = v;
    V[(size_t)i * ld + j] = i == j ? 1.0 : 0.0;
  }
  __syncthreads();

  int status = 1;                        // 1: not converged within kMaxSweeps
  for (int sweep = 0; sweep <= kMaxSweeps; ++sweep) {
    double off = 0.0, dia = 0.0;
    for (int e = tid; e < n * n; e += THREADS) {
      const int i = e / n, j = e % n;
      const double v = Aw[(size_t)i * ld + j];
      if (i == j) dia += v * v; else off += v * v;
    }
    off = block_sum<THREADS>(off, red);
    dia = block_sum<THREADS>(dia, red);
    if (off <= kOffTol * kOffTol * (off + dia)) { status = 0; break; }     // uniform: same sums in every thread
    if (sweep == kMaxSweeps) break;
    for (int round = 0; round < n - 1; ++round) {
      if (tid < half) {
        // round-robin pairing of n players: index n-1 stays, the others rotate
        int p, q;
        if (tid == 0) { p = n - 1; q = round; }
        else { p = (round + tid) % (n - 1); q = (round - tid + (n - 1)) % (n - 1); }
        double c = 1.0, s = 0.0;
        if (p < m && q < m) {
          const double apq = Aw[(size_t)p * ld + q];
          if (apq != 0.0) {
            const double tau = (Aw[(size_t)q * ld + q] - Aw[(size_t)p * ld + p]) / (2.0 * apq);
            const double t = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
            c = 1.0 / sqrt(1.0 + t * t);
            s = t * c;
          }
        }
        rot_c[tid] = c; rot_s[tid] = s; rot_p[tid] = (short)p; rot_q[tid] = (short)q;
      }
      __syncthreads();
      // A <- J^T A J, one 2x2 block per item: rows (p1, q1) of pair P, columns (p2, q2) of pair R.  The
      // block's new value depends on the block alone, and blocks are disjoint, so read-modify-write in place.
      for (int e = tid; e < half * half; e += THREADS) {
        const int P = e / half, R = e % half;
        const double c1 = rot_c[P], s1 = rot_s[P], c2 = rot_c[R], s2 = rot_s[R];
        const int p1 = rot_p[P], q1 = rot_q[P], p2 = rot_p[R], q2 = rot_q[R];
        const double a_pp = Aw[(size_t)p1 * ld + p2], a_pq = Aw[(size_t)p1 * ld + q2];
        const double a_qp = Aw[(size_t)q1 * ld + p2], a_qq = Aw[(size_t)q1 * ld + q2];
        const double r_pp = c1 * a_pp - s1 * a_qp, r_pq = c1 * a_pq - s1 * a_qq;     // rows: J_P^T B
        const double r_qp = s1 * a_pp + c1 * a_qp, r_qq = s1 * a_pq + c1 * a_qq;
        Aw[(size_t)p1 * ld + p2] = c2 * r_pp - s2 * r_pq;                             // columns: (.) J_R
        Aw[(size_t)p1 * ld + q2] = s2 * r_pp + c2 * r_pq;
        Aw[(size_t)q1 * ld + p2] = c2 * r_qp - s2 * r_qq;
        Aw[(size_t)q1 * ld + q2] = s2 * r_qp + c2 * r_qq;
      }
      for (int e = tid; e < half * n; e += THREADS) {            // V <- V J, columns p and q of row k
        const int R = e % half, k = e / half;
        const double c = rot_c[R], s = rot_s[R];
        const int p = rot_p[R], q = rot_q[R];
        const double vp = V[(size_t)k * ld + p], vq = V[(size_t)k * ld + q];
        V[(size_t)k * ld + p] = c * vp - s * vq;
        V[(size_t)k * ld + q] = s * vp + c * vq;
      }
      __syncthreads();
    }
  }

  // ascending order by rank (ties broken by index), eigenvectors as columns of U
  for (int i = tid; i < m; i += THREADS) {
    const double di = Aw[(size_t)i * ld + i];
    int rank = 0;
    for (int j = 0; j < m; ++j) {
      const double dj = Aw[(size_t)j * ld + j];
      rank += (dj < di || (dj == di && j < i)) ? 1 : 0;
    }
    D[rank] = di;
    rank_of[i] = (short)rank;
  }
  __syncthreads();
  for (int e = tid; e < m * m; e += THREADS) {
    const int k = e / m, i = e % m;
    U[(size_t)k * m + rank_of[i]] = V[(size_t)k * ld + i];
  }
  if (info && tid == 0) *info = status;
}

constexpr int kSolveThreads = 256;

// c[l] = U ((U^T A) / (D + reg_l)) for each regulariser of the sweep.
__global__ __launch_bounds__(kSolveThreads) void eigh_solve_kernel(EighSolveArgs a) {
  __shared__ double y[kEighMaxSeq];
  __shared__ double red[kSolveThreads / 64];
  __shared__ double sh_scale;
  const int tid = threadIdx.x, m = a.n_seq;
  const size_t prob = blockIdx.x;        // one problem per workgroup
  a.D += prob * m; a.U += prob * m * m; a.A += prob * m; a.c += prob * a.n_lambda * m;
  if (a.ema_state) a.ema_state += prob * 2;
  if (a.info) a.info += prob;
  double tr = 0.0;
  for (int j = tid; j < m; j += kSolveThreads) {
    double s = 0.0;
    for (int i = 0; i < m; ++i) s += a.U[(size_t)i * m + j] * (double)a.A[i];
    y[j] = s;
    tr += a.D[j];
  }
  const double mean_d = block_sum<kSolveThreads>(tr, red) / (double)m;
  if (tid == 0) {
    double scale = 1.0;                                   // ABSOLUTE
    if (a.reg_mode == 1) scale = mean_d;                  // this batch's mean eigenvalue
    if (a.reg_mode == 2) {                                // trailing mean over minibatches, this one included
      const double prev = (double)a.ema_state[0];
      const bool first = a.ema_state[1] == 0.f;
      scale = first ? mean_d : (double)a.ema_decay * prev + (1.0 - (double)a.ema_decay) * mean_d;
      a.ema_state[0] = (float)scale;
      a.ema_state[1] = a.ema_state[1] + 1.f;
    }
    sh_scale = scale;
  }
  __syncthreads();
  const double scale = sh_scale;
  int bad = 0;
  for (int l = 0; l < a.n_lambda; ++l) {
    const double reg = (double)a.lambdas[l] * scale;
    for (int i = tid; i < m; i += kSolveThreads) {
      double s = 0.0;
      for (int j = 0; j < m; ++j) {
        const double den = a.D[j] + reg;
        if (den > 0.0) s += a.U[(size_t)i * m + j] * (y[j] / den);
        else if (i == 0) ++bad;
      }
      a.c[(size_t)l * m + i] = (float)s;
    }
  }
  if (a.info && tid == 0) *a.info = bad;
}

}  // namespace

size_t eigh_workspace(int m) {
  const int n = (m + 1) & ~1;
  return 2 * (size_t)n * (n + 1) * sizeof(double);
}

template <int THREADS>
hipError_t launch_jacobi(const float* K, int m, int batch, double* D, double* U, int32_t* info, size_t smem,
                         double* gA, double* gV, size_t ws_stride, hipStream_t s) {
  auto kern = jacobi_eigh_kernel<THREADS>;
  // once per process (static initialisation is thread-safe); a failure is returned by every call
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kEighLdsBytes);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3(batch), dim3(THREADS), smem, s, K, m, D, U, info, gA, gV, ws_stride);
  return hipGetLastError();
}

hipError_t launch_ntk_eigh(const float* K, int m, int batch, double* D, double* U, int32_t* info, void* workspace,
                           hipStream_t s) {
  const int n = (m + 1) & ~1;
  const size_t one = (size_t)n * (n + 1) * sizeof(double);
  double* ws = static_cast<double*>(workspace);
  size_t smem;
  double *gA = nullptr, *gV = nullptr;
  if (2 * one <= kEighLdsBytes) smem = 2 * one;                       // both in LDS
  else if (one <= kEighLdsBytes) { smem = one; gV = ws; }             // work matrix in LDS, eigenvectors in L2
  else { smem = 0; gA = ws; gV = ws + (size_t)n * (n + 1); }
  const size_t ws_stride = eigh_workspace(m) / sizeof(double);      // doubles per problem
  return n <= 32 ? launch_jacobi<256>(K, m, batch, D, U, info, smem, gA, gV, ws_stride, s)
                 : launch_jacobi<1024>(K, m, batch, D, U, info, smem, gA, gV, ws_stride, s);
}

hipError_t launch_eigh_solve(const EighSolveArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(eigh_solve_kernel, dim3(a.batch), dim3(kSolveThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace isopo
