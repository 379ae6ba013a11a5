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
// The m x m problem is tiny next to the contractions around it, so one
// workgroup per problem works in fp64: a
// right-looking Cholesky factorisation in panels and two triangular solves.  The
// matrix lives in LDS (m <= 128) or in a caller-provided global scratch (larger
// m); the panel being factored is in LDS, column-major, and each thread holds one
// of its rows in registers (one barrier per column); A rides along as one more
// row of the matrix, which makes the forward solve part of the factorisation, and
// the backward solve runs panel by panel as well.  The result is the unique
// solution; the eigendecomposition the interacting listing uses reaches the same
// vector.  A non-positive pivot is reported, never clamped.
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

// A value every lane holds alike, moved to scalar registers (the column entries all rows are updated with:
// thirty-one doubles next to a 32-double row would not fit the vector registers of a 1024-thread workgroup).
__device__ __forceinline__ double uniform_value(double x) {
  const int lo = __builtin_amdgcn_readfirstlane(__double2loint(x));
  const int hi = __builtin_amdgcn_readfirstlane(__double2hiint(x));
  return __hiloint2double(hi, lo);
}

// Panel rows in LDS: one padding element after every 32 rows of a column, so that the trailing update's
// lanes, which read groups of four consecutive rows 32 bytes apart, spread over all banks.
__device__ __forceinline__ int panel_pos(int lr) { return lr + (lr >> 5); }
__host__ __device__ constexpr int panel_stride(int m) { return ((m + 1) + ((m + 1) >> 5) + 1 + 3) & ~3; }

// (K + reg I) c = A: M [m + 1, m] fp64 in LDS or global memory (row m holds A, then y), the panel of NB columns
// in LDS as PT[column][row - k0] with row stride RS.  kThreads threads; c is left in cs.
//
// Panel step: thread t holds the panel rows t and t + kThreads (R = 2: only a 1025-row panel has the second;
// the launch gives smaller problems enough threads for R = 1) in registers.  Per column kk: every row's entry
// goes to LDS, one barrier, then each thread reads the pivot and the entries (q, kk) of the rows q > kk (the
// same addresses for all lanes) and eliminates column kk from its rows with the unscaled entries,
// row[q] -= row[kk] * (q, kk) / pivot; its own entry of L is row[kk] / sqrt(pivot).
// The upper triangle of the diagonal block is carried along and never read.  The trailing matrix (rows up to
// and including the row of A) then takes the rank-NB update in 4 x 4 register blocks whose factors come from
// the panel in LDS.
template <int kThreads, int NB, int R>
__device__ bool cholesky_solve(const float* __restrict__ K, const float* __restrict__ A, int m, double reg,
                               double* __restrict__ M, double* cs /* LDS [m] */, double* PT /* LDS */, int* fail_col) {
  const int tid = threadIdx.x;
  const int RS = panel_stride(m);
  // the whole square, so that every later read is of a defined value; the upper triangle never enters a result
  for (int e = tid; e < m * m; e += kThreads) {
    const int r = e / m, q = e - r * m;
    M[e] = (double)K[e] + (r == q ? reg : 0.0);
  }
  for (int i = tid; i < m; i += kThreads) M[(size_t)m * m + i] = (double)A[i];
  __syncthreads();

  for (int k0 = 0; k0 < m; k0 += NB) {
    const int nbk = m - k0 < NB ? m - k0 : NB;
    const int nrows = m + 1 - k0;                        // rows k0 .. m
    // panel -> LDS (a wave reads NB-element pieces of rows)
    for (int e = tid; e < nrows * NB; e += kThreads) {
      const int lr = e / NB, kk = e % NB;
      if (kk < nbk) PT[kk * RS + panel_pos(lr)] = M[(size_t)(k0 + lr) * m + k0 + kk];
    }
    __syncthreads();
    // the thread's rows (R = 2 only where m + 1 > kThreads) in registers; waves without a row only keep the barriers
    const bool wave_has_rows = (tid & ~(kWave - 1)) < nrows;
    double row[R][NB];
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int lr = tid + i * kThreads;
#pragma unroll
      for (int q = 0; q < NB; ++q) row[i][q] = (lr < nrows && q < nbk) ? PT[q * RS + panel_pos(lr)] : 0.0;
    }
    bool failed = false;                                           // uniform
#pragma unroll
    for (int kk = 0; kk < NB; ++kk) {
      if (kk >= nbk || failed) continue;                           // no break: the loop has to unroll for row[][] to stay in registers
      // column kk as the columns before it left it: every row's entry goes to the column's own place in LDS
#pragma unroll
      for (int i = 0; i < R; ++i) {
        const int lr = tid + i * kThreads;
        if (lr < nrows) PT[kk * RS + panel_pos(lr)] = row[i][kk];
      }
      __syncthreads();
      const double d = uniform_value(PT[kk * RS + panel_pos(kk)]);
      if (!(d > 0.0)) { *fail_col = k0 + kk; failed = true; continue; }      // every thread reads the same value
      if (!wave_has_rows) continue;
      const double rsq = 1.0 / sqrt(d), rd = rsq * rsq;
      double f[R];
#pragma unroll
      for (int i = 0; i < R; ++i) {
        f[i] = row[i][kk] * rd;
        row[i][kk] *= rsq;                                         // the entry of L; the pivot's own row: d / sqrt(d)
      }
      // eight columns at a time, so that only eight of the column's entries are held at once
#pragma unroll
      for (int q0 = kk + 1; q0 < NB; q0 += 8) {
        double b[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (q0 + j < NB) b[j] = uniform_value(PT[kk * RS + panel_pos(q0 + j)]);   // entry (q, kk); for q >= nbk a row below the block: unused
#pragma unroll
        for (int i = 0; i < R; ++i)
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (q0 + j < NB) row[i][q0 + j] -= f[i] * b[j];
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (failed) return false;
    __syncthreads();                                               // the last column has been read
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int lr = tid + i * kThreads;
#pragma unroll
      for (int q = 0; q < NB; ++q)
        if (lr < nrows && q < nbk) PT[q * RS + panel_pos(lr)] = row[i][q];
    }
    __syncthreads();
    for (int e = tid; e < nrows * NB; e += kThreads) {
      const int lr = e / NB, kk = e % NB;
      if (kk < nbk) M[(size_t)(k0 + lr) * m + k0 + kk] = PT[kk * RS + panel_pos(lr)];
    }
    // trailing update: rows t0 .. m (the row of A included), columns t0 .. min(row, m - 1)
    const int t0 = k0 + nbk;
    const int nbr = (m + 1 - t0 + 3) >> 2, nbq = (m - t0 + 3) >> 2;
    for (int e = tid; e < nbr * nbq; e += kThreads) {
      const int br = e / nbq, bq = e - br * nbq;
      if (bq > br) continue;
      const int r0 = t0 + 4 * br, q0 = t0 + 4 * bq;
      int lr[4], lq[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        lr[i] = panel_pos((r0 + i <= m ? r0 + i : m) - k0);
        lq[i] = panel_pos((q0 + i < m ? q0 + i : m - 1) - k0);
      }
      double acc[4][4] = {};
      for (int kk = 0; kk < nbk; ++kk) {
        double a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[i] = PT[kk * RS + lr[i]]; b[i] = PT[kk * RS + lq[i]]; }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int r = r0 + i, q = q0 + j;
          if (r <= m && q < m && (q <= r)) M[(size_t)r * m + q] -= acc[i][j];
        }
    }
    __syncthreads();
  }

  // backward: L^T c = y (y is row m of M), last panel first.  The sums over the rows below a panel are split
  // over kThreads / NB row groups and met in LDS; wave 0 then solves the panel's triangle, lane = column.
  constexpr int RG = kThreads / NB;
  double* red = PT;                                       // [RG][NB + 1]
  double* tri = PT + RG * (NB + 1);                       // [NB][NB + 1]: the panel's diagonal block of L
  const int kk = tid % NB, rg = tid / NB;
  for (int k0 = ((m - 1) / NB) * NB; k0 >= 0; k0 -= NB) {
    const int nbk = m - k0 < NB ? m - k0 : NB;
    const int t0 = k0 + nbk;
    double acc = 0.0;
    if (kk < nbk)
      for (int r = t0 + rg; r < m; r += RG) acc += M[(size_t)r * m + k0 + kk] * cs[r];
    red[rg * (NB + 1) + kk] = acc;
    for (int e = tid; e < NB * NB; e += kThreads) {
      const int r = e / NB, q = e % NB;
      if (r < nbk && q <= r) tri[r * (NB + 1) + q] = M[(size_t)(k0 + r) * m + k0 + q];
    }
    __syncthreads();
    if (tid < kWave) {
      const int lane = tid;
      double v = 0.0;
      if (lane < nbk) {
        double sum = 0.0;
        for (int g = 0; g < RG; ++g) sum += red[g * (NB + 1) + lane];
        v = M[(size_t)m * m + k0 + lane] - sum;
      }
      double cv = 0.0;
      for (int j = nbk - 1; j >= 0; --j) {
        const double cj = __shfl(v, j, kWave) / tri[j * (NB + 1) + j];
        if (lane == j) cv = cj;
        if (lane < j) v -= tri[j * (NB + 1) + lane] * cj;
      }
      if (lane < nbk) cs[k0 + lane] = cv;
    }
    __syncthreads();
  }
  return true;
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

  if (gws) {
    if constexpr (kThreads == 1024) {
      double* Mg = gws + (size_t)prob * ((size_t)m * m + m);
      double* PT = reinterpret_cast<double*>(smem);
      int fail_col = 0;
      const bool ok = m <= kTransformWidePanelMax ? cholesky_solve<1024, 32, 1>(K, A, m, reg, Mg, f2s, PT, &fail_col)
                                                  : cholesky_solve<1024, 16, 2>(K, A, m, reg, Mg, f2s, PT, &fail_col);
      for (int i = tid; i < m; i += kThreads) c[i] = ok ? (float)f2s[i] : __builtin_nanf("");
      if (info && tid == 0) info[prob] = ok ? 0 : fail_col + 1;
    }
    return;
  }

  // the matrix in LDS as well, panels of 16 columns
  double* Ml = reinterpret_cast<double*>(smem);
  int fail_col = 0;
  const bool ok = cholesky_solve<kThreads, 16, 1>(K, A, m, reg, Ml, f2s, Ml + (size_t)(m + 1) * m, &fail_col);
  for (int i = tid; i < m; i += kThreads) c[i] = ok ? (float)f2s[i] : __builtin_nanf("");
  if (info && tid == 0) info[prob] = ok ? 0 : fail_col + 1;
}

}  // namespace

// Dynamic LDS of the INTERACTING transform: the panel (32 columns up to kTransformWidePanelMax sequences in
// global scratch, else 16) or what the backward solve keeps there instead (at most 1024 / 16 + 16 rows of 17),
// and up to kTransformLdsMax sequences the matrix with the row of A in front of it.
constexpr size_t transform_lds_bytes(int m) {
  const bool lds = m <= kTransformLdsMax;
  const int nb = (!lds && m <= kTransformWidePanelMax) ? 32 : 16;
  size_t panel = (size_t)nb * panel_stride(m);
  const size_t backward = nb == 32 ? (size_t)(32 + 32) * 33 : (size_t)(64 + 16) * 17;
  if (panel < backward) panel = backward;
  return ((lds ? (size_t)(m + 1) * m : 0) + panel) * sizeof(double);
}

template <int THREADS>
hipError_t launch_transform_t(const TransformArgs& a, size_t smem, double* gws, hipStream_t s) {
  auto kern = transform_kernel<THREADS>;
  // once per process and instantiation (static initialisation is thread-safe); a failure is returned by every call
  constexpr int max_smem = (int)transform_lds_bytes(kTransformLdsMax) > (int)transform_lds_bytes(kTransformWidePanelMax)
                               ? (int)transform_lds_bytes(kTransformLdsMax) : (int)transform_lds_bytes(kTransformWidePanelMax);
  static_assert(transform_lds_bytes(ISOPO_MAX_SEQ_TRANSFORM) <= (size_t)max_smem && max_smem + 8704 <= 160 * 1024, "LDS budget");
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, max_smem);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3(a.batch), dim3(THREADS), smem, s, a.K, a.A, a.n_seq, a.variant, a.reg_mode, a.lambda,
                     a.c, a.info, gws, a.ema_state, a.ema_decay);
  return hipGetLastError();
}

hipError_t launch_transform(const TransformArgs& a, hipStream_t s) {
  const bool lds = a.n_seq <= kTransformLdsMax;
  const size_t smem = a.variant == 1 ? transform_lds_bytes(a.n_seq) : 0;
  double* gws = (a.variant == 1 && !lds) ? a.workspace : nullptr;
  // the trailing update of column k has (m-k)^2/2 independent elements: more threads for larger problems
  if (a.n_seq <= 48) return launch_transform_t<256>(a, smem, gws, s);
  if (a.n_seq <= 96) return launch_transform_t<512>(a, smem, gws, s);
  return launch_transform_t<1024>(a, smem, gws, s);
}

}  // namespace isopo
