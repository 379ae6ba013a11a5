// Eigendecomposition route of the interacting variant (interacting listing:
// D, U = eigh(ntk); c = U ((1 / (D + regularization)) * (U^T A))).
//
// One decomposition serves any number of regularisers, so a sweep over lambda
// costs one factorisation instead of one Cholesky per value.  K is m x m with
// m the number of sequences (tens to a few hundred), so one workgroup per problem
// (a block's projections go in one launch) runs a cyclic two-sided Jacobi iteration
// in fp64: each round applies m/2 disjoint
// plane rotations (round-robin pairing), first to the rows, then to the columns
// of the work matrix and to the accumulated eigenvector matrix, both in LDS.
// Problems too large for that (95 sequences and more) take the classical dense
// route further down: Householder tridiagonalisation and implicit QL.
// Eigenvalues come out ascending, eigenvectors as columns.
#include "common.h"
#include "kernels.h"

namespace isopo {
namespace {

constexpr int kMaxPairs = kEighMaxSeq / 2;
constexpr int kMaxSweeps = 40;
constexpr double kOffTol = 1e-14;      // stop when ||off(A)||_F <= kOffTol * ||A||_F
// Sizes from which the tridiagonal route below replaces the Jacobi iteration: where the Jacobi iteration's two
// matrices no longer both fit LDS (measured: Jacobi 2.1 ms against 2.4 ms at 80, 4.1 against 3.3 ms at 96).
constexpr int kEighTridiagonalFrom = 95;

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

// ---- larger problems: Householder tridiagonalisation, then implicit QL on the tridiagonal matrix -----
// Once its matrices no longer fit LDS the Jacobi iteration streams them through one compute unit in each
// of its ~10 n rounds (9.3 ms at n = 128, 84 ms at n = 256).  The classical dense route needs one
// O(n^3) reduction instead: K = Q T Q^T with Q a product of n - 2 reflectors H_k = I - tau_k v_k v_k^T and T
// tridiagonal, then T = Z diag(D) Z^T by implicit QL steps with Wilkinson's shift, whose plane rotations
// are applied to the columns of Q as they are generated, so that U = Q Z comes out in place.  One workgroup
// per problem, fp64 throughout.  K is scaled by a power of two so that its largest entry lies in [1, 2)
// (exact; D is scaled back at the end).
//   work matrix A (n x n, global scratch, kept bit-symmetric): rows k+1.. of the trailing block are updated
//     as A -= v w^T + w v^T; row k then holds v_k for the accumulation of Q
//   Zt (n x n, global scratch) holds Q^T, later (Q Z)^T: a rotation of columns i, i+1 of Z is a rotation of rows
//     i, i+1 of Zt, which thread k applies to element k of both rows (coalesced)
constexpr int kMaxQlIterations = 60;       // per eigenvalue

template <int THREADS>
__global__ __launch_bounds__(THREADS) void tridiag_eigh_kernel(const float* __restrict__ Kb, int m,
                                                               double* __restrict__ Db, double* __restrict__ Ub,
                                                               int32_t* __restrict__ infob, double* __restrict__ wsb,
                                                               size_t ws_stride) {
  __shared__ double d[kEighMaxSeq], e[kEighMaxSeq], tau[kEighMaxSeq], v[kEighMaxSeq], w[kEighMaxSeq];
  __shared__ double rc[kEighMaxSeq], rs[kEighMaxSeq];
  __shared__ double red[THREADS / 64];
  __shared__ short rank_of[kEighMaxSeq];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int WAVES = THREADS / 64;
  const size_t prob = blockIdx.x;        // one problem per workgroup
  const float* K = Kb + prob * m * m;
  double* D = Db + prob * m;
  double* U = Ub + prob * m * m;
  int32_t* info = infob ? infob + prob : nullptr;
  double* A = wsb + prob * ws_stride;
  double* Zt = A + (size_t)m * m;
  const int n = m;

  // symmetrised, scaled copy; Zt = I
  double amax = 0.0;
  for (int el = tid; el < n * n; el += THREADS) {
    const int i = el / n, j = el % n;
    const double a = 0.5 * ((double)K[(size_t)i * n + j] + (double)K[(size_t)j * n + i]);
    A[el] = a;
    Zt[el] = i == j ? 1.0 : 0.0;
    const double aa = fabs(a);
    amax = aa > amax ? aa : amax;        // a NaN never wins; it surfaces as "not converged" below
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { const double t = __shfl_xor(amax, o); amax = t > amax ? t : amax; }
  __syncthreads();
  if (lane == 0) red[wave] = amax;
  __syncthreads();
  amax = 0.0;
#pragma unroll
  for (int q = 0; q < WAVES; ++q) amax = red[q] > amax ? red[q] : amax;
  int expo = 0;
  if (amax > 0.0 && amax < 1.7e308) (void)frexp(amax, &expo);
  const double down = scalbn(1.0, 1 - expo), up = scalbn(1.0, expo - 1);
  __syncthreads();
  for (int el = tid; el < n * n; el += THREADS) A[el] *= down;
  __syncthreads();

  // ---- tridiagonalisation: three barriers per column ----
  for (int k = 0; k + 2 < n; ++k) {
    // trailing block: indices k+1 .. n-1; row k holds the column to reduce (the matrix is symmetric)
    if (wave == 0) {                                          // the reflector, by one wave
      double* rowk = A + (size_t)k * n;
      double sig = 0.0;
      for (int j = k + 2 + lane; j < n; j += 64) { const double x = rowk[j]; sig += x * x; }
      sig = wave_sum(sig);
      const double x0 = rowk[k + 1];
      if (lane == 0) d[k] = rowk[k];
      if (sig == 0.0) {                                       // column already reduced
        if (lane == 0) { e[k] = x0; tau[k] = 0.0; }
      } else {
        const double nrm = sqrt(x0 * x0 + sig);
        const double alpha = x0 > 0.0 ? -nrm : nrm;
        const double v0 = x0 - alpha;
        if (lane == 0) { e[k] = alpha; tau[k] = 2.0 / (v0 * v0 + sig); }
        for (int j = k + 1 + lane; j < n; j += 64) {
          const double vj = j == k + 1 ? v0 : rowk[j];
          v[j] = vj;
          rowk[j] = vj;                                       // kept for the accumulation of Q
        }
      }
    }
    __syncthreads();
    const double tk = tau[k];
    if (tk == 0.0) continue;                                  // uniform
    // p = tau A22 v: a wave takes four rows at a time (four independent streams of loads), lanes along the row
    for (int i0 = k + 1 + wave; i0 < n; i0 += 4 * WAVES) {
      double acc[4] = {0.0, 0.0, 0.0, 0.0};
      const double* row[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) row[q] = A + (size_t)(i0 + q * WAVES < n ? i0 + q * WAVES : n - 1) * n;
      for (int j = k + 1 + lane; j < n; j += 64) {
        const double vj = v[j];
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[q] += row[q][j] * vj;
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const double a = wave_sum(acc[q]);
        if (lane == 0 && i0 + q * WAVES < n) w[i0 + q * WAVES] = tk * a;
      }
    }
    __syncthreads();
    // every wave forms p.v by itself (the same sum in the same order: the same bits), then
    // A22 -= v w^T + w v^T with w = p - (tau/2)(p.v) v formed where it is used; the two products are added
    // before they are subtracted, so (i, j) and (j, i) get the same bits
    double pv = 0.0;
    for (int j = k + 1 + lane; j < n; j += 64) pv += w[j] * v[j];
    const double kk = 0.5 * tk * wave_sum(pv);
    for (int i0 = k + 1 + wave; i0 < n; i0 += 4 * WAVES) {
      double* row[4];
      double vi[4], wi[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int i = i0 + q * WAVES < n ? i0 + q * WAVES : n - 1;
        row[q] = A + (size_t)i * n; vi[q] = v[i]; wi[q] = __dsub_rn(w[i], __dmul_rn(kk, v[i]));
      }
      for (int j = k + 1 + lane; j < n; j += 64) {
        const double vj = v[j], wj = __dsub_rn(w[j], __dmul_rn(kk, vj));
        double a[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) a[q] = row[q][j];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const double p1 = __dmul_rn(vi[q], wj), p2 = __dmul_rn(wi[q], vj);
          if (i0 + q * WAVES < n) row[q][j] = __dsub_rn(a[q], __dadd_rn(p1, p2));
        }
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    if (n >= 2) { d[n - 2] = A[(size_t)(n - 2) * n + n - 2]; e[n - 2] = A[(size_t)(n - 2) * n + n - 1]; }
    d[n - 1] = A[(size_t)(n - 1) * n + n - 1];
    e[n - 1] = 0.0;
  }
  __syncthreads();

  // ---- Zt = Q^T = H_{n-3} ... H_0, accumulated from the last reflector: Zt <- Zt H_k ----
  // One barrier per reflector: v_k sits in one of two LDS buffers (v, w) while the next one is fetched into the other.
  {
    int kq = n - 3;
    while (kq >= 0 && tau[kq] == 0.0) --kq;                   // uniform
    if (kq >= 0)
      for (int j = kq + 1 + tid; j < n; j += THREADS) v[j] = A[(size_t)kq * n + j];
    __syncthreads();
    for (int par = 0; kq >= 0; par ^= 1) {
      const int k = kq;
      const double tk = tau[k];
      const double* vk = par ? w : v;
      double* vnext = par ? v : w;
      kq = k - 1;
      while (kq >= 0 && tau[kq] == 0.0) --kq;                 // the next reflector that does anything (uniform)
      if (kq >= 0)
        for (int j = kq + 1 + tid; j < n; j += THREADS) vnext[j] = A[(size_t)kq * n + j];
      for (int i0 = k + 1 + wave; i0 < n; i0 += 4 * WAVES) {
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
        double* row[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) row[q] = Zt + (size_t)(i0 + q * WAVES < n ? i0 + q * WAVES : n - 1) * n;
        for (int j = k + 1 + lane; j < n; j += 64) {
          const double vj = vk[j];
#pragma unroll
          for (int q = 0; q < 4; ++q) acc[q] += row[q][j] * vj;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[q] = tk * wave_sum(acc[q]);
        for (int j = k + 1 + lane; j < n; j += 64) {
          const double vj = vk[j];
          double a[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) a[q] = row[q][j];
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (i0 + q * WAVES < n) row[q][j] = a[q] - acc[q] * vj;
        }
      }
      __syncthreads();
    }
  }

  // ---- implicit QL with Wilkinson's shift ----
  // The last wave generates the plane rotations of a QL step (a sequential recurrence over the tridiagonal
  // matrix alone) while threads k < n apply the previous step's rotations to Zt: two rotation buffers in
  // LDS (the second one reuses v and w), one barrier per step.  All 64 lanes of the generating wave compute
  // the same values, so that its control flow is scalar; the entries of d and e a step walks over are read
  // 64 at a time, one per lane, and handed to the recurrence by v_readlane: no LDS round trip on the
  // dependent chain.
  __shared__ int meta[2][4];               // {0: rotations of rows lo..hi | 1: finished with status lo, lo, hi}
  const bool producer = wave == WAVES - 1;
  int l = 0, iter = 0;                     // producer state (uniform over the wave)
  double tst = 0.0;                        // largest |d| + |e| seen so far: what "negligible" is measured against
  auto lane_value = [](double x, int src) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), src);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), src);
    return __hiloint2double(hi, lo);
  };
  auto produce = [&](int buf) {
    double* pc = buf ? v : rc;
    double* ps = buf ? w : rs;
    for (;;) {
      if (l >= n) { if (lane == 0) { meta[buf][0] = 1; meta[buf][1] = 0; } return; }
      const double t = fabs(d[l]) + fabs(e[l]);
      tst = t > tst ? t : tst;
      int mm = n - 1;                      // first index >= l whose e is negligible (e[n-1] = 0 counts)
      for (int base = l; base < n; base += 64) {
        const int idx = base + lane;
        const bool stop = idx >= n - 1 || fabs(e[idx < n ? idx : n - 1]) <= 1.1102230246251565e-16 * tst;
        const unsigned long long hit = __ballot(stop);
        if (hit) { mm = base + __ffsll((long long)hit) - 1; break; }
      }
      mm = __builtin_amdgcn_readfirstlane(mm);
      if (mm == l) { ++l; iter = 0; continue; }                              // d[l] is an eigenvalue
      if (iter++ >= kMaxQlIterations) { if (lane == 0) { meta[buf][0] = 1; meta[buf][1] = 1; } return; }
      double g = (d[l + 1] - d[l]) / (2.0 * e[l]);
      const double r0 = sqrt(g * g + 1.0);
      g = d[mm] - d[l] + e[l] / (g + (g >= 0.0 ? r0 : -r0));
      double sn = 1.0, cs = 1.0, p = 0.0, dip1 = d[mm];
      int i = mm - 1;
      bool under = false;
      while (i >= l && !under) {
        const int cnt = __builtin_amdgcn_readfirstlane(i - l + 1 < 64 ? i - l + 1 : 64);
        const int mine = i - lane >= 0 ? i - lane : 0;
        const double dl = d[mine], el = e[mine];          // this step writes d and e above index i only
        for (int q = 0; q < cnt; ++q, --i) {
          const double ei = lane_value(el, q), di = lane_value(dl, q);
          const double f = sn * ei, b = cs * ei;
          const double h = f * f + g * g;
          if (__builtin_amdgcn_readfirstlane((int)(h == 0.0))) {
            if (lane == 0) { e[i + 1] = 0.0; d[i + 1] = dip1 - p; e[mm] = 0.0; }
            under = true;
            break;
          }
          const double inv = rsqrt(h);
          sn = f * inv; cs = g * inv;
          const double g2 = dip1 - p;
          const double r2 = (di - g2) * sn + 2.0 * cs * b;
          p = sn * r2;
          g = cs * r2 - b;
          if (lane == 0) { e[i + 1] = h * inv; d[i + 1] = g2 + p; pc[i] = cs; ps[i] = sn; }
          dip1 = di;
        }
      }
      if (!under && lane == 0) { d[l] -= p; e[l] = g; e[mm] = 0.0; }
      const int lo = under ? i + 1 : l, hi = mm - 1;
      if (hi < lo) continue;
      if (lane == 0) { meta[buf][0] = 0; meta[buf][1] = lo; meta[buf][2] = hi; }
      return;
    }
  };
  if (producer) produce(0);
  __syncthreads();
  int status = 0;
  for (int cur = 0;; cur ^= 1) {
    const int kind = meta[cur][0], lo = meta[cur][1], hi = meta[cur][2];
    if (kind != 0) { status = lo; break; }                                   // uniform
    if (producer) produce(cur ^ 1);
    if (tid < n) {
      const double* pc = cur ? v : rc;
      const double* ps = cur ? w : rs;
      double carry = Zt[(size_t)(hi + 1) * n + tid];
      for (int i = hi; i >= lo; i -= 8) {
        double z[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) z[q] = Zt[(size_t)(i - q >= lo ? i - q : lo) * n + tid];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          if (i - q >= lo) {
            const double cs = pc[i - q], sn = ps[i - q];
            Zt[(size_t)(i - q + 1) * n + tid] = sn * z[q] + cs * carry;
            carry = cs * z[q] - sn * carry;
          }
        }
      }
      Zt[(size_t)lo * n + tid] = carry;
    }
    __syncthreads();
  }
  __syncthreads();

  // ascending order by rank (ties broken by index), eigenvectors as columns of U
  for (int i = tid; i < n; i += THREADS) {
    const double di = d[i];
    int rank = 0;
    for (int j = 0; j < n; ++j) {
      const double dj = d[j];
      rank += (dj < di || (dj == di && j < i)) ? 1 : 0;
    }
    D[rank] = di * up;
    rank_of[i] = (short)rank;
  }
  __syncthreads();
  for (int el = tid; el < n * n; el += THREADS) {
    const int i = el / n, k = el % n;
    U[(size_t)k * n + rank_of[i]] = Zt[(size_t)i * n + k];
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
  const size_t ws_stride = eigh_workspace(m) / sizeof(double);      // doubles per problem
  if (m >= kEighTridiagonalFrom) {
    hipLaunchKernelGGL(tridiag_eigh_kernel<1024>, dim3(batch), dim3(1024), 0, s, K, m, D, U, info, ws, ws_stride);
    return hipGetLastError();
  }
  if (2 * one <= kEighLdsBytes) smem = 2 * one;                       // both in LDS
  else if (one <= kEighLdsBytes) { smem = one; gV = ws; }             // work matrix in LDS, eigenvectors in L2
  else { smem = 0; gA = ws; gV = ws + (size_t)n * (n + 1); }
  return n <= 32 ? launch_jacobi<256>(K, m, batch, D, U, info, smem, gA, gV, ws_stride, s)
                 : launch_jacobi<1024>(K, m, batch, D, U, info, smem, gA, gV, ws_stride, s);
}

hipError_t launch_eigh_solve(const EighSolveArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(eigh_solve_kernel, dim3(a.batch), dim3(kSolveThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace isopo
