// Ghost form of the layer's Gram matrix.  Each token gradient is the rank-one
// matrix delta_t x_t^T (efficient-implementation paragraph), so
//     <g^(t), g^(s)> = (x_t . x_s)(delta_t . delta_s)
// (its t = s case is eq. (two)), and summing over the tokens of two sequences
//     K_ij = sum_{t in i} sum_{s in j} (x_t . x_s)(delta_t . delta_s)
// without ever forming a per-sequence gradient.
//
// Two kernels.  fp32 inputs: one workgroup takes a 64x64 block of token pairs (bt <= bs); each of its
// four waves forms a 32x32 block of P = X X^T and Q = Delta Delta^T on the matrix cores (the reduction
// index is the fast index of both operands, so fragments are plain 16-byte loads).  bf16 inputs: a
// 128x128 block per workgroup, staged through LDS (further down).  Both multiply P and Q element-wise in
// registers and reduce the products by (sequence of t, sequence of s).  Only token pairs t <= s are
// used; a pair t < s inside one sequence counts twice.  Segment sums go to an fp64 upper-triangular
// accumulator with atomics (the accumulation order varies from run to run, but in fp64, so that the fp32
// K changes by at most one rounding of the final conversion).
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

// ---- bf16, LDS-tiled ---------------------------------------------------------------------------------
// One workgroup takes a 128x128 block of token pairs (tile ti <= tj).  The 128 + 128 token rows are
// streamed global -> LDS in 64-feature slices (row-contiguous DMA, 16-byte columns XOR-swizzled with the
// row so that the row-per-lane fragment reads spread over the banks) through a four-stage ring, first
// over the d_in features of X (P), then over the d_out features of Delta (Q).  Each wave owns a 64x64
// sub-block: two row fragments and two column fragments feed four MFMAs per 16-feature step.
typedef void __attribute__((address_space(3)))* lds_void_ptr;
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef v4u __attribute__((address_space(3)))* lds_v4u_ptr;

constexpr int kGT = 128;                 // tokens per tile side
constexpr int kGStages = 4;
constexpr int kGStageBytes = 2 * kGT * 128;      // 256 rows x 128 bytes

__device__ __forceinline__ void ghost_load_lds16(const void* gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(gptr) : "memory");
}

// acc[bi][bj] (32x32: rows = tokens of tile ti, columns = tokens of tile tj) += over the d features of M
__device__ __forceinline__ void ghost_product_pass(const unsigned short* __restrict__ M, int d, int n_tokens, int ti,
                                                   int tj, unsigned smem_base, int lane, int wave,
                                                   f32x16 (&acc)[2][2]) {
  constexpr int KW = 64, LPW = 8;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int wi = wave >> 1, wj = wave & 1;
  const int n_super = (d + KW - 1) / KW;
  const char* src[LPW];
  int vec_off[LPW];
#pragma unroll
  for (int q = 0; q < LPW; ++q) {
    const int row = (wave * LPW + q) * 8 + lane / 8;               // 0..255: tile ti's rows, then tile tj's
    int tok = row < kGT ? ti * kGT + row : tj * kGT + (row - kGT);
    if (tok >= n_tokens) tok = n_tokens - 1;                        // rows past the end are masked in the epilogue
    src[q] = reinterpret_cast<const char*>(M + (size_t)tok * d);
    vec_off[q] = ((lane % 8) ^ ((row >> 1) & 7)) * 16;
  }
  auto issue = [&](int k) {
#pragma unroll
    for (int q = 0; q < LPW; ++q) {
      long long byte = (long long)k * 128 + vec_off[q];
      const long long last = ((long long)d - 8) * 2;
      if (byte > last) byte = last;                                 // tail and look-ahead: stays inside the row
      ghost_load_lds16(src[q] + byte, smem_base + (unsigned)(k % kGStages) * kGStageBytes +
                                          (unsigned)(wave_s * LPW + q) * 1024);
    }
  };
#pragma unroll
  for (int s = 0; s < kGStages - 1; ++s) issue(s);
  const int frow = lane & 31, half = lane >> 5;
  for (int k = 0; k < n_super; ++k) {
    __builtin_amdgcn_s_waitcnt(0x0f70 | (((kGStages - 2) * LPW) & 15) | ((((kGStages - 2) * LPW) >> 4) << 14));
    __builtin_amdgcn_s_barrier();
    issue(k + kGStages - 1);
    const unsigned sb = smem_base + (unsigned)(k % kGStages) * kGStageBytes;
    const int valid = d - k * KW;
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      const int vec = st * 2 + half;
      v4u fa[2], fb[2];
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int ra = wi * 64 + b * 32 + frow, rb = kGT + wj * 64 + b * 32 + frow;
        fa[b] = *(lds_v4u_ptr)(sb + (unsigned)ra * 128 + (unsigned)((vec ^ ((ra >> 1) & 7)) * 16));
        fb[b] = *(lds_v4u_ptr)(sb + (unsigned)rb * 128 + (unsigned)((vec ^ ((rb >> 1) & 7)) * 16));
        if (valid < KW && vec * 8 >= valid) fa[b] = v4u{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
          acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[bi]),
                                                                __builtin_bit_cast(bf16x8, fb[bj]), acc[bi][bj], 0, 0, 0);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);
  __builtin_amdgcn_s_barrier();            // the ring is reused by the next pass
}

__global__ __launch_bounds__(256) void ghost_gram_tiled_kernel(const unsigned short* __restrict__ X,
                                                               const unsigned short* __restrict__ Delta,
                                                               const int32_t* __restrict__ tok_seq, int n_tokens,
                                                               int d_in, int d_out, int n_seq, int n_tiles,
                                                               double* __restrict__ K64) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const unsigned smem_base = (unsigned)(size_t)(lds_void_ptr)smem;
  int ti = 0, rem = blockIdx.x;              // blockIdx.x enumerates tile pairs (ti <= tj) row by row
  while (rem >= n_tiles - ti) { rem -= n_tiles - ti; ++ti; }
  const int tj = ti + rem;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wi = wave >> 1, wj = wave & 1;

  f32x16 P[2][2], Q[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) { P[a][b][v] = 0.f; Q[a][b][v] = 0.f; }
  ghost_product_pass(X, d_in, n_tokens, ti, tj, smem_base, lane, wave, P);
  ghost_product_pass(Delta, d_out, n_tokens, ti, tj, smem_base, lane, wave, Q);

  const int r32 = lane & 31;
#pragma unroll
  for (int bi = 0; bi < 2; ++bi) {
#pragma unroll
    for (int bj = 0; bj < 2; ++bj) {
      const int t0 = ti * kGT + wi * 64 + bi * 32, s0 = tj * kGT + wj * 64 + bj * 32;
      if (t0 >= n_tokens || s0 >= n_tokens || t0 > s0) continue;      // wave-uniform; t0 > s0: every pair has t > s
      // lane holds column s = s0 + lane%32 and rows t = t0 + acc_row(v, lane)
      const int s = s0 + r32;
      const bool s_ok = s < n_tokens;
      const int q = s_ok ? tok_seq[s] : -1;
      const int t_last = min(t0 + 31, n_tokens - 1), s_last = min(s0 + 31, n_tokens - 1);
      const int r_first = tok_seq[t0], r_last = tok_seq[t_last];
      const int q_first = tok_seq[s0], q_last = tok_seq[s_last];
      const bool uniform = (r_first == r_last) && (q_first == q_last);
      double run = 0.0;
      int run_r = -1;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int t = t0 + acc_row(v, lane);
        if (t >= n_tokens || !s_ok || t > s) continue;
        const int r = uniform ? r_first : tok_seq[t];
        const double w = (t == s) ? 1.0 : ((r == q) ? 2.0 : 1.0);
        const double h = w * (double)P[bi][bj][v] * (double)Q[bi][bj][v];
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
    if (a.bf16) {
      const int nt = (a.n_tokens + kGT - 1) / kGT;
      constexpr size_t smem = (size_t)kGStages * kGStageBytes;
      // once per process (static initialisation is thread-safe); a failure is returned by every call
      static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(ghost_gram_tiled_kernel),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (attr != hipSuccess) return attr;
      hipLaunchKernelGGL(ghost_gram_tiled_kernel, dim3((unsigned)((long long)nt * (nt + 1) / 2)), dim3(256), smem, s,
                         static_cast<const unsigned short*>(a.X), static_cast<const unsigned short*>(a.Delta), a.tok_seq,
                         a.n_tokens, a.d_in, a.d_out, a.n_seq, nt, a.K64);
    } else
      hipLaunchKernelGGL((ghost_gram_kernel<false>), dim3((unsigned)pairs), dim3(256), 0, s, a.X, a.Delta, a.tok_seq,
                         a.n_tokens, a.d_in, a.d_out, a.n_seq, (int)n_tiles, a.K64);
  }
  hipLaunchKernelGGL(ghost_finish_kernel, dim3((unsigned)((kk + 255) / 256)), dim3(256), 0, s, a.K64, a.n_seq, a.K);
  return hipGetLastError();
}

}  // namespace isopo
