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

// acc[bi][bj] (32x32: rows = tokens of tile ti, columns = tokens of tile tj) += over 64-feature slices
// [k_begin, k_end) of the d features of M
__device__ __forceinline__ void ghost_product_pass(const unsigned short* __restrict__ M, int d, int n_tokens, int ti,
                                                   int tj, unsigned smem_base, int lane, int wave, int k_begin,
                                                   int k_end, f32x16 (&acc)[2][2]) {
  constexpr int KW = 64, LPW = 8;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int wi = wave >> 1, wj = wave & 1;
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
      ghost_load_lds16(src[q] + byte, smem_base + (unsigned)((k - k_begin) % kGStages) * kGStageBytes +
                                          (unsigned)(wave_s * LPW + q) * 1024);
    }
  };
#pragma unroll
  for (int s = 0; s < kGStages - 1; ++s) issue(k_begin + s);
  const int frow = lane & 31, half = lane >> 5;
  for (int k = k_begin; k < k_end; ++k) {
    __builtin_amdgcn_s_waitcnt(0x0f70 | (((kGStages - 2) * LPW) & 15) | ((((kGStages - 2) * LPW) >> 4) << 14));
    __builtin_amdgcn_s_barrier();
    issue(k + kGStages - 1);
    const unsigned sb = smem_base + (unsigned)((k - k_begin) % kGStages) * kGStageBytes;
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

// One 32x32 block of the token-pair matrix: rows t0.., columns s0.. .  False when the block lies past the last
// token or wholly below the diagonal (every pair has t > s); wave-uniform.
__device__ __forceinline__ bool ghost_block_live(int t0, int s0, int n_tokens) {
  return t0 < n_tokens && s0 < n_tokens && t0 <= s0;
}

// K64[seq(t)][seq(s)] += w P Q over the pairs t <= s of a live 32x32 block (w = 2 for the off-diagonal pairs of one
// sequence, which stand for their mirror images too).  Lane holds column s = s0 + lane%32 and rows
// t = t0 + acc_row(v, lane).
__device__ __forceinline__ void ghost_block_reduce(const f32x16& P, const f32x16& Q, int t0, int s0, int lane,
                                                   const int32_t* __restrict__ tok_seq, int n_tokens, int n_seq,
                                                   double* __restrict__ K64) {
  const int s = s0 + (lane & 31);
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

constexpr int kGBlockFloats = 16 * 64;            // one wave's 32x32 accumulator block
constexpr int kGTileFloats = 16 * kGBlockFloats;  // the 16 blocks of a 128x128 tile

// SPLIT = false: one workgroup per tile pair walks all features and adds its pairs to K64.
// SPLIT = true (few tile pairs, a short microbatch): the 64-feature slices of both operands are cut into `split`
// ranges and workgroup (pair, a) forms the parts P_a, Q_a of the two products over range a only; the parts go to
// `parts` [pair][a][P, Q][block][v][lane] in fp32, and ghost_gram_parts_kernel sums them before the Hadamard
// product, which is not linear in the ranges.
template <bool SPLIT>
__global__ __launch_bounds__(256) void ghost_gram_tiled_kernel(const unsigned short* __restrict__ X,
                                                               const unsigned short* __restrict__ Delta,
                                                               const int32_t* __restrict__ tok_seq, int n_tokens,
                                                               int d_in, int d_out, int n_seq, int n_tiles,
                                                               int split, float* __restrict__ parts,
                                                               double* __restrict__ K64) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const unsigned smem_base = (unsigned)(size_t)(lds_void_ptr)smem;
  const int fa = SPLIT ? (int)(blockIdx.x % (unsigned)split) : 0;
  int ti = 0, rem = SPLIT ? (int)(blockIdx.x / (unsigned)split) : (int)blockIdx.x;   // tile pairs (ti <= tj) row by row
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
  const int nx = (d_in + 63) / 64, nd = (d_out + 63) / 64;       // 64-feature slices
  if constexpr (SPLIT) {
    ghost_product_pass(X, d_in, n_tokens, ti, tj, smem_base, lane, wave, (int)((long long)nx * fa / split),
                       (int)((long long)nx * (fa + 1) / split), P);
    ghost_product_pass(Delta, d_out, n_tokens, ti, tj, smem_base, lane, wave, (int)((long long)nd * fa / split),
                       (int)((long long)nd * (fa + 1) / split), Q);
  } else {
    ghost_product_pass(X, d_in, n_tokens, ti, tj, smem_base, lane, wave, 0, nx, P);
    ghost_product_pass(Delta, d_out, n_tokens, ti, tj, smem_base, lane, wave, 0, nd, Q);
  }

#pragma unroll
  for (int bi = 0; bi < 2; ++bi) {
#pragma unroll
    for (int bj = 0; bj < 2; ++bj) {
      const int t0 = ti * kGT + wi * 64 + bi * 32, s0 = tj * kGT + wj * 64 + bj * 32;
      if (!ghost_block_live(t0, s0, n_tokens)) continue;
      if constexpr (SPLIT) {
        float* dst = parts + (size_t)blockIdx.x * (2 * kGTileFloats) + (size_t)(wave * 4 + bi * 2 + bj) * kGBlockFloats;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          dst[v * 64 + lane] = P[bi][bj][v];
          dst[kGTileFloats + v * 64 + lane] = Q[bi][bj][v];
        }
      } else {
        ghost_block_reduce(P[bi][bj], Q[bi][bj], t0, s0, lane, tok_seq, n_tokens, n_seq, K64);
      }
    }
  }
}

// Second step of the split launch: one workgroup per (tile pair, 32x32 block).  Wave w sums the parts
// a = w, w + 4, ... of P and of Q; the four partial sums meet in LDS and wave 0 forms the products.
__global__ __launch_bounds__(256) void ghost_gram_parts_kernel(const float* __restrict__ parts,
                                                               const int32_t* __restrict__ tok_seq, int n_tokens,
                                                               int n_seq, int n_tiles, int split,
                                                               double* __restrict__ K64) {
  __shared__ float sums[4][2][kGBlockFloats];
  const int blk = blockIdx.x & 15;                 // wave * 4 + bi * 2 + bj of the first step
  int ti = 0, rem = blockIdx.x >> 4;
  while (rem >= n_tiles - ti) { rem -= n_tiles - ti; ++ti; }
  const int tj = ti + rem;
  const int w1 = blk >> 2, bi = (blk >> 1) & 1, bj = blk & 1;
  const int t0 = ti * kGT + (w1 >> 1) * 64 + bi * 32, s0 = tj * kGT + (w1 & 1) * 64 + bj * 32;
  if (!ghost_block_live(t0, s0, n_tokens)) return;          // uniform over the workgroup
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  f32x16 P, Q;
#pragma unroll
  for (int v = 0; v < 16; ++v) { P[v] = 0.f; Q[v] = 0.f; }
  for (int a = wave; a < split; a += 4) {
    const float* src = parts + ((size_t)(blockIdx.x >> 4) * split + a) * (2 * kGTileFloats) + (size_t)blk * kGBlockFloats;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      P[v] += src[v * 64 + lane];
      Q[v] += src[kGTileFloats + v * 64 + lane];
    }
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    sums[wave][0][v * 64 + lane] = P[v];
    sums[wave][1][v * 64 + lane] = Q[v];
  }
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    P[v] = (sums[0][0][v * 64 + lane] + sums[1][0][v * 64 + lane]) + (sums[2][0][v * 64 + lane] + sums[3][0][v * 64 + lane]);
    Q[v] = (sums[0][1][v * 64 + lane] + sums[1][1][v * 64 + lane]) + (sums[2][1][v * 64 + lane] + sums[3][1][v * 64 + lane]);
  }
  ghost_block_reduce(P, Q, t0, s0, lane, tok_seq, n_tokens, n_seq, K64);
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
      static const hipError_t attr = [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ghost_gram_tiled_kernel<false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        return hipFuncSetAttribute(reinterpret_cast<const void*>(ghost_gram_tiled_kernel<true>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      }();
      if (attr != hipSuccess) return attr;
      const int split = ghost_feature_split(a.n_tokens, a.d_in, a.d_out);
      const unsigned n_pairs = (unsigned)((long long)nt * (nt + 1) / 2);
      const unsigned short* Xb = static_cast<const unsigned short*>(a.X);
      const unsigned short* Db = static_cast<const unsigned short*>(a.Delta);
      if (split > 1) {
        if (!a.parts) return hipErrorInvalidValue;
        hipLaunchKernelGGL(ghost_gram_tiled_kernel<true>, dim3(n_pairs * split), dim3(256), smem, s, Xb, Db, a.tok_seq,
                           a.n_tokens, a.d_in, a.d_out, a.n_seq, nt, split, a.parts, a.K64);
        hipLaunchKernelGGL(ghost_gram_parts_kernel, dim3(n_pairs * 16), dim3(256), 0, s, a.parts, a.tok_seq, a.n_tokens,
                           a.n_seq, nt, split, a.K64);
      } else {
        hipLaunchKernelGGL(ghost_gram_tiled_kernel<false>, dim3(n_pairs), dim3(256), smem, s, Xb, Db, a.tok_seq,
                           a.n_tokens, a.d_in, a.d_out, a.n_seq, nt, 1, static_cast<float*>(nullptr), a.K64);
      }
    } else
      hipLaunchKernelGGL((ghost_gram_kernel<false>), dim3((unsigned)pairs), dim3(256), 0, s, a.X, a.Delta, a.tok_seq,
                         a.n_tokens, a.d_in, a.d_out, a.n_seq, (int)n_tiles, a.K64);
  }
  hipLaunchKernelGGL(ghost_finish_kernel, dim3((unsigned)((kk + 255) / 256)), dim3(256), 0, s, a.K64, a.n_seq, a.K);
  return hipGetLastError();
}

}  // namespace isopo
