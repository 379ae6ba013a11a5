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

#include <type_traits>

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
  if (r_first == r_last && q_first == q_last) {
    // one sequence pair in the whole block: one wave sum, one atomic
    double run = 0.0;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int t = t0 + acc_row(v, lane);
      if (t >= n_tokens || !s_ok || t > s) continue;
      const double w = (t == s) ? 1.0 : ((r_first == q) ? 2.0 : 1.0);
      run += w * (double)P[v] * (double)Q[v];
    }
    run = wave_sum(run);
    if (lane == 0) atomicAdd(&K64[(size_t)r_first * n_seq + q_first], run);
    return;
  }
  const int n_r = r_last - r_first + 1, n_q = q_last - q_first + 1;
  if (n_r * n_q <= 8) {
    // a few sequence boundaries cross the block: one wave sum and one atomic per (row sequence, column
    // sequence) rather than one atomic per lane and run, which would queue on K's few cache lines
    for (int r = r_first; r <= r_last; ++r) {
      double part = 0.0;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int t = t0 + acc_row(v, lane);
        if (t >= n_tokens || !s_ok || t > s || tok_seq[t] != r) continue;
        const double w = (t == s) ? 1.0 : ((r == q) ? 2.0 : 1.0);
        part += w * (double)P[v] * (double)Q[v];
      }
      for (int c = q_first; c <= q_last; ++c) {
        const double sum = wave_sum(q == c ? part : 0.0);
        if (lane == 0 && sum != 0.0) atomicAdd(&K64[(size_t)r * n_seq + c], sum);
      }
    }
    return;
  }
  // many short sequences: a lane adds each run of rows of one sequence by itself
  double run = 0.0;
  int run_r = -1;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int t = t0 + acc_row(v, lane);
    if (t >= n_tokens || !s_ok || t > s) continue;
    const int r = tok_seq[t];
    const double w = (t == s) ? 1.0 : ((r == q) ? 2.0 : 1.0);
    const double h = w * (double)P[v] * (double)Q[v];
    if (r != run_r) {
      if (run_r >= 0) atomicAdd(&K64[(size_t)run_r * n_seq + q], run);
      run_r = r;
      run = 0.0;
    }
    run += h;
  }
  if (run_r >= 0) atomicAdd(&K64[(size_t)run_r * n_seq + q], run);
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

  ghost_block_reduce(P, Q, t0, s0, lane, tok_seq, n_tokens, n_seq, K64);
}

// ---- bf16, LDS-tiled ---------------------------------------------------------------------------------
// One workgroup takes a 128x128 block of token pairs (tile ti <= tj).  The 128 + 128 token rows are
// streamed global -> LDS in 64-feature slices (row-contiguous DMA, 16-byte columns XOR-swizzled with the
// row so that the row-per-lane fragment reads spread over the banks) through a two-stage ring, first
// over the d_in features of X (P), then over the d_out features of Delta (Q).  Two workgroups share a
// compute unit (64 KiB of LDS, 128 accumulator registers per lane each): one's barrier and DMA wait
// overlap the other's MFMAs.  Each wave owns a 64x64 sub-block: two row fragments and two column
// fragments feed four MFMAs per 16-feature step.
typedef void __attribute__((address_space(3)))* lds_void_ptr;
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef v4u __attribute__((address_space(3)))* lds_v4u_ptr;

constexpr int kGT = 128;                 // tokens per tile side
constexpr int kGKW = 64;                 // features per ring stage
constexpr int kGStages = 2;
constexpr int kGRowBytes = kGKW * 2;             // LDS row pitch
constexpr int kGStageBytes = 2 * kGT * kGRowBytes;
constexpr int kGRun = 64;                        // workgroups an XCD holds at a time: 32 compute units x 2
static_assert(kGStages * kGStageBytes * 2 <= 160 * 1024, "two workgroups per compute unit share the LDS");

typedef int v4i __attribute__((ext_vector_type(4)));

// 16 bytes per lane from a buffer straight into LDS: lane l lands at lds_addr + 16 l.  Offsets at or beyond the
// descriptor's byte count are out of range: nothing is fetched and zeros arrive.
__device__ __forceinline__ void ghost_load_lds16(v4i rsrc, unsigned lds_addr, unsigned voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               : : "s"(lds_addr), "v"(voff), "s"(rsrc) : "memory");
}

// 16-byte column c of LDS row `row` holds global column c ^ ghost_swizzle(row): sixteen consecutive rows read
// at one global column then touch sixteen different groups of four banks.
__device__ __forceinline__ int ghost_swizzle(int row) {
  constexpr int cols = kGRowBytes / 16;          // 4 (64-byte rows) or 8 (128-byte rows)
  return (row >> (cols == 4 ? 2 : 1)) & (cols - 1);
}

// acc[bi][bj] (32x32: rows = tokens of tile ti, columns = tokens of tile tj) += over kGKW-feature slices
// [k_begin, k_end) of the d features of M
__device__ __forceinline__ void ghost_product_pass(const unsigned short* __restrict__ M, int d, int n_tokens, int ti,
                                                   int tj, unsigned smem_base, int lane, int wave, int k_begin,
                                                   int k_end, f32x16 (&acc)[2][2]) {
  constexpr int COLS = kGRowBytes / 16, ROWS_PER_LOAD = 64 / COLS;      // one wave-load is 1 KiB of whole rows
  constexpr int LPW = 2 * kGT / ROWS_PER_LOAD / 4;                      // wave-loads per wave and stage
  static_assert(kGStages == 2 && 4 * LPW * ROWS_PER_LOAD == 2 * kGT, "waves 0, 1 stage tile ti's rows, waves 2, 3 tile tj's");
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int wi = wave >> 1, wj = wave & 1;
  // The rows this wave stages belong to one tile; a buffer descriptor over that tile's valid rows lets the
  // loads take a 32-bit offset per lane (one addition per load and stage; 64-bit addresses clamped lane by lane
  // cost some sixty vector instructions per stage, as much issue time as the stage's MFMAs).  Rows past the
  // last token are out of range and arrive as zeros; a 16-byte column past the row's end reads into the next
  // row or out of range (the fragments of such columns are zeroed below).
  const int row0 = (wave_s < 2 ? ti : tj) * kGT;
  int rows_valid = n_tokens - row0;
  rows_valid = rows_valid < 0 ? 0 : (rows_valid > kGT ? kGT : rows_valid);
  const unsigned long long base = (unsigned long long)(M + (size_t)row0 * d);
  v4i rsrc;
  rsrc[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)base);
  rsrc[1] = __builtin_amdgcn_readfirstlane((int)((unsigned)(base >> 32) & 0xffffu));
  rsrc[2] = __builtin_amdgcn_readfirstlane((int)((unsigned)rows_valid * (unsigned)d * 2u));     // at most 128 rows of 64 Ki features
  rsrc[3] = 0x00020000;
  unsigned voff[LPW];
#pragma unroll
  for (int q = 0; q < LPW; ++q) {
    const int row = (wave * LPW + q) * ROWS_PER_LOAD + lane / COLS;  // 0..255: tile ti's rows, then tile tj's
    voff[q] = (unsigned)(row & (kGT - 1)) * (unsigned)d * 2u + (unsigned)k_begin * kGRowBytes +
              (unsigned)(((lane % COLS) ^ ghost_swizzle(row)) * 16);
  }
  // the next slice of kGKW features into ring stage `stage` (look-ahead slices past k_end are never read)
  auto issue = [&](int stage) {
#pragma unroll
    for (int q = 0; q < LPW; ++q) {
      ghost_load_lds16(rsrc, smem_base + (unsigned)stage * kGStageBytes + (unsigned)(wave_s * LPW + q) * 1024, voff[q]);
      voff[q] += kGRowBytes;
    }
  };
  issue(0);
  const int frow = lane & 31, half = lane >> 5;
  // fragment addresses of the first 32-row block in stage 0: the second block (32 rows on, the same swizzle) and
  // stage 1 are immediate offsets away
  constexpr int KS = kGKW / 16;
  static_assert(COLS == 8, "rows 32 apart share their swizzle");
  unsigned ada[KS], adb[KS];
#pragma unroll
  for (int st = 0; st < KS; ++st) {
    const int vec = st * 2 + half;
    const int ra = wi * 64 + frow, rb = kGT + wj * 64 + frow;
    ada[st] = smem_base + (unsigned)ra * kGRowBytes + (unsigned)((vec ^ ghost_swizzle(ra)) * 16);
    adb[st] = smem_base + (unsigned)rb * kGRowBytes + (unsigned)((vec ^ ghost_swizzle(rb)) * 16);
  }
  // TAIL: the last slice of a feature count that is no multiple of kGKW (its own body, so that the full slices
  // carry no selects)
  auto stage_body = [&](int k, auto stage_c, auto tail_c) {
    constexpr int STAGE = decltype(stage_c)::value;
    constexpr bool TAIL = decltype(tail_c)::value;
    __builtin_amdgcn_s_waitcnt(0x0f70);      // this wave's part of slice k has landed; the barrier makes it everyone's
    __builtin_amdgcn_s_barrier();
    issue(STAGE ^ 1);
    // every 16-feature step has its own fragment registers, and the reads of step st + 1 are issued ahead of
    // the MFMAs of step st: with one or two waves per SIMD nothing else hides the LDS latency
    v4u fa[KS][2], fb[KS][2];
#pragma unroll
    for (int st = 0; st < KS; ++st)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        fa[st][b] = *(lds_v4u_ptr)(ada[st] + (unsigned)(STAGE * kGStageBytes + b * 32 * kGRowBytes));
        fb[st][b] = *(lds_v4u_ptr)(adb[st] + (unsigned)(STAGE * kGStageBytes + b * 32 * kGRowBytes));
      }
    if constexpr (TAIL) {
      const int valid = d - k * kGKW;            // features of this slice that exist
#pragma unroll
      for (int st = 0; st < KS; ++st)
#pragma unroll
        for (int b = 0; b < 2; ++b)
          if ((st * 2 + half) * 8 >= valid) { fa[st][b] = v4u{0u, 0u, 0u, 0u}; fb[st][b] = v4u{0u, 0u, 0u, 0u}; }
    }
#pragma unroll
    for (int st = 0; st < KS; ++st)
#pragma unroll
      for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
          acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[st][bi]),
                                                                __builtin_bit_cast(bf16x8, fb[st][bj]), acc[bi][bj], 0, 0, 0);
    // order: reads of steps 0 and 1, then four MFMAs and the next step's four reads in turn
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
    for (int st = 0; st < KS; ++st) {
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      if (st + 2 < KS) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
    }
  };
  constexpr std::integral_constant<int, 0> s0{};
  constexpr std::integral_constant<int, 1> s1{};
  int k_full = d / kGKW;                       // slices [k_begin, k_full) are whole; at most one more follows
  k_full = k_full < k_begin ? k_begin : (k_full > k_end ? k_end : k_full);
  int k = k_begin;
  for (; k + 1 < k_full; k += 2) {
    stage_body(k, s0, std::false_type{});
    stage_body(k + 1, s1, std::false_type{});
  }
  if (k < k_full) {
    stage_body(k, s0, std::false_type{});
    if (k + 1 < k_end) stage_body(k + 1, s1, std::true_type{});
  } else if (k < k_end) {
    stage_body(k, s0, std::true_type{});
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);
  __builtin_amdgcn_s_barrier();            // the ring is reused by the next pass
}

// Order of the tile pairs (ti <= tj) in the unsplit launch: bands of kGBand tile rows, column by column inside
// a band, so that consecutive pairs form compact blocks of the triangle.
constexpr int kGBand = 8;
__device__ __forceinline__ void ghost_pair_at(long long pos, int n_tiles, int& ti, int& tj) {
  int b0 = 0, h;
  for (;;) {
    h = min(kGBand, n_tiles - b0);                                           // rows of this band
    const long long cnt = (long long)h * (h + 1) / 2 + (long long)h * (n_tiles - b0 - h);
    if (pos < cnt) break;
    pos -= cnt;
    b0 += kGBand;
  }
  const int head = h * (h + 1) / 2;               // the band's first h columns hold 1, 2, ..., h pairs
  if (pos < head) {
    int j = 0;
    while (pos >= j + 1) { pos -= j + 1; ++j; }
    tj = b0 + j;
    ti = b0 + (int)pos;
  } else {
    pos -= head;
    tj = b0 + h + (int)(pos / h);
    ti = b0 + (int)(pos % h);
  }
}

constexpr int kGBlockFloats = 16 * 64;            // one wave's 32x32 accumulator block
constexpr int kGTileFloats = 16 * kGBlockFloats;  // the 16 blocks of a 128x128 tile

// SPLIT = false: one workgroup per tile pair walks all features and adds its pairs to K64; `count` is the
// length of the runs of consecutive pairs an XCD takes.
// SPLIT = true (few tile pairs, a short microbatch): the 64-feature slices of both operands are cut into
// `count` ranges and workgroup (pair, a) forms the parts P_a, Q_a of the two products over range a only; the
// parts go to `parts` [pair][a][P, Q][block][lane][v] in fp32, and ghost_gram_parts_kernel sums them before
// the Hadamard product, which is not linear in the ranges.
template <bool SPLIT>
__global__ __launch_bounds__(256, 2) void ghost_gram_tiled_kernel(const unsigned short* __restrict__ X,
                                                               const unsigned short* __restrict__ Delta,
                                                               const int32_t* __restrict__ tok_seq, int n_tokens,
                                                               int d_in, int d_out, int n_seq, int n_tiles,
                                                               int count, float* __restrict__ parts,
                                                               double* __restrict__ K64) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int split = SPLIT ? count : 1;
  const unsigned smem_base = (unsigned)(size_t)(lds_void_ptr)smem;
  int fa = 0, ti = 0, tj, part = 0;
  if constexpr (SPLIT) {
    // Workgroups go to the eight XCDs round robin.  XCD x takes the x-th eighth of the range-major list of
    // (range, tile pair): the columns of X and Delta that a range covers then pass through one or two L2s,
    // not all eight.
    const int x = blockIdx.x & 7, e = blockIdx.x >> 3;
    const int n_pairs = n_tiles * (n_tiles + 1) / 2, total = n_pairs * split;       // at most 512
    const int first = x * total / 8;
    if (e >= (x + 1) * total / 8 - first) return;                    // the grid is padded to 8 * ceil(total / 8)
    fa = (first + e) / n_pairs;
    int rem = (first + e) % n_pairs;
    part = rem * split + fa;
    while (rem >= n_tiles - ti) { rem -= n_tiles - ti; ++ti; }       // tile pairs (ti <= tj) row by row
    tj = ti + rem;
  } else {
    // Workgroups go to the eight XCDs round robin.  XCD x takes the pair list in runs of `count` consecutive
    // pairs (at most kGRun, what its 32 compute units hold at a time): with the banded order a run covers
    // about 8 x 8 tiles, so the workgroups that share an L2 stream 16 row tiles between them rather than 65.
    const long long e = blockIdx.x >> 3, x = blockIdx.x & 7, run = count;
    const long long pos = ((e / run) * 8 + x) * run + e % run;
    if (pos >= (long long)n_tiles * (n_tiles + 1) / 2) return;       // the grid is padded to whole runs
    ghost_pair_at(pos, n_tiles, ti, tj);
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wi = wave >> 1, wj = wave & 1;

  f32x16 P[2][2], Q[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) { P[a][b][v] = 0.f; Q[a][b][v] = 0.f; }
  const int nx = (d_in + kGKW - 1) / kGKW, nd = (d_out + kGKW - 1) / kGKW;       // ring stages
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
        float* dst = parts + (size_t)part * (2 * kGTileFloats) + (size_t)(wave * 4 + bi * 2 + bj) * kGBlockFloats;
        // a lane's sixteen values are contiguous: four 16-byte stores, a wave covers 4 KiB without gaps
#pragma unroll
        for (int v = 0; v < 16; v += 4) {
          *reinterpret_cast<f32x4*>(dst + lane * 16 + v) =
              f32x4{P[bi][bj][v], P[bi][bj][v + 1], P[bi][bj][v + 2], P[bi][bj][v + 3]};
          *reinterpret_cast<f32x4*>(dst + kGTileFloats + lane * 16 + v) =
              f32x4{Q[bi][bj][v], Q[bi][bj][v + 1], Q[bi][bj][v + 2], Q[bi][bj][v + 3]};
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
    for (int v = 0; v < 16; v += 4) {
      const f32x4 p4 = *reinterpret_cast<const f32x4*>(src + lane * 16 + v);
      const f32x4 q4 = *reinterpret_cast<const f32x4*>(src + kGTileFloats + lane * 16 + v);
#pragma unroll
      for (int u = 0; u < 4; ++u) { P[v + u] += p4[u]; Q[v + u] += q4[u]; }
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
        const unsigned grid = 8 * ((n_pairs * split + 7) / 8);
        hipLaunchKernelGGL(ghost_gram_tiled_kernel<true>, dim3(grid), dim3(256), smem, s, Xb, Db, a.tok_seq,
                           a.n_tokens, a.d_in, a.d_out, a.n_seq, nt, split, a.parts, a.K64);
        hipLaunchKernelGGL(ghost_gram_parts_kernel, dim3(n_pairs * 16), dim3(256), 0, s, a.parts, a.tok_seq, a.n_tokens,
                           a.n_seq, nt, split, a.K64);
      } else {
        // a multiple of eight runs of equal length, so that every XCD gets the same number of pairs
        const unsigned n_runs = 8 * ((n_pairs + 8 * kGRun - 1) / (8 * kGRun));
        const unsigned run = (n_pairs + n_runs - 1) / n_runs;
        hipLaunchKernelGGL(ghost_gram_tiled_kernel<false>, dim3(n_runs * run), dim3(256), smem, s, Xb, Db, a.tok_seq,
                           a.n_tokens, a.d_in, a.d_out, a.n_seq, nt, (int)run, static_cast<float*>(nullptr), a.K64);
      }
    } else
      hipLaunchKernelGGL((ghost_gram_kernel<false>), dim3((unsigned)pairs), dim3(256), 0, s, a.X, a.Delta, a.tok_seq,
                         a.n_tokens, a.d_in, a.d_out, a.n_seq, (int)n_tiles, a.K64);
  }
  hipLaunchKernelGGL(ghost_finish_kernel, dim3((unsigned)((kk + 255) / 256)), dim3(256), 0, s, a.K64, a.n_seq, a.K);
  return hipGetLastError();
}

}  // namespace isopo
