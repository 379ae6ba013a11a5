// Token-reduction contraction on the matrix cores, fp32 inputs:
//     out[o][k] = sum_t scale(t) * Delta[t][o] * X[t][k]
// which is the per-sequence log-probability gradient G_i = Delta_i^T X_i of both
// hook listings (`grad_out.T @ act_in`) when t runs over one sequence, and the
// weighted contraction dW = Delta^T diag(c_tok) X (`grad += advantages[i] *
// scale_i * seq_logprob_grad`) when t runs over all tokens.  (bf16 inputs, the
// benchmark's case, take the streaming kernel in seq_grad_stream.hip.)
//
// Both operands are token-major: the reduction index is the slow index of X and
// of Delta.  Tiles are staged in LDS as [token][feature], exactly as they lie in
// HBM (coalesced 16-byte loads along the feature axis).  The fp32 MFMA takes one
// value per lane, so a plain 32-bit LDS read already has the register layout.
//
// Work item = (sequence range, 2-D tile of the [d_out, d_in] output).  The
// K-loop walks the tokens of the range sequence by sequence, BK rows at a time;
// the last block of a sequence is zero-filled, so ragged lengths need no
// host-side padding.
#include "common.h"
#include "kernels.h"

namespace isopo {
namespace {

struct SeqGradParams {
  const void* X;
  const void* Delta;
  const int32_t* off;
  const float* c;
  void* out;
  int d_in, d_out, n_seq;
  int row0, row_end;
  int out_row0;
  long long out_seq_stride;
  float beta;
  int tiles_m, tiles_n;
  unsigned n_blocks;
};

template <int BM, int BN, int BK, int PAD, bool WEIGHTED>
__global__ __launch_bounds__(256) void seq_grad_kernel(SeqGradParams p) {
  typedef float T;
  constexpr int kVec = 4;                        // elements per 16-byte vector
  constexpr int WM = BM / 2, WN = BN / 2;        // 2x2 waves
  constexpr int FM = WM / 32, FN = WN / 32;      // 32x32 MFMA blocks per wave
  constexpr int PA = BM + PAD, PB = BN + PAD;    // LDS row pitch in elements
  constexpr int VA = BM / kVec, VB = BN / kVec;  // 16-byte vectors per tile row
  constexpr int RA = 256 / VA, RB = 256 / VB;    // tile rows covered per pass of the workgroup
  constexpr int NA = BK / RA, NB = BK / RB;      // passes
  static_assert(256 % VA == 0 && 256 % VB == 0 && BK % RA == 0 && BK % RB == 0, "tile shape");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T* As = reinterpret_cast<T*>(smem);            // [2][BK][PA]
  T* Bs = As + 2 * BK * PA;                      // [2][BK][PB]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  const unsigned work = xcd_contiguous(blockIdx.x, p.n_blocks);
  const int tiles = p.tiles_m * p.tiles_n;
  const int item = work / tiles, tile = work % tiles;
  const int tile_m = tile / p.tiles_n, tile_n = tile % p.tiles_n;
  const int seq_begin = WEIGHTED ? 0 : item;
  const int seq_end = WEIGHTED ? p.n_seq : item + 1;
  const int m0 = p.row0 + tile_m * BM;           // first output row (index into d_out)
  const int n0 = tile_n * BN;                    // first output column (index into d_in)

  const T* __restrict__ Xg = static_cast<const T*>(p.X);
  const T* __restrict__ Dg = static_cast<const T*>(p.Delta);

  const int a_cv = tid % VA, a_r = tid / VA;
  const int b_cv = tid % VB, b_r = tid / VB;
  const bool a_ok = (m0 + a_cv * kVec) < p.row_end;
  const bool b_ok = (n0 + b_cv * kVec) < p.d_in;
  const T* a_src = Dg + m0 + a_cv * kVec;
  const T* b_src = Xg + n0 + b_cv * kVec;

  uint4 ra[NA], rb[NB];
  auto gload = [&](int t, int t_end) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      const int tt = t + a_r + i * RA;
      ra[i] = (a_ok && tt < t_end) ? *reinterpret_cast<const uint4*>(a_src + (size_t)tt * p.d_out)
                                   : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int tt = t + b_r + i * RB;
      rb[i] = (b_ok && tt < t_end) ? *reinterpret_cast<const uint4*>(b_src + (size_t)tt * p.d_in)
                                   : make_uint4(0, 0, 0, 0);
    }
  };
  auto sstore = [&](int buf, float scale) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      uint4 v = ra[i];
      if constexpr (WEIGHTED) {
        float4 f = __builtin_bit_cast(float4, v);
        f.x *= scale; f.y *= scale; f.z *= scale; f.w *= scale;
        v = __builtin_bit_cast(uint4, f);
      }
      *reinterpret_cast<uint4*>(As + (buf * BK + a_r + i * RA) * PA + a_cv * kVec) = v;
    }
#pragma unroll
    for (int i = 0; i < NB; ++i)
      *reinterpret_cast<uint4*>(Bs + (buf * BK + b_r + i * RB) * PB + b_cv * kVec) = rb[i];
  };

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  auto compute = [&](int buf) {
    const T* at = As + buf * BK * PA + wm * WM;
    const T* bt = Bs + buf * BK * PB + wn * WN;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      float af[FM], bf[FN];
      const int kr = kk + (lane >> 5), col = lane & 31;
#pragma unroll
      for (int i = 0; i < FM; ++i) af[i] = at[kr * PA + i * 32 + col];
#pragma unroll
      for (int j = 0; j < FN; ++j) bf[j] = bt[kr * PB + j * 32 + col];
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
  };

  // Walk the token blocks of sequences [seq_begin, seq_end).  Uniform over the workgroup.
  int seq = seq_begin - 1, t = 0, t_end = 0;
  float scale = 1.f;
  auto next_block = [&](int& bt0, int& bt1, float& bs) -> bool {
    while (t >= t_end) {
      if (++seq >= seq_end) return false;
      t = p.off[seq];
      t_end = p.off[seq + 1];
      if constexpr (WEIGHTED) scale = p.c ? p.c[seq] : 1.f;
    }
    bt0 = t;
    bt1 = t_end;
    bs = scale;
    t += BK;
    return true;
  };

  int bt0, bt1;
  float bs;
  bool have = next_block(bt0, bt1, bs);
  if (have) {
    gload(bt0, bt1);
    sstore(0, bs);
    __syncthreads();
    int cur = 0;
    while (true) {
      const bool more = next_block(bt0, bt1, bs);
      if (more) gload(bt0, bt1);
      compute(cur);
      if (more) sstore(cur ^ 1, bs);
      __syncthreads();
      if (!more) break;
      cur ^= 1;
    }
  }

  // Epilogue.  Lane l holds column (l%32) and rows acc_row(v, l) of each block.
  const int col_in_blk = lane & 31;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int n = n0 + wn * WN + j * 32 + col_in_blk;
      if (n >= p.d_in) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm * WM + i * 32 + acc_row(v, lane);
        if (m >= p.row_end) continue;
        const size_t idx = (size_t)(m - p.out_row0) * p.d_in + n;
        if constexpr (WEIGHTED) {
          float* o = static_cast<float*>(p.out) + idx;
          *o = (p.beta != 0.f ? p.beta * *o : 0.f) + acc[i][j][v];
        } else {
          static_cast<float*>(p.out)[(size_t)item * p.out_seq_stride + idx] = acc[i][j][v];
        }
      }
    }
  }
}

template <int BM, int BN, int BK, int PAD, bool WEIGHTED>
hipError_t launch_cfg(const SeqGradArgs& a, hipStream_t s) {
  SeqGradParams p;
  p.X = a.X; p.Delta = a.Delta; p.off = a.off; p.c = a.c; p.out = a.out;
  p.d_in = a.d_in; p.d_out = a.d_out; p.n_seq = a.n_seq;
  p.row0 = a.row0; p.row_end = a.row0 + a.rows; p.out_row0 = a.out_row0;
  p.out_seq_stride = a.out_seq_stride; p.beta = a.beta;
  p.tiles_m = (a.rows + BM - 1) / BM;
  p.tiles_n = (a.d_in + BN - 1) / BN;
  const long long items = WEIGHTED ? 1 : a.n_seq;
  const long long blocks = items * p.tiles_m * p.tiles_n;
  if (blocks <= 0) return hipSuccess;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  p.n_blocks = (unsigned)blocks;
  constexpr size_t smem = 2ull * BK * ((BM + PAD) + (BN + PAD)) * sizeof(float);
  auto kern = seq_grad_kernel<BM, BN, BK, PAD, WEIGHTED>;
  // once per process and instantiation (static initialisation is thread-safe); a failure is returned by every call
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3(p.n_blocks), dim3(256), smem, s, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_seq_grad(const SeqGradArgs& a, hipStream_t s) {
  if (a.bf16) return launch_seq_grad_stream(a, s);
  if (a.per_sequence) return launch_cfg<64, 64, 16, 4, false>(a, s);
  return launch_cfg<64, 64, 16, 4, true>(a, s);
}

}  // namespace isopo
