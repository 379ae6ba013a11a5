// Token-position-sample estimate of each sequence's Fisher norm, in ghost form.
//
// The non-interacting listing estimates ||G_i||_F from n_s sampled token rows j
// (a0 = act_in[samples], g0 = grad_out[samples]; eq. formal-F-norm):
//     F_i^2 = sum_j (G_i . g^(j))^2 / sum_j ||g^(j)||^2,   g^(j) = g0_j a0_j^T.
// Since G_i = sum_{t in i} delta_t x_t^T is a sum of rank-one terms as well,
//     G_i . g^(j) = sum_{t in i} (delta_t . g0_j)(x_t . a0_j)       (eq. (one), summed over t)
//     ||g^(j)||^2 = ||g0_j||^2 ||a0_j||^2                            (eq. (two))
// so the coefficients c_i = A_i / sqrt(F_i^2 + reg) need no per-sequence
// gradient at all: two token-by-sample products P = Delta G0^T, Q = X A0^T
// (2 N n_s (d_in + d_out) flop, a few per cent of the layer's contraction), their
// element-wise product, and a segment sum over the tokens of each sequence.
//
// One workgroup takes 128 tokens (32 per wave).  Token rows and sample rows are
// streamed global -> LDS (row-contiguous DMA, XOR-swizzled 16-byte columns) in a
// four-stage ring; each wave multiplies its 32 tokens against all sample blocks
// on the matrix cores.  Segment sums go to an fp64 accumulator with atomics
// (order varies, but in fp64: the fp32 result moves by at most one rounding).
#include "common.h"
#include "kernels.h"

namespace isopo {
namespace {

typedef void __attribute__((address_space(3)))* lds_void_ptr;
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef v4u __attribute__((address_space(3)))* lds_v4u_ptr;

constexpr int kStages = 4;
constexpr int kRowBytes = 128;                 // bytes per row and stage
constexpr int kVpr = kRowBytes / 16;           // 16-byte vectors per row: 8
constexpr int kTok = 128;                      // tokens per workgroup
constexpr int kMaxSampleBlocks = 4;            // n_samples <= 128

__device__ __forceinline__ void load_lds16(const void* gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(gptr) : "memory");
}
// non-temporal cache policy: the token rows, which this pass reads once (the sample rows are re-read by
// every workgroup and keep the default)
__device__ __forceinline__ void load_lds16_nt(const void* gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" : : "s"(lds_addr), "v"(gptr) : "memory");
}

struct GroupParams {
  const void* X;
  const void* Delta[kFisherMaxGroup];
  int d_out[kFisherMaxGroup];
  int d_in, n_layers;
  double* S64;           // [n_layers][n_seq][32*NBS] segment sums s_ij of this group's layers
  double* den;           // [n_layers][n_samples] ||g0_j||^2 ||a0_j||^2
};
struct Params {
  GroupParams group[kFisherMaxGroups];     // blockIdx.y picks the group
  const int32_t* off;
  const int32_t* idx;
  int n_tokens, n_seq, n_samples;
  int32_t* tok_seq;      // [n_tokens]
  double* S64;           // all groups' segment sums, back to back
};

// The sequence of every token (binary search in the offsets) and zeros in the segment-sum accumulator.
__global__ __launch_bounds__(256) void prep_kernel(Params p, long long n_acc) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n_acc) p.S64[i] = 0.0;
  if (i < p.n_tokens) {
    const int t = (int)i;
    int lo = 0, hi = p.n_seq;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (p.off[mid] <= t) lo = mid; else hi = mid;
    }
    p.tok_seq[t] = lo;
  }
}

__global__ void zero_f64_kernel(double* p, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.0;
}

// One token-by-sample product block per wave: acc[b] (32 tokens x 32 samples) += T S_b^T over d features.
template <int NBS, bool BF16>
__device__ __forceinline__ void product_pass(const void* M, int d, const int32_t* __restrict__ idx, int n_samples,
                                             int n_tokens, int t0, unsigned smem_base, int lane, int wave,
                                             f32x16 (&acc)[NBS]) {
  constexpr int kEs = BF16 ? 2 : 4;
  constexpr int kV = 16 / kEs;                          // elements per 16-byte vector
  constexpr int KW = kRowBytes / kEs;                   // elements per row and stage
  constexpr int ROWS = kTok + 32 * NBS;                 // token rows, then sample rows
  constexpr int STAGE = ROWS * kRowBytes;
  constexpr int LOADS = ROWS * kRowBytes / 1024;        // 1 KiB wave-loads per stage (8 rows each)
  constexpr int LPW = (LOADS + 3) / 4;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int n_super = (d + KW - 1) / KW;

  const char* src[LPW];
  int vec_off[LPW];
  bool active[LPW];
#pragma unroll
  for (int q = 0; q < LPW; ++q) {
    const int load = wave * LPW + q;
    active[q] = load < LOADS;
    const int row = (active[q] ? load : 0) * 8 + lane / kVpr;
    const int pos = lane % kVpr;
    long long grow;
    if (row < kTok) {
      const int t = t0 + row;
      grow = t < n_tokens ? t : n_tokens - 1;
    } else {
      const int j = row - kTok;
      grow = min(max(idx[j < n_samples ? j : 0], 0), n_tokens - 1);
    }
    src[q] = static_cast<const char*>(M) + (size_t)grow * d * kEs;
    vec_off[q] = (pos ^ ((row >> 1) & (kVpr - 1))) * 16;
  }
  auto issue = [&](int k) {
#pragma unroll
    for (int q = 0; q < LPW; ++q) {
      long long byte = (long long)k * kRowBytes + vec_off[q];
      const long long last = ((long long)d - kV) * kEs;
      if (byte > last) byte = last;          // tail and look-ahead past the end: stays inside the row
      const int load = wave_s * LPW + q;
      const unsigned dst = smem_base + (unsigned)(k % kStages) * STAGE + (unsigned)load * 1024;
      if (load * 8 < kTok) load_lds16_nt(src[q] + byte, dst);
      else if (load < LOADS) load_lds16(src[q] + byte, dst);
    }
  };
  // every wave issues the same number of loads per stage only if LOADS is a multiple of 4
  static_assert(LOADS % 4 == 0, "wave-loads per stage divide evenly over the four waves");

#pragma unroll
  for (int s = 0; s < kStages - 1; ++s) issue(s);
  const int frow = lane & 31, half = lane >> 5;
  for (int k = 0; k < n_super; ++k) {
    __builtin_amdgcn_s_waitcnt(0x0f70 | (((kStages - 2) * LPW) & 15) | ((((kStages - 2) * LPW) >> 4) << 14));
    __builtin_amdgcn_s_barrier();
    issue(k + kStages - 1);
    const unsigned sb = smem_base + (unsigned)(k % kStages) * STAGE;
    const int valid = d - k * KW;
#pragma unroll
    for (int st = 0; st < kVpr / 2; ++st) {
      const int vec = st * 2 + half;
      const int ra = wave * 32 + frow;
      v4u fa = *(lds_v4u_ptr)(sb + (unsigned)ra * kRowBytes + (unsigned)((vec ^ ((ra >> 1) & (kVpr - 1))) * 16));
      if (valid < KW && vec * kV >= valid) fa = v4u{0u, 0u, 0u, 0u};
#pragma unroll
      for (int b = 0; b < NBS; ++b) {
        const int rb = kTok + b * 32 + frow;
        const v4u fb = *(lds_v4u_ptr)(sb + (unsigned)rb * kRowBytes + (unsigned)((vec ^ ((rb >> 1) & (kVpr - 1))) * 16));
        if constexpr (BF16) {
          acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa), __builtin_bit_cast(bf16x8, fb),
                                                           acc[b], 0, 0, 0);
        } else {
          const f32x4 xa = __builtin_bit_cast(f32x4, fa), xb = __builtin_bit_cast(f32x4, fb);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[e], xb[e], acc[b], 0, 0, 0);
        }
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);
  __builtin_amdgcn_s_barrier();          // the ring is reused by the next pass
}

template <int NBS, bool BF16>
__global__ __launch_bounds__(256) void fisher_samples_kernel(Params p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const unsigned smem_base = (unsigned)(size_t)(lds_void_ptr)smem;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t0 = blockIdx.x * kTok;
  const GroupParams& g = p.group[blockIdx.y];

  // Q = X A0^T once for the group, then per layer P = Delta G0^T, H = P o Q and the segment sums
  f32x16 Q[NBS];
#pragma unroll
  for (int b = 0; b < NBS; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) Q[b][v] = 0.f;
  product_pass<NBS, BF16>(g.X, g.d_in, p.idx, p.n_samples, p.n_tokens, t0, smem_base, lane, wave, Q);

  // lane holds sample column (lane & 31) of each block and token rows acc_row(v, lane) of the wave's 32 tokens
  const int tw = t0 + wave * 32;
  const bool live = tw < p.n_tokens;                  // wave-uniform; idle waves still join every pass's barriers
  const int t_last = min(tw + 31, p.n_tokens - 1);
  const int r_first = live ? p.tok_seq[tw] : 0, r_last = live ? p.tok_seq[t_last] : 0;
  const int ncol = 32 * NBS;
  for (int l = 0; l < g.n_layers; ++l) {
    f32x16 P[NBS];
#pragma unroll
    for (int b = 0; b < NBS; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) P[b][v] = 0.f;
    product_pass<NBS, BF16>(g.Delta[l], g.d_out[l], p.idx, p.n_samples, p.n_tokens, t0, smem_base, lane, wave, P);
    if (!live) continue;
    double* S64 = g.S64 + (size_t)l * p.n_seq * ncol;
    double* den = g.den + (size_t)l * p.n_samples;
#pragma unroll
    for (int b = 0; b < NBS; ++b) {
      const int j = b * 32 + (lane & 31);
      // ||g^(j)||^2 = ||g0_j||^2 ||a0_j||^2 (eq. (two)) is the product's own entry at the sampled row:
      // P[idx_j][j] = g0_j . g0_j and Q[idx_j][j] = a0_j . a0_j; exactly one lane of the grid holds it
      if (j < p.n_samples) {
        const int tj = min(max(p.idx[j], 0), p.n_tokens - 1);
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (tw + acc_row(v, lane) == tj) den[j] = (double)P[b][v] * (double)Q[b][v];
      }
      if (r_first == r_last) {
        double s = 0.0;
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (tw + acc_row(v, lane) < p.n_tokens) s += (double)P[b][v] * (double)Q[b][v];
        s += __shfl_xor(s, 32, kWave);
        if (lane < 32 && j < p.n_samples) atomicAdd(&S64[(size_t)r_first * ncol + j], s);
      } else {
        double run = 0.0;
        int run_r = -1;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int t = tw + acc_row(v, lane);
          if (t >= p.n_tokens) continue;
          const int r = p.tok_seq[t];
          if (r != run_r) {
            if (run_r >= 0 && j < p.n_samples) atomicAdd(&S64[(size_t)run_r * ncol + j], run);
            run_r = r;
            run = 0.0;
          }
          run += (double)P[b][v] * (double)Q[b][v];
        }
        if (run_r >= 0 && j < p.n_samples) atomicAdd(&S64[(size_t)run_r * ncol + j], run);
      }
    }
  }
}

__device__ double block_sum256(double x, double* red) {
  x = wave_sum(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// F_i^2 = sum_j s_ij^2 / sum_j den_j ;  c_i = A_i / sqrt(F_i^2 + reg).  One workgroup, fixed order.
__global__ __launch_bounds__(256) void fisher_samples_finish_kernel(const double* __restrict__ S64,
                                                                    const double* __restrict__ den, int n_seq,
                                                                    int n_samples, int ncol, const float* __restrict__ A,
                                                                    float lambda, int reg_mode, float* __restrict__ ema_state,
                                                                    float ema_decay, float* __restrict__ c,
                                                                    float* __restrict__ f2_out, double* __restrict__ f2_tmp) {
  __shared__ double red[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int layer = blockIdx.x;                    // one workgroup per layer of the group
  S64 += (size_t)layer * n_seq * ncol;
  den += (size_t)layer * n_samples;
  f2_tmp += (size_t)layer * n_seq;
  c += (size_t)layer * n_seq;
  if (f2_out) f2_out += (size_t)layer * n_seq;
  if (ema_state) ema_state += 2 * layer;
  const double d = block_sum256(tid < n_samples ? den[tid] : 0.0, red);      // n_samples <= 128
  // one wave per sequence: lanes stride over the samples
  double part = 0.0;
  for (int i = wave; i < n_seq; i += 4) {
    double s = 0.0;
    for (int j = lane; j < n_samples; j += 64) {
      const double x = S64[(size_t)i * ncol + j];
      s += x * x;
    }
    s = wave_sum(s);
    const double f2 = d > 0.0 ? s / d : 0.0;
    if (lane == 0) { f2_tmp[i] = f2; part += f2; }
  }
  const double mean = block_sum256(part, red) / n_seq;
  __shared__ double sh_scale;
  if (tid == 0) {
    double scale = 1.0;                                  // absolute
    if (reg_mode == 1) scale = mean;                     // this batch's mean F^2
    if (reg_mode == 2) {                                 // trailing mean over minibatches, this one included
      const bool first = ema_state[1] == 0.f;
      scale = first ? mean : (double)ema_decay * (double)ema_state[0] + (1.0 - (double)ema_decay) * mean;
      ema_state[0] = (float)scale;
      ema_state[1] = ema_state[1] + 1.f;
    }
    sh_scale = scale;
  }
  __syncthreads();
  const double reg = (double)lambda * sh_scale;
  __syncthreads();                                   // f2_tmp written by lane 0 of each wave, read by all below
  for (int i = tid; i < n_seq; i += 256) {
    const double den_i = f2_tmp[i] + reg;
    c[i] = den_i > 0.0 ? (float)((double)A[i] / sqrt(den_i)) : 0.f;
    if (f2_out) f2_out[i] = (float)f2_tmp[i];
  }
}

template <int NBS, bool BF16>
hipError_t launch_main(const Params& p, int n_groups, hipStream_t s) {
  constexpr size_t smem = (size_t)kStages * (kTok + 32 * NBS) * kRowBytes;
  auto kern = fisher_samples_kernel<NBS, BF16>;
  // once per process (static initialisation is thread-safe); a failure is returned by every call
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3((p.n_tokens + kTok - 1) / kTok, n_groups), dim3(256), smem, s, p);
  return hipGetLastError();
}

size_t align256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

size_t fisher_samples_workspace(int n_tokens, int n_seq, int n_samples, int n_layers) {
  const int ncol = 32 * ((n_samples + 31) / 32);
  return align256((size_t)n_tokens * 4) + align256((size_t)n_layers * n_seq * ncol * 8) +
         align256((size_t)n_layers * n_samples * 8) + align256((size_t)n_layers * n_seq * 8);
}

hipError_t launch_fisher_samples(const FisherSamplesArgs& a, hipStream_t s) {
  const int nbs = (a.n_samples + 31) / 32;
  if (nbs < 1 || nbs > kMaxSampleBlocks || a.n_groups < 1 || a.n_groups > kFisherMaxGroups) return hipErrorInvalidValue;
  int n_layers = 0;
  for (int g = 0; g < a.n_groups; ++g) {
    if (a.group[g].n_layers < 1 || a.group[g].n_layers > kFisherMaxGroup) return hipErrorInvalidValue;
    n_layers += a.group[g].n_layers;
  }
  const int ncol = 32 * nbs;
  // workspace: token -> sequence map, then per layer (all groups' layers back to back, in group order) the
  // segment sums, the sample norms and the fp64 F^2
  char* ws = static_cast<char*>(a.workspace);
  Params p;
  p.off = a.off; p.idx = a.sample_idx;
  p.n_tokens = a.n_tokens; p.n_seq = a.n_seq; p.n_samples = a.n_samples;
  p.tok_seq = reinterpret_cast<int32_t*>(ws);
  ws += align256((size_t)a.n_tokens * 4);
  p.S64 = reinterpret_cast<double*>(ws);
  ws += align256((size_t)n_layers * a.n_seq * ncol * 8);
  double* den = reinterpret_cast<double*>(ws);
  ws += align256((size_t)n_layers * a.n_samples * 8);
  double* f2_tmp = reinterpret_cast<double*>(ws);
  // A short microbatch does not fill the chip with one workgroup per (128 tokens, group), and a lone workgroup
  // is bound by the latency of its walk over the features, not by bandwidth: then every layer becomes a group
  // of its own (its input's product is formed once per layer instead of once per group, the walks are shorter
  // and there are more of them: 0.18 -> 0.10 ms for a 1.5B-class block at 3200 tokens, 0.21 -> 0.15 ms at 10^4,
  // a loss of 4 - 10 % from 1.6 * 10^4 tokens on).
  const int token_tiles = (a.n_tokens + kTok - 1) / kTok;
  const bool one_layer_per_group = n_layers > a.n_groups && n_layers <= kFisherMaxGroups && token_tiles * n_layers <= 640;
  int n_launch_groups = a.n_groups;
  if (one_layer_per_group) {
    n_launch_groups = n_layers;
    int layer = 0;
    for (int g = 0; g < a.n_groups; ++g)
      for (int l = 0; l < a.group[g].n_layers; ++l, ++layer) {
        GroupParams& q = p.group[layer];
        q.X = a.group[g].X; q.d_in = a.group[g].d_in; q.n_layers = 1;
        for (int k = 0; k < kFisherMaxGroup; ++k) { q.Delta[k] = nullptr; q.d_out[k] = 0; }
        q.Delta[0] = a.group[g].Delta[l]; q.d_out[0] = a.group[g].d_out[l];
        q.S64 = p.S64 + (size_t)layer * a.n_seq * ncol;
        q.den = den + (size_t)layer * a.n_samples;
      }
    for (int g = n_layers; g < kFisherMaxGroups; ++g) {
      GroupParams& q = p.group[g];
      q.X = nullptr; q.d_in = 0; q.n_layers = 0; q.S64 = nullptr; q.den = nullptr;
      for (int k = 0; k < kFisherMaxGroup; ++k) { q.Delta[k] = nullptr; q.d_out[k] = 0; }
    }
  } else {
    int first = 0;
    for (int g = 0; g < kFisherMaxGroups; ++g) {
      GroupParams& q = p.group[g];
      const bool live = g < a.n_groups;
      q.X = live ? a.group[g].X : nullptr;
      q.d_in = live ? a.group[g].d_in : 0;
      q.n_layers = live ? a.group[g].n_layers : 0;
      for (int l = 0; l < kFisherMaxGroup; ++l) {
        q.Delta[l] = live && l < q.n_layers ? a.group[g].Delta[l] : nullptr;
        q.d_out[l] = live && l < q.n_layers ? a.group[g].d_out[l] : 0;
      }
      q.S64 = p.S64 + (size_t)first * a.n_seq * ncol;
      q.den = den + (size_t)first * a.n_samples;
      first += q.n_layers;
    }
  }

  // Longest walk first: the workgroups of the launch's last group are the ones that run on a half-empty chip
  // at the end, so that group should be the one with the fewest features to walk.
  auto features = [](const GroupParams& q) {
    long long f = q.d_in;
    for (int l = 0; l < q.n_layers; ++l) f += q.d_out[l];
    return f;
  };
  for (int i = 1; i < n_launch_groups; ++i)          // insertion sort, descending, stable
    for (int j = i; j > 0 && features(p.group[j]) > features(p.group[j - 1]); --j) {
      const GroupParams t = p.group[j];
      p.group[j] = p.group[j - 1];
      p.group[j - 1] = t;
    }

  const long long ns = (long long)n_layers * a.n_seq * ncol;
  if (a.n_tokens > 0) {
    const long long items = ns > a.n_tokens ? ns : (long long)a.n_tokens;
    hipLaunchKernelGGL(prep_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, s, p, ns);
    hipError_t e;
    switch (nbs * 2 + (a.bf16 ? 1 : 0)) {
      case 2: e = launch_main<1, false>(p, n_launch_groups, s); break;
      case 3: e = launch_main<1, true>(p, n_launch_groups, s); break;
      case 4: e = launch_main<2, false>(p, n_launch_groups, s); break;
      case 5: e = launch_main<2, true>(p, n_launch_groups, s); break;
      case 6: e = launch_main<3, false>(p, n_launch_groups, s); break;
      case 7: e = launch_main<3, true>(p, n_launch_groups, s); break;
      case 8: e = launch_main<4, false>(p, n_launch_groups, s); break;
      default: e = launch_main<4, true>(p, n_launch_groups, s); break;
    }
    if (e != hipSuccess) return e;
  } else {
    hipLaunchKernelGGL(zero_f64_kernel, dim3((unsigned)((ns + 255) / 256)), dim3(256), 0, s, p.S64, ns);
    const long long nd = (long long)n_layers * a.n_samples;
    hipLaunchKernelGGL(zero_f64_kernel, dim3((unsigned)((nd + 255) / 256)), dim3(256), 0, s, den, nd);
  }
  hipLaunchKernelGGL(fisher_samples_finish_kernel, dim3(n_layers), dim3(256), 0, s, p.S64, den, a.n_seq,
                     a.n_samples, ncol, a.A, a.lambda, a.reg_mode, a.ema_state, a.ema_decay, a.c, a.fisher_sq, f2_tmp);
  return hipGetLastError();
}

}  // namespace isopo
