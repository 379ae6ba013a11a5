// Gram matrix and weighted sum over the stash of per-sequence gradients.
//
//   K_ij = sum_p S[i][p] * S[j][p]          (interacting listing: ntk[i, j] =
//                                            sum(seq_grads[i] * seq_grads[j]))
//   dW[p] = beta dW[p] + sum_i c_i S[i][p]  (stack(seq_grads, -1) @ coefficients)
//
// Both read the stash once and are bound by HBM.  For the Gram matrix the
// reduction index p is the fast index of every S[i], which is the register
// layout the MFMA wants for both operands, and since K = S S^T the A and B
// fragments are the same registers: a wave loads one 16-byte piece per lane and
// row block and issues mfma(a_i, a_j) for every block pair i <= j.
//
// Determinism: the p -> wave assignment is a fixed formula, the four waves of a
// workgroup are added in wave order through LDS into the workgroup's slot of a
// partial buffer, and the finishing kernel adds the slots in a fixed tree; K is
// bit-reproducible and exactly symmetric.
#include "common.h"
#include "kernels.h"

namespace isopo {
namespace {

constexpr int kGramBlocks = 1024;           // workgroups of the streaming kernel (4 per CU)
constexpr int kGramWaves = 4;               // waves per workgroup
constexpr int kGramSlots = kGramBlocks;     // one partial slot per workgroup
constexpr int kMaxRowBlocks = 4;            // 32-row blocks a single wave keeps pairs for (n_seq <= 128)

__host__ __device__ constexpr int tri(int nb) { return nb * (nb + 1) / 2; }
// index of block pair (bi <= bj) in row-major upper-triangular order
__host__ __device__ inline int pair_index(int bi, int bj, int nb) { return bi * nb - bi * (bi - 1) / 2 + (bj - bi); }

struct GramParams {
  const void* stash;
  long long seq_stride, p0, p1;
  int n_seq;
  int first;
  float* partials;
  long long slot_floats;
};

// One wave handles "super steps" of kSuper consecutive 32-byte-per-row pieces, so
// that each row is read in runs of kSuper*32 bytes and kSuper*NB loads are in flight.
template <int NB, bool BF16>
__global__ __launch_bounds__(256) void stash_gram_kernel(GramParams p) {
  constexpr int kElemPerVec = BF16 ? 8 : 4;           // per 16-byte lane load
  constexpr int kStepElems = 2 * kElemPerVec;         // per row and micro step (two lane halves)
  constexpr int kSuper = NB == 1 ? 16 : (NB == 2 ? 8 : 4);
  __shared__ float red[tri(NB) * 1024];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane & 31, half = lane >> 5;
  const long long gw = (long long)blockIdx.x * kGramWaves + wave;
  const long long n_waves = (long long)gridDim.x * kGramWaves;

  f32x16 acc[tri(NB)];
#pragma unroll
  for (int q = 0; q < tri(NB); ++q)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;

  const char* base[NB];
  bool row_ok[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const int r = b * 32 + row;
    row_ok[b] = r < p.n_seq;
    base[b] = static_cast<const char*>(p.stash) + (size_t)(row_ok[b] ? r : 0) * p.seq_stride * (BF16 ? 2 : 4);
  }

  const long long n_elems = p.p1 - p.p0;
  const long long n_super = (n_elems + kSuper * kStepElems - 1) / (kSuper * kStepElems);
  for (long long u = gw; u < n_super; u += n_waves) {
    uint4 frag[NB][kSuper];
#pragma unroll
    for (int q = 0; q < kSuper; ++q) {
      const long long e = p.p0 + (u * kSuper + q) * kStepElems + half * kElemPerVec;
      const bool in = e < p.p1;     // p1 - p0 is a multiple of the vector width
#pragma unroll
      for (int b = 0; b < NB; ++b)
        frag[b][q] = (in && row_ok[b]) ? *reinterpret_cast<const uint4*>(base[b] + e * (BF16 ? 2 : 4))
                                       : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int q = 0; q < kSuper; ++q) {
#pragma unroll
      for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int bj = bi; bj < NB; ++bj) {
          f32x16& a = acc[pair_index(bi, bj, NB)];
          if constexpr (BF16) {
            a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, frag[bi][q]),
                                                        __builtin_bit_cast(bf16x8, frag[bj][q]), a, 0, 0, 0);
          } else {
            const float4 fa = __builtin_bit_cast(float4, frag[bi][q]);
            const float4 fb = __builtin_bit_cast(float4, frag[bj][q]);
            a = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.x, fb.x, a, 0, 0, 0);
            a = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.y, fb.y, a, 0, 0, 0);
            a = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.z, fb.z, a, 0, 0, 0);
            a = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.w, fb.w, a, 0, 0, 0);
          }
        }
    }
  }

  // waves 0..3 added in order; layout [pair][v][lane]
  for (int w = 0; w < kGramWaves; ++w) {
    if (wave == w) {
#pragma unroll
      for (int q = 0; q < tri(NB); ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float* o = red + (q * 16 + v) * 64 + lane;
          *o = (w == 0 ? 0.f : *o) + acc[q][v];
        }
    }
    __syncthreads();
  }
  float* out = p.partials + (long long)blockIdx.x * p.slot_floats;
  for (int e = threadIdx.x; e < tri(NB) * 1024; e += 256) out[e] = (p.first ? 0.f : out[e]) + red[e];
}

// One 1024-thread block per 64 consecutive slot elements: wave w adds slots w, w+16, ... in order,
// the 16 waves are added in wave order; only entries with i <= j are written, mirrored.
__global__ __launch_bounds__(1024) void stash_gram_finish_kernel(const float* __restrict__ partials, int n_slots,
                                                                 long long slot_floats, int n_seq, int nb,
                                                                 float* __restrict__ K) {
  __shared__ float red[16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long long e = (long long)blockIdx.x * 64 + lane;      // element of the slot layout [pair][v][lane]
  float s = 0.f;
  for (int w = wave; w < n_slots; w += 16) s += partials[(long long)w * slot_floats + e];
  red[wave][lane] = s;
  __syncthreads();
  if (wave != 0) return;
  s = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) s += red[w][lane];
  const int q = (int)(e >> 10), v = (int)(e >> 6) & 15;
  int bi = 0, rem = q;
  while (rem >= nb - bi) { rem -= nb - bi; ++bi; }
  const int bj = bi + rem;
  const int i = bi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3), j = bj * 32 + (lane & 31);
  if (i < n_seq && j < n_seq && i <= j) {
    K[(size_t)i * n_seq + j] = s;
    K[(size_t)j * n_seq + i] = s;
  }
}

template <bool BF16, bool OUTB>
__global__ __launch_bounds__(256) void stash_weighted_sum_kernel(const void* __restrict__ stash, long long seq_stride,
                                                                 long long n_vec, int n_seq,
                                                                 const float* __restrict__ c, float beta,
                                                                 void* __restrict__ dW_out) {
  constexpr int kV = BF16 ? 8 : 4;
  for (long long vi = (long long)blockIdx.x * blockDim.x + threadIdx.x; vi < n_vec;
       vi += (long long)gridDim.x * blockDim.x) {
    float s[kV];
#pragma unroll
    for (int e = 0; e < kV; ++e) s[e] = 0.f;
    const char* src = static_cast<const char*>(stash) + vi * 16;
#pragma unroll 8
    for (int i = 0; i < n_seq; ++i) {
      const float ci = c[i];
      typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
      const u32x4* vp = reinterpret_cast<const u32x4*>(src + (size_t)i * seq_stride * (BF16 ? 2 : 4));
      const u32x4 vv = __builtin_nontemporal_load(vp);     // read once: 5.2 -> 5.8 TB/s with the full grid below
      const uint4 v = make_uint4(vv[0], vv[1], vv[2], vv[3]);
      if constexpr (BF16) {
        const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          s[2 * e] += ci * __builtin_bit_cast(float, w[e] << 16);
          s[2 * e + 1] += ci * __builtin_bit_cast(float, w[e] & 0xffff0000u);
        }
      } else {
        const float4 f = __builtin_bit_cast(float4, v);
        s[0] += ci * f.x; s[1] += ci * f.y; s[2] += ci * f.z; s[3] += ci * f.w;
      }
    }
    if constexpr (OUTB) {
      // bf16 dW (bf16 stash only): the thread's eight values are one 16-byte vector
      static_assert(!OUTB || BF16, "a bf16 dW is formed from a bf16 stash");
      uint4* o = static_cast<uint4*>(dW_out) + vi;
      unsigned w[4] = {0u, 0u, 0u, 0u};
      if (beta != 0.f) {
        const uint4 old = *o;
        w[0] = old.x; w[1] = old.y; w[2] = old.z; w[3] = old.w;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float lo = s[2 * e] + beta * __builtin_bit_cast(float, w[e] << 16);
        const float hi = s[2 * e + 1] + beta * __builtin_bit_cast(float, w[e] & 0xffff0000u);
        w[e] = (unsigned)f32_to_bf16_bits(lo) | ((unsigned)f32_to_bf16_bits(hi) << 16);
      }
      *o = make_uint4(w[0], w[1], w[2], w[3]);
    } else {
      float* o = static_cast<float*>(dW_out) + vi * kV;
#pragma unroll
      for (int e = 0; e < kV; e += 4) {
        float4 r = make_float4(s[e], s[e + 1], s[e + 2], s[e + 3]);
        if (beta != 0.f) {
          const float4 old = *reinterpret_cast<const float4*>(o + e);
          r.x += beta * old.x; r.y += beta * old.y; r.z += beta * old.z; r.w += beta * old.w;
        }
        *reinterpret_cast<float4*>(o + e) = r;
      }
    }
  }
}

// The same from a stash in tile order (see stash_tile_order_ok): a thread's eight values are four rows of
// two columns of dW, 16 apart; a wave stores, per value, four rows' runs of 16 consecutive floats, and the
// values q and q + 4 complete each other's 128-byte lines.
template <int T, bool OUTB>
__global__ __launch_bounds__(256) void stash_weighted_sum_tiled_kernel(const void* __restrict__ stash, long long seq_stride,
                                                                       long long n_vec, int n_seq,
                                                                       const float* __restrict__ c, float beta,
                                                                       void* __restrict__ dW_out, int d_in, int tiles_n) {
  constexpr int NP = T / 64;                       // 16x32 pieces per 16-row strip of a quadrant
  constexpr int QV = (T / 2) * (T / 2) / 8;        // 16-byte vectors per quadrant
  constexpr int TV = T * T / 8;                    // ... per tile
  for (long long vi = (long long)blockIdx.x * blockDim.x + threadIdx.x; vi < n_vec;
       vi += (long long)gridDim.x * blockDim.x) {
    float s[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] = 0.f;
    const char* src = static_cast<const char*>(stash) + vi * 16;
#pragma unroll 8
    for (int i = 0; i < n_seq; ++i) {
      const float ci = c[i];
      typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
      const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + (size_t)i * seq_stride * 2));
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s[2 * e] += ci * __builtin_bit_cast(float, w[e] << 16);
        s[2 * e + 1] += ci * __builtin_bit_cast(float, w[e] & 0xffff0000u);
      }
    }
    const long long tile = vi / TV;
    const int r = (int)(vi % TV), quad = r / QV, r2 = r % QV, piece = r2 / 64, lane = r2 % 64;
    const int strip = piece / NP, jp = piece % NP;
    const int tile_m = (int)(tile / tiles_n), tile_n = (int)(tile % tiles_n);
    const int n0 = tile_n * T + (quad & 1) * (T / 2) + jp * 32 + (lane & 15);
    const int m0 = tile_m * T + (quad >> 1) * (T / 2) + strip * 16 + 4 * (lane >> 4);
    if constexpr (OUTB) {
      // bf16 dW: neighbouring lanes hold neighbouring columns; the even lane takes its neighbour's values of
      // the left 16 columns and stores pairs there, the odd lane does the same for the right 16 columns
      // (n_vec is a multiple of 64 for a stash in tile order, so every lane of a wave is here)
      __bf16* dW = static_cast<__bf16*>(dW_out);
      const bool odd = lane & 1;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float got = __shfl_xor(odd ? s[q] : s[q + 4], 1, kWave);
        float lo = odd ? got : s[q], hi = odd ? s[q + 4] : got;
        unsigned* o = reinterpret_cast<unsigned*>(dW + (size_t)(m0 + q) * d_in + (n0 & ~1) + (odd ? 16 : 0));
        if (beta != 0.f) {
          const unsigned old = *o;
          lo += beta * __builtin_bit_cast(float, old << 16);
          hi += beta * __builtin_bit_cast(float, old & 0xffff0000u);
        }
        *o = (unsigned)f32_to_bf16_bits(lo) | ((unsigned)f32_to_bf16_bits(hi) << 16);
      }
    } else {
      float* dW = static_cast<float*>(dW_out);
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        float* o = dW + (size_t)(m0 + (q & 3)) * d_in + n0 + 16 * (q >> 2);
        *o = (beta != 0.f ? beta * *o : 0.f) + s[q];
      }
    }
  }
}

template <int NB>
hipError_t launch_gram_nb(const GramParams& p, bool bf16, hipStream_t s) {
  if (bf16)
    hipLaunchKernelGGL((stash_gram_kernel<NB, true>), dim3(kGramBlocks), dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL((stash_gram_kernel<NB, false>), dim3(kGramBlocks), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace

int stash_gram_slots() { return kGramSlots; }

size_t stash_gram_slot_floats(int n_seq) {
  const int nb = (n_seq + 31) / 32;
  return (size_t)tri(nb) * 1024;
}

size_t stash_gram_partial_bytes(int n_seq, bool bf16) {
  if (n_seq > 128)
    return bf16 ? (size_t)stash_gram_large_slots(n_seq) * stash_gram_large_slot_floats(n_seq) * sizeof(float) : 0;
  return (size_t)kGramSlots * stash_gram_slot_floats(n_seq) * sizeof(float);
}

static int slots_used(bool bf16) { return bf16 ? stash_gram_stream_slots() : kGramSlots; }

hipError_t launch_stash_gram(const StashGramArgs& a, hipStream_t s) {
  const int nb = (a.n_seq + 31) / 32;
  if (nb > kMaxRowBlocks) return a.bf16 ? launch_stash_gram_large(a, s) : hipErrorInvalidValue;
  if (a.bf16) return launch_stash_gram_stream(a, s);
  GramParams p;
  p.stash = a.stash; p.seq_stride = a.seq_stride; p.p0 = a.p0; p.p1 = a.p1;
  p.n_seq = a.n_seq; p.first = a.first ? 1 : 0; p.partials = a.partials;
  p.slot_floats = (long long)stash_gram_slot_floats(a.n_seq);
  switch (nb) {
    case 1: return launch_gram_nb<1>(p, a.bf16, s);
    case 2: return launch_gram_nb<2>(p, a.bf16, s);
    case 3: return launch_gram_nb<3>(p, a.bf16, s);
    default: return launch_gram_nb<4>(p, a.bf16, s);
  }
}

hipError_t launch_stash_gram_finish(const float* partials, bool bf16, int n_seq, float* K, hipStream_t s) {
  if (n_seq > 128) return bf16 ? launch_stash_gram_large_finish(partials, n_seq, K, s) : hipErrorInvalidValue;
  const int nb = (n_seq + 31) / 32;
  const long long slot_floats = (long long)stash_gram_slot_floats(n_seq);
  hipLaunchKernelGGL(stash_gram_finish_kernel, dim3((unsigned)(slot_floats / 64)), dim3(1024), 0, s, partials,
                     slots_used(bf16), slot_floats, n_seq, nb, K);
  return hipGetLastError();
}

hipError_t launch_stash_weighted_sum(const void* stash, bool bf16, long long seq_stride, long long n_elem, int n_seq,
                                     const float* c, float beta, void* dW, bool dw_bf16, hipStream_t s) {
  const long long n_vec = n_elem / (bf16 ? 8 : 4);
  if (n_vec <= 0) return hipSuccess;
  if (dw_bf16 && !bf16) return hipErrorInvalidValue;
  // one 16-byte vector per thread (the kernel's loop strides over the rest of a stash beyond 2^39 elements)
  long long blocks = (n_vec + 255) / 256;
  if (blocks > 0x7fffffffLL) blocks = 0x7fffffffLL;
  if (bf16 && dw_bf16)
    hipLaunchKernelGGL((stash_weighted_sum_kernel<true, true>), dim3((unsigned)blocks), dim3(256), 0, s, stash, seq_stride,
                       n_vec, n_seq, c, beta, dW);
  else if (bf16)
    hipLaunchKernelGGL((stash_weighted_sum_kernel<true, false>), dim3((unsigned)blocks), dim3(256), 0, s, stash, seq_stride,
                       n_vec, n_seq, c, beta, dW);
  else
    hipLaunchKernelGGL((stash_weighted_sum_kernel<false, false>), dim3((unsigned)blocks), dim3(256), 0, s, stash, seq_stride,
                       n_vec, n_seq, c, beta, dW);
  return hipGetLastError();
}

template <int T, bool OUTB>
static hipError_t launch_tiled_t(const void* stash, long long D, long long n_vec, int n_seq, const float* c, float beta,
                                 void* dW, int d_in, hipStream_t s) {
  long long blocks = (n_vec + 255) / 256;
  if (blocks > 0x7fffffffLL) blocks = 0x7fffffffLL;
  hipLaunchKernelGGL((stash_weighted_sum_tiled_kernel<T, OUTB>), dim3((unsigned)blocks), dim3(256), 0, s, stash, D, n_vec,
                     n_seq, c, beta, dW, d_in, d_in / T);
  return hipGetLastError();
}

hipError_t launch_stash_weighted_sum_tiled(const void* stash, int tile, int d_out, int d_in, int n_seq, const float* c,
                                           float beta, void* dW, bool dw_bf16, hipStream_t s) {
  if ((tile != 256 && tile != 128) || d_out % tile || d_in % tile) return hipErrorInvalidValue;
  const long long D = (long long)d_out * d_in, n_vec = D / 8;
  if (n_vec <= 0) return hipSuccess;
  if (tile == 256)
    return dw_bf16 ? launch_tiled_t<256, true>(stash, D, n_vec, n_seq, c, beta, dW, d_in, s)
                   : launch_tiled_t<256, false>(stash, D, n_vec, n_seq, c, beta, dW, d_in, s);
  return dw_bf16 ? launch_tiled_t<128, true>(stash, D, n_vec, n_seq, c, beta, dW, d_in, s)
                 : launch_tiled_t<128, false>(stash, D, n_vec, n_seq, c, beta, dW, d_in, s);
}

}  // namespace isopo
