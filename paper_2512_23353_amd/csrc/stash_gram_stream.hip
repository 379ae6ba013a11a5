// Gram matrix of a bf16 stash, streaming variants (n_seq <= 128 first; larger batches further down):
//     K_ij = sum_p S[i][p] * S[j][p]        (interacting listing:
//                                            ntk[i, j] = sum(seq_grads[i] * seq_grads[j]))
// One pass over the stash, bound by HBM.  The stash rows are 10^7..10^8 elements
// apart, so fragment-shaped loads (one row per lane) touch 32 cache lines per
// instruction and use 32 bytes of each.  Here the loads are row-contiguous
// instead: global_load_lds moves 16 bytes per lane straight into LDS, a wave
// covering whole 1 KiB / 512 B / 256 B runs of a row, into a ring of 32 KiB
// stages (all rows x KW elements).  Each wave then reads MFMA fragments for its
// share of the stage's 16-element steps with ds_read_b128 (16-byte column index
// XOR-swizzled with the row, so the row-per-lane reads do not pile on one bank)
// and issues mfma(a_i, a_j) for every row-block pair i <= j; the A and B
// fragments of K = S S^T are the same registers.
//
// Deterministic: fixed p -> workgroup -> wave assignment, waves added in order
// through LDS into the workgroup's partial slot, slots added in a fixed tree by
// the finishing kernel.
#include "common.h"
#include "kernels.h"

namespace isopo {
namespace {

typedef unsigned short u16;
typedef void __attribute__((address_space(3)))* lds_void_ptr;
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef v4u __attribute__((address_space(3)))* lds_v4u_ptr;

constexpr int kBlocks = 256;           // persistent workgroups, one per CU
constexpr int kStageBytes = 32768;
constexpr int kStages = 4;

__host__ __device__ constexpr int tri(int nb) { return nb * (nb + 1) / 2; }
__host__ __device__ constexpr int pair_index(int bi, int bj, int nb) { return bi * nb - bi * (bi - 1) / 2 + (bj - bi); }

struct Params {
  const u16* stash;
  long long seq_stride, p0, p1;
  int n_seq, first;
  float* partials;
  long long slot_floats;
};

// 16 bytes per lane, global -> LDS (lane l lands at lds_addr + 16*l).  Inline asm keeps the compiler's
// LDS-DMA tracking from waiting on every outstanding load before each LDS read.
__device__ __forceinline__ void load_lds16(const void* gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(gptr) : "memory");
}
// The same with the non-temporal cache policy, for the one-pass kernels (up to 256 sequences): every stash
// byte is read once, and keeping it out of the caches' replacement order is worth 13 % of the pass for up
// to 128 sequences (6.2 -> 7.05 TB/s on a 3.8 GB stash) and 3 % for 129..256 (72 GB stash).  The super-block
// pair kernel reads a row once per pair and keeps the default policy.
__device__ __forceinline__ void load_lds16_nt(const void* gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" : : "s"(lds_addr), "v"(gptr) : "memory");
}

// NB   32-row blocks that carry sequences (pairs are formed among these)
// NBL  row blocks of the LDS layout: 1, 2 or 4 (NBL >= NB); stage = 32*NBL rows x KW elements
template <int NB, int NBL>
__global__ __launch_bounds__(256) void stash_gram_stream_kernel(Params p) {
  constexpr int ROWS = 32 * NBL;
  constexpr int RB = kStageBytes / ROWS;           // bytes per row and stage: 1024, 512, 256
  constexpr int KW = RB / 2;                        // elements per row and stage
  constexpr int VPR = RB / 16;                      // 16-byte vectors per row: 64, 32, 16
  constexpr int RPL = 1024 / RB;                    // rows per 1 KiB wave-load: 1, 2, 4
  constexpr int LPW = kStageBytes / 1024 / 4;       // wave-loads per wave and stage: 8
  constexpr int STEPS = KW / 16 / 4;                // 16-element steps per wave and stage: 8, 4, 2
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const unsigned smem_base = (unsigned)(size_t)(lds_void_ptr)smem;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);

  const long long n_elems = p.p1 - p.p0;
  const long long n_super = (n_elems + KW - 1) / KW;
  const long long my_first = blockIdx.x;
  const long long my_count = my_first < n_super ? (n_super - my_first + gridDim.x - 1) / gridDim.x : 0;

  // DMA addressing: wave-load q of this wave covers rows (wave*LPW + q)*RPL .. +RPL-1
  const char* src[LPW];
  int vec_off[LPW];
#pragma unroll
  for (int q = 0; q < LPW; ++q) {
    const int row = (wave * LPW + q) * RPL + lane / VPR;
    const int pos = lane % VPR;
    const int g = pos ^ (row & (VPR - 1) & 31);                 // global vector this LDS slot holds
    const int r = row < p.n_seq ? row : p.n_seq - 1;            // padded rows re-read a real row; their K entries are dropped
    src[q] = reinterpret_cast<const char*>(p.stash + (size_t)r * p.seq_stride + p.p0);
    vec_off[q] = g * 16;
  }
  auto issue = [&](long long k) {     // k-th super step of this workgroup -> ring stage k % kStages
    const long long u = my_first + k * gridDim.x;
    const long long e0 = u * KW;                                     // element offset of the stage within [p0, p1)
    const unsigned stage = smem_base + (unsigned)(k % kStages) * kStageBytes;
#pragma unroll
    for (int q = 0; q < LPW; ++q) {
      long long byte = e0 * 2 + vec_off[q];
      const long long last = (n_elems - 8) * 2;
      if (byte > last) byte = last;                               // tail: stays inside the row, zeroed at read time
      if (k >= my_count) byte = 0;                                // look-ahead past the end: harmless re-read
      load_lds16_nt(src[q] + byte, stage + (unsigned)(wave_s * LPW + q) * 1024);
    }
  };

  f32x16 acc[tri(NB)];
#pragma unroll
  for (int q = 0; q < tri(NB); ++q)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;

  // fragment addressing: lane (row = lane&31, half = lane>>5) of row block b, step s of this wave
  const int frow = lane & 31, half = lane >> 5;

#pragma unroll
  for (int s = 0; s < kStages - 1; ++s) issue(s);

  for (long long k = 0; k < my_count; ++k) {
    // this wave's part of stage k landed, then everyone's; the stage of step k-1 is free after the barrier
    __builtin_amdgcn_s_waitcnt(0x0f70 | (((kStages - 2) * LPW) & 15) | ((((kStages - 2) * LPW) >> 4) << 14));
    __builtin_amdgcn_s_barrier();
    issue(k + kStages - 1);
    const unsigned sb = smem_base + (unsigned)(k % kStages) * kStageBytes;
    const long long u = my_first + k * gridDim.x;
    const long long valid = n_elems - u * KW;                    // elements of this stage inside [p0, p1)
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      const int step = wave * STEPS + s;                         // 16-element step within the stage
      const int vec = step * 2 + half;                           // 16-byte vector within the row
      v4u frag[NB];
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int row = b * 32 + frow;
        const unsigned a = sb + (unsigned)row * RB + (unsigned)((vec ^ (row & (VPR - 1) & 31)) * 16);
        frag[b] = *(lds_v4u_ptr)(a);
        if (valid < KW && (long long)vec * 8 >= valid) frag[b] = v4u{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int bj = bi; bj < NB; ++bj)
          acc[pair_index(bi, bj, NB)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, frag[bi]), __builtin_bit_cast(bf16x8, frag[bj]), acc[pair_index(bi, bj, NB)],
              0, 0, 0);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);      // drain the look-ahead loads before LDS is reused / released
  __builtin_amdgcn_s_barrier();

  // waves 0..3 added in order through LDS (reusing the ring); slot layout [pair][v][lane]
  float* red = reinterpret_cast<float*>(smem);
  for (int w = 0; w < 4; ++w) {
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

template <int NB, int NBL>
hipError_t launch(const Params& p, hipStream_t s) {
  constexpr size_t smem = (size_t)kStages * kStageBytes;
  static_assert((size_t)tri(NB) * 4096 <= smem, "reduction scratch fits the ring");
  auto kern = stash_gram_stream_kernel<NB, NBL>;
  // once per process (static initialisation is thread-safe); a failure is returned by every call
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3(kBlocks), dim3(256), smem, s, p);
  return hipGetLastError();
}


// ---- more than 128 sequences --------------------------------------------------------------------
// K is cut into 128x128 super blocks; one launch row (blockIdx.y) per super-block pair (I <= J).  A
// workgroup streams the 128 (I == J) or 256 (I < J) rows of its pair through the same kind of LDS ring
// and wave w forms the four 32x32 blocks (4I + w, 4J + 0..3).  Off-diagonal pairs read both row groups,
// so the stash is read (number of super blocks + 1)/2 times on average; this path serves the large-batch
// stress shape, where the contraction dominates anyway.  Partials: [gridDim.x][nbp*nbp blocks][16][64].
struct LargeParams {
  const u16* stash;
  long long seq_stride, p0, p1;
  int n_seq, first, nsb, nbp;       // super blocks, padded 32-row blocks per side (4 * nsb)
  float* partials;
  long long slot_floats;
};

template <bool DIAG>
__global__ __launch_bounds__(256) void stash_gram_pair_kernel(LargeParams p) {
  constexpr int ROWS = DIAG ? 128 : 256;
  constexpr int RB = kStageBytes / ROWS;            // 256 or 128 bytes per row and stage
  constexpr int KW = RB / 2;
  constexpr int VPR = RB / 16;                       // 16 or 8
  constexpr int RPL = 1024 / RB;                     // 4 or 8 rows per wave-load
  constexpr int LPW = kStageBytes / 1024 / 4;        // 8
  constexpr int STEPS = KW / 16;                     // every wave walks all steps of a stage
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const unsigned smem_base = (unsigned)(size_t)(lds_void_ptr)smem;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);

  // blockIdx.y enumerates the pairs of its kind: DIAG -> I = J = y; else the y-th pair with I < J
  int I, J;
  if (DIAG) {
    I = J = blockIdx.y;
  } else {
    int rem = blockIdx.y;
    I = 0;
    while (rem >= p.nsb - 1 - I) { rem -= p.nsb - 1 - I; ++I; }
    J = I + 1 + rem;
  }

  const long long n_elems = p.p1 - p.p0;
  const long long n_super = (n_elems + KW - 1) / KW;
  const long long my_first = blockIdx.x;
  const long long my_count = my_first < n_super ? (n_super - my_first + gridDim.x - 1) / gridDim.x : 0;

  const char* src[LPW];
  int vec_off[LPW];
#pragma unroll
  for (int q = 0; q < LPW; ++q) {
    const int row = (wave * LPW + q) * RPL + lane / VPR;               // row of the stage
    const int pos = lane % VPR;
    const int g = pos ^ (row & (VPR - 1));
    int seq = (row < 128 ? I * 128 + row : J * 128 + (row - 128));
    if (seq >= p.n_seq) seq = p.n_seq - 1;                             // padded rows: entries never written
    src[q] = reinterpret_cast<const char*>(p.stash + (size_t)seq * p.seq_stride + p.p0);
    vec_off[q] = g * 16;
  }
  auto issue = [&](long long k) {
    const long long e0 = (my_first + k * gridDim.x) * KW;
    const unsigned stage = smem_base + (unsigned)(k % kStages) * kStageBytes;
#pragma unroll
    for (int q = 0; q < LPW; ++q) {
      long long byte = e0 * 2 + vec_off[q];
      const long long last = (n_elems - 8) * 2;
      if (byte > last) byte = last;
      if (k >= my_count) byte = 0;
      load_lds16(src[q] + byte, stage + (unsigned)(wave_s * LPW + q) * 1024);
    }
  };

  f32x16 acc[4];
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
  const int frow = lane & 31, half = lane >> 5;

#pragma unroll
  for (int s = 0; s < kStages - 1; ++s) issue(s);
  for (long long k = 0; k < my_count; ++k) {
    __builtin_amdgcn_s_waitcnt(0x0f70 | (((kStages - 2) * LPW) & 15) | ((((kStages - 2) * LPW) >> 4) << 14));
    __builtin_amdgcn_s_barrier();
    issue(k + kStages - 1);
    const unsigned sb = smem_base + (unsigned)(k % kStages) * kStageBytes;
    const long long valid = n_elems - (my_first + k * gridDim.x) * KW;
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      const int vec = st * 2 + half;
      const bool dead = valid < KW && (long long)vec * 8 >= valid;
      const int ra = wave * 32 + frow;
      v4u fa = *(lds_v4u_ptr)(sb + (unsigned)ra * RB + (unsigned)((vec ^ (ra & (VPR - 1))) * 16));
      if (dead) fa = v4u{0u, 0u, 0u, 0u};
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int rb = (DIAG ? 0 : 128) + b * 32 + frow;
        v4u fb = *(lds_v4u_ptr)(sb + (unsigned)rb * RB + (unsigned)((vec ^ (rb & (VPR - 1))) * 16));
        if (dead) fb = v4u{0u, 0u, 0u, 0u};
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa), __builtin_bit_cast(bf16x8, fb),
                                                         acc[b], 0, 0, 0);
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);

  float* out = p.partials + (long long)blockIdx.x * p.slot_floats;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const int bi = 4 * I + wave, bj = 4 * J + b;
    float* o = out + ((long long)(bi * p.nbp + bj) * 16) * 64 + lane;
#pragma unroll
    for (int v = 0; v < 16; ++v) o[v * 64] = (p.first ? 0.f : o[v * 64]) + acc[b][v];
  }
}

// ---- 129..256 sequences in one pass ---------------------------------------------------------------
// A 128-element slice of all 256 rows is two 32 KiB half-stages (rows 0..127 and 128..255, 256 bytes
// per row: shorter runs per row stream noticeably slower from HBM).  LDS holds a ring of five
// half-stages: two are multiplied while three are in flight.  The 36 upper-triangle 32x32 blocks of the
// 8x8 block grid are dealt to the four waves by block row: wave w takes rows w and 7-w, nine blocks
// each, and reads the row-block fragments it needs per 16-element step.  Every wave walks every step.
// The fragments of step s + 1 are read between the MFMAs of step s (two register sets), so no MFMA
// waits for the LDS.  A slice that is not whole (only the last one of [p0, p1) can be) takes a plain
// masking loop after the main one.  The stash is read exactly once; partials have the large path's layout.
constexpr int kWideHalves = 5;

template <int W>
__device__ __forceinline__ void wide_body(const LargeParams& p, unsigned smem_base, int lane, int wave_s,
                                          const char* const (&src)[2][8], const int (&vec_off)[8],
                                          long long n_elems, long long my_first, long long my_count) {
  constexpr int RB = 256, KW = 128, VPR = 16, LPW = 8, STEPS = 8;
  constexpr int R0 = W, R1 = 7 - W;                  // this wave's two block rows
  auto issue = [&](long long j) {                    // half-stage j = 2 * slice + half
    const long long e0 = (my_first + (j >> 1)) * KW;
    const unsigned stage = smem_base + (unsigned)(j % kWideHalves) * kStageBytes;
    const int h = (int)(j & 1);
#pragma unroll
    for (int q = 0; q < LPW; ++q) {
      long long byte = e0 * 2 + vec_off[q];
      const long long last = (n_elems - 8) * 2;
      if (byte > last) byte = last;
      if ((j >> 1) >= my_count) byte = 0;
      load_lds16_nt((h ? src[1][q] : src[0][q]) + byte, stage + (unsigned)(wave_s * LPW + q) * 1024);
    }
  };
  f32x16 acc[9];
#pragma unroll
  for (int b = 0; b < 9; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
  const int frow = lane & 31, half = lane >> 5;
  // the nine products of one 16-element step from this wave's fragments of row blocks R0..7
  auto multiply = [&](const v4u (&frag)[8]) {
    int q = 0;
#pragma unroll
    for (int bj = R0; bj < 8; ++bj, ++q)
      acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, frag[R0]),
                                                       __builtin_bit_cast(bf16x8, frag[bj]), acc[q], 0, 0, 0);
#pragma unroll
    for (int bj = R1; bj < 8; ++bj, ++q)
      acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, frag[R1]),
                                                       __builtin_bit_cast(bf16x8, frag[bj]), acc[q], 0, 0, 0);
  };
  auto read_step = [&](v4u (&frag)[8], unsigned sb0, unsigned sb1, int st) {
    const int vec = st * 2 + half;
#pragma unroll
    for (int b = R0; b < 8; ++b) {                   // row blocks below R0 pair with no block of this wave
      const int row = (b & 3) * 32 + frow;
      frag[b] = *(lds_v4u_ptr)((b < 4 ? sb0 : sb1) + (unsigned)row * RB + (unsigned)((vec ^ (row & (VPR - 1))) * 16));
    }
  };

  // Only the very last slice of [p0, p1) can be short; it goes through the masking loop below.
  const bool short_tail = (n_elems % KW) != 0 && my_first + my_count == (n_elems + KW - 1) / KW;
  const long long n_whole = my_count - (short_tail ? 1 : 0);

  issue(0); issue(1); issue(2);
  for (long long k = 0; k < n_whole; ++k) {
    // half-stages 2k and 2k+1 landed (only 2k+2 may still be out), then everyone's; the two half-stages of
    // slice k-1 are free after the barrier and take 2k+3 and 2k+4
    __builtin_amdgcn_s_waitcnt(0x0f70 | LPW);
    __builtin_amdgcn_s_barrier();
    issue(2 * k + 3);
    issue(2 * k + 4);
    const unsigned sb0 = smem_base + (unsigned)((2 * k) % kWideHalves) * kStageBytes;
    const unsigned sb1 = smem_base + (unsigned)((2 * k + 1) % kWideHalves) * kStageBytes;
    // Two fragment sets: the reads of step st + 1 go out between the MFMAs of step st, one read behind each
    // of the first MFMAs, so that no MFMA waits for the LDS and the four waves' reads are spread out.
    v4u frag[2][8];
    read_step(frag[0], sb0, sb1, 0);
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      if (st + 1 < STEPS) read_step(frag[(st + 1) & 1], sb0, sb1, st + 1);
      multiply(frag[st & 1]);
      if (st == 0) __builtin_amdgcn_sched_group_barrier(0x100, 8 - R0, 0);      // step 0's own reads first
      if (st + 1 < STEPS) {
#pragma unroll
        for (int r = 0; r < 8 - R0; ++r) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 9 - (8 - R0), 0);
      } else {
        __builtin_amdgcn_sched_group_barrier(0x008, 9, 0);
      }
    }
  }
  if (short_tail) {
    const long long k = n_whole;
    __builtin_amdgcn_s_waitcnt(0x0f70 | LPW);
    __builtin_amdgcn_s_barrier();
    issue(2 * k + 3);
    issue(2 * k + 4);
    const unsigned sb0 = smem_base + (unsigned)((2 * k) % kWideHalves) * kStageBytes;
    const unsigned sb1 = smem_base + (unsigned)((2 * k + 1) % kWideHalves) * kStageBytes;
    const long long valid = n_elems - (my_first + k) * KW;
#pragma unroll 1
    for (int st = 0; st < STEPS; ++st) {
      const int vec = st * 2 + half;
      const bool dead = (long long)vec * 8 >= valid;
      v4u frag[8];
      read_step(frag, sb0, sb1, st);
#pragma unroll
      for (int b = R0; b < 8; ++b)
        if (dead) frag[b] = v4u{0u, 0u, 0u, 0u};
      multiply(frag);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);

  float* out = p.partials + (long long)blockIdx.x * p.slot_floats;
  int q = 0;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int bi = pass == 0 ? R0 : R1;
#pragma unroll
    for (int bj = bi; bj < 8; ++bj, ++q) {
      float* o = out + ((long long)(bi * 8 + bj) * 16) * 64 + lane;
#pragma unroll
      for (int v = 0; v < 16; ++v) o[v * 64] = (p.first ? 0.f : o[v * 64]) + acc[q][v];
    }
  }
}

__global__ __launch_bounds__(256) void stash_gram_wide_kernel(LargeParams p) {
  constexpr int KW = 128, VPR = 16, RPL = 4, LPW = 8;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const unsigned smem_base = (unsigned)(size_t)(lds_void_ptr)smem;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const long long n_elems = p.p1 - p.p0;
  const long long n_super = (n_elems + KW - 1) / KW;
  // a contiguous run of slices per workgroup: each of its 256 row streams walks consecutive cache lines
  const long long my_first = n_super * blockIdx.x / gridDim.x;
  const long long my_count = n_super * (blockIdx.x + 1) / gridDim.x - my_first;
  const char* src[2][LPW];
  int vec_off[LPW];
#pragma unroll
  for (int q = 0; q < LPW; ++q) {
    const int row = (wave * LPW + q) * RPL + lane / VPR;                // row within a half-stage, 0..127
    const int pos = lane % VPR;
    vec_off[q] = (pos ^ (row & (VPR - 1))) * 16;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int r = h * 128 + row;
      const int seq = r < p.n_seq ? r : p.n_seq - 1;                    // padded rows: entries never written
      src[h][q] = reinterpret_cast<const char*>(p.stash + (size_t)seq * p.seq_stride + p.p0);
    }
  }
  // every wave runs the same loop (same barriers), specialised on its block rows
  switch (wave_s) {
    case 0: wide_body<0>(p, smem_base, lane, wave_s, src, vec_off, n_elems, my_first, my_count); break;
    case 1: wide_body<1>(p, smem_base, lane, wave_s, src, vec_off, n_elems, my_first, my_count); break;
    case 2: wide_body<2>(p, smem_base, lane, wave_s, src, vec_off, n_elems, my_first, my_count); break;
    default: wide_body<3>(p, smem_base, lane, wave_s, src, vec_off, n_elems, my_first, my_count); break;
  }
}

// grid: one 1024-thread block per (block bi <= bj, v); 16 waves add the slots, then wave order.
__global__ __launch_bounds__(1024) void stash_gram_large_finish_kernel(const float* __restrict__ partials, int n_slots,
                                                                       long long slot_floats, int n_seq, int nbp,
                                                                       float* __restrict__ K) {
  __shared__ float red[16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int blk = blockIdx.x >> 4, v = blockIdx.x & 15;
  const int bi = blk / nbp, bj = blk % nbp;
  if (bi > bj || bi * 32 >= n_seq || bj * 32 >= n_seq) return;
  const long long e = ((long long)blk * 16 + v) * 64 + lane;
  float s = 0.f;
  for (int w = wave; w < n_slots; w += 16) s += partials[(long long)w * slot_floats + e];
  red[wave][lane] = s;
  __syncthreads();
  if (wave != 0) return;
  s = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) s += red[w][lane];
  const int i = bi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3), j = bj * 32 + (lane & 31);
  if (i < n_seq && j < n_seq && i <= j) {
    K[(size_t)i * n_seq + j] = s;
    K[(size_t)j * n_seq + i] = s;
  }
}

template <bool DIAG>
hipError_t launch_pair(const LargeParams& p, int gx, int n_pairs, hipStream_t s) {
  if (n_pairs <= 0) return hipSuccess;
  constexpr size_t smem = (size_t)kStages * kStageBytes;
  auto kern = stash_gram_pair_kernel<DIAG>;
  // once per process (static initialisation is thread-safe); a failure is returned by every call
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3(gx, n_pairs), dim3(256), smem, s, p);
  return hipGetLastError();
}

}  // namespace

int stash_gram_stream_slots() { return kBlocks; }

// Large batches (n_seq > 128).
int stash_gram_large_slots(int n_seq) {
  if (n_seq <= 256) return kBlocks;          // one-pass kernel: one persistent workgroup per CU
  const int nsb = (n_seq + 127) / 128;
  const int pairs = nsb * (nsb + 1) / 2;
  int gx = 512 / pairs;
  return gx < 16 ? 16 : (gx > 128 ? 128 : gx);
}
size_t stash_gram_large_slot_floats(int n_seq) {
  const int nbp = 4 * ((n_seq + 127) / 128);
  return (size_t)nbp * nbp * 1024;
}
hipError_t launch_stash_gram_large(const StashGramArgs& a, hipStream_t s) {
  if (!a.bf16 || a.n_seq <= 128) return hipErrorInvalidValue;
  LargeParams p;
  p.stash = static_cast<const u16*>(a.stash); p.seq_stride = a.seq_stride; p.p0 = a.p0; p.p1 = a.p1;
  p.n_seq = a.n_seq; p.first = a.first ? 1 : 0; p.partials = a.partials;
  p.nsb = (a.n_seq + 127) / 128; p.nbp = 4 * p.nsb;
  p.slot_floats = (long long)stash_gram_large_slot_floats(a.n_seq);
  const int gx = stash_gram_large_slots(a.n_seq);
  if (a.n_seq <= 256) {
    constexpr size_t smem = (size_t)kWideHalves * kStageBytes;          // 160 KiB: the whole LDS of a CU
    // once per process (static initialisation is thread-safe); a failure is returned by every call
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(stash_gram_wide_kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(stash_gram_wide_kernel, dim3(gx), dim3(256), smem, s, p);
    return hipGetLastError();
  }
  hipError_t e = launch_pair<true>(p, gx, p.nsb, s);
  if (e != hipSuccess) return e;
  return launch_pair<false>(p, gx, p.nsb * (p.nsb - 1) / 2, s);
}
hipError_t launch_stash_gram_large_finish(const float* partials, int n_seq, float* K, hipStream_t s) {
  const int nbp = 4 * ((n_seq + 127) / 128);
  hipLaunchKernelGGL(stash_gram_large_finish_kernel, dim3((unsigned)(nbp * nbp * 16)), dim3(1024), 0, s, partials,
                     stash_gram_large_slots(n_seq), (long long)stash_gram_large_slot_floats(n_seq), n_seq, nbp, K);
  return hipGetLastError();
}

hipError_t launch_stash_gram_stream(const StashGramArgs& a, hipStream_t s) {
  const int nb = (a.n_seq + 31) / 32;
  if (nb > 4 || !a.bf16 || a.n_seq < 1) return hipErrorInvalidValue;
  Params p;
  p.stash = static_cast<const u16*>(a.stash); p.seq_stride = a.seq_stride; p.p0 = a.p0; p.p1 = a.p1;
  p.n_seq = a.n_seq; p.first = a.first ? 1 : 0; p.partials = a.partials;
  p.slot_floats = (long long)stash_gram_slot_floats(a.n_seq);
  switch (nb) {
    case 1: return launch<1, 1>(p, s);
    case 2: return launch<2, 2>(p, s);
    case 3: return launch<3, 4>(p, s);
    default: return launch<4, 4>(p, s);
  }
}

}  // namespace isopo
