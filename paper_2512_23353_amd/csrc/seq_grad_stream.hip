// Token-reduction contraction, bf16, streaming variant: the kernel behind the
// per-sequence gradients G_i = Delta_i^T X_i (`grad_out.T @ act_in` of both hook
// listings) and behind the unweighted dW = Delta^T X.
//
// Design (gfx950):
//  * Operand tiles go from HBM/L2 straight into LDS with buffer_load ... lds
//    (16 bytes per lane, no VGPR staging, no LDS-write instructions).  The
//    buffer descriptor covers exactly the rows of the current token block, so
//    rows past the end of a sequence are out of range and arrive as zeros:
//    ragged tails cost no branches.  The loads' cursor moves on by additions, and
//    a block's descriptors are formed one block ahead, between MFMAs: what
//    stands ahead of a block's first MFMA every wave of the workgroup waits for.
//  * LDS holds a ring of NSTAGE token blocks ([token][feature], the HBM layout).
//    NSTAGE-1 blocks are in flight while one is multiplied; one s_barrier per block.
//  * MFMA fragments need 8 consecutive tokens of one feature per lane; they come
//    from the LDS transpose read (ds_read_b64_tr_b16).  Rows are not padded:
//    the 16-byte column index is XOR-swizzled with the token row
//    (f(r) = 4*(r&3) ^ (r&2)), which makes both the linear DMA writes and the
//    transpose reads bank-conflict free.
//  * Two inner loops.  The tile-order stash and the sum over all tokens use the
//    16x16x32 MFMA (less energy per flop, and the part runs at its power cap): a
//    token block is one K = 32 step of 64 MFMAs per wave (32 with eight waves per
//    workgroup, which the sums over all tokens use on the 256x256 tile); the DMA
//    instructions of the block NSTAGE-1 ahead (eight per wave, or four) go out
//    behind the first half of them, the barrier sits mid-block, the next block's
//    fragments are read behind the second half.  The row-major stash keeps the 32x32x16 MFMA, whose
//    accumulator blocks its transposing epilogue is written for: fragments
//    double-buffered in registers, the reads of the next half block interleaved
//    one-to-one with the MFMAs of the current one, the DMA instructions between
//    the MFMAs of the second half block.
//  * Per-sequence mode: XCD x owns the x-th eighth of the output tiles of every
//    sequence, so all eight L2s see every sequence (balanced under ragged
//    lengths) and neighbouring workgroups share operand panels.  When the tile
//    count is no multiple of eight that would leave XCDs unevenly loaded (or
//    idle); the host then cuts the sequence-major list of (sequence, tile) pairs
//    into eight contiguous ranges of equal work (tokens plus a fixed charge per
//    workgroup) and each XCD walks one.  For a row-major stash the bf16 tile is
//    transposed through LDS in the epilogue so that every lane stores 16 bytes;
//    for a stash in tile order (TILED) every lane stores the 16 bytes it holds,
//    with no LDS round trip at all.
//  * Sum-over-all-tokens mode with few output tiles (narrow projections, long
//    microbatches): the token range is split into chunks, a workgroup takes one
//    (chunk, tile) pair from its XCD's range of the same kind of list, and the
//    fp32 partial tiles are added to dW with hardware float atomics after a pass
//    that applies beta.  With more tiles than compute units only the tiles of the
//    last, partial round of one tile per unit are split; the others stay whole.
#include "common.h"
#include "kernels.h"

#include <type_traits>

namespace isopo {
namespace {

typedef unsigned short u16;
typedef s16x4 __attribute__((address_space(3)))* lds_s16x4_ptr;
typedef void __attribute__((address_space(3)))* lds_void_ptr;
typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));

struct StreamParams {
  const u16* X;
  const u16* Delta;
  const int32_t* off;
  const float* c;                  // weighted sum over all tokens: one coefficient per sequence
  void* out;
  int d_in, d_out, n_seq, n_tokens;
  int row0, row_end, out_row0;
  long long out_seq_stride;
  float beta;
  int tiles_m, tiles_n;
  unsigned n_blocks;
  int n_chunks, chunk_tokens;      // sum-over-all-tokens mode: token chunks (1: no split)
  int whole_tiles;                 // sum-over-all-tokens mode: tiles before this one are not split
  int xcd_start[9];                // XCD x takes (item, tile) pairs [xcd_start[x], xcd_start[x+1]), item-major
  unsigned* queue;                 // persistent mode: eight work counters, one per XCD, zero at launch
};

// 16 bytes per lane from a buffer straight into LDS: lane l lands at lds_addr + 16*l.
// Inline asm, so that the compiler's LDS-DMA tracking does not put a vmcnt(0) before
// every later LDS read; the kernel orders them itself with s_waitcnt vmcnt(n) + s_barrier.
__device__ __forceinline__ void load_lds16(v4i rsrc, unsigned lds_addr, unsigned voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               : : "s"(lds_addr), "v"(voff), "s"(rsrc) : "memory");
}

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Two fp32 -> one dword of two bf16 (round to nearest even), one v_cvt_pk_bf16_f32.
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// Accumulator element -> VGPR at the point of use.  Without this the register allocator copies the
// whole 256-register tile out of the AGPRs before the epilogue and spills.
__device__ __forceinline__ float acc_read(float a) {
  float v;
  asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
  return v;
}

constexpr int BK = 32;

// Column-blocked tile order: ids run down 8-column strips of the tile grid, so the 32 workgroups an
// XCD runs at a time cover about 4 tile rows x 8 tile columns (12 operand panels) rather than
// 2 x 16 (18 panels): fewer L2 misses per flop.
__device__ __forceinline__ void strip_tile_coords(int tile, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
  constexpr int W = 8;
  const int strip = tile / (tiles_m * W);
  const int c0 = strip * W;
  const int w = tiles_n - c0 < W ? tiles_n - c0 : W;     // the last strip may be narrower
  const int in_strip = tile - strip * tiles_m * W;
  tile_m = in_strip / w;
  tile_n = c0 + in_strip % w;
}

// NW: waves per workgroup.  Four: a 2 x 2 arrangement of BM/2 x BN/2 wave tiles, one wave per SIMD on the
// 256x256 tile with its accumulators pinned to the AGPRs.  Eight (16x16x32 loop only): 2 x 4, wave tiles of
// BM/2 x BN/4, two waves per SIMD, 128 accumulators per lane in VGPRs, half the DMA instructions per wave, so
// that twice as many waves issue operand loads.  On the workload's operands, where the board's power limit sets
// the rate, the two are within a few per cent of each other: the per-sequence launch is no faster with eight
// and keeps four; the sums over all tokens are 1 - 5 % faster with eight (more where the launch is not at the
// power limit) and take eight on the 256x256 tile.
template <int BM, int BN, int NSTAGE, bool PER_SEQ, bool PERSIST, bool TILED, bool WTD, int NW>
__device__ __forceinline__ void seq_grad_stream_body(const StreamParams& p) {
  static_assert(PER_SEQ || !TILED, "tile order is a layout of the per-sequence stash");
  static_assert(!PER_SEQ || !WTD, "the coefficients weight the sum over all tokens");
  // the 16x16x32 inner loop: the tile-order stash and the sum over all tokens (the row-major stash keeps the
  // 32x32x16 loop, whose accumulator blocks its transposing epilogue is written for)
  constexpr bool MF16 = TILED || !PER_SEQ;
  static_assert(PER_SEQ || !PERSIST, "the persistent mode serves the per-sequence gradients");
  static_assert(NW == 4 || (NW == 8 && (TILED || !PER_SEQ)), "eight waves: the 16x16x32 loop only");
  constexpr int WNC = NW / 2, NT = 64 * NW;                    // waves along the tile's columns; threads
  constexpr int WM = BM / 2, WN = BN / WNC, FM = WM / 32, FN = WN / 32;
  constexpr unsigned PA = BM * 2, PB = BN * 2;                 // LDS row pitch, bytes (no padding: swizzled)
  constexpr unsigned A_BYTES = BK * PA, B_BYTES = BK * PB, STAGE = A_BYTES + B_BYTES;
  constexpr int LA = A_BYTES / 1024 / NW, LB = B_BYTES / 1024 / NW;   // 1 KiB wave-loads per wave and tile
  constexpr int RA = 1024 / PA, RB = 1024 / PB;                // tile rows per wave-load
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const unsigned smem_base = (unsigned)(size_t)(lds_void_ptr)smem;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WNC, wn = wave % WNC;

  // Persistent mode (per-sequence only): the grid is a chosen number of workgroups, a multiple of eight;
  // the workgroups of XCD x pull that XCD's work items one at a time from the counter queue[x].  The
  // launch then occupies that many compute units and no more, and kernels queued on other streams (the
  // passes over the previous layer's stash) run on the rest.
  __shared__ int sh_next;
  for (int round = 0;; ++round) {
    int e;
    if constexpr (PERSIST) {
      if (round > 0) {
        // nobody still reads the previous item's LDS (epilogue staging) or its sh_next
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_s_barrier();
      }
      if (tid == 0) sh_next = (int)atomicAdd(p.queue + (blockIdx.x & 7), 1u);
      __syncthreads();
      e = sh_next;
    } else {
      e = (int)(blockIdx.x >> 3);
    }
    int item, tile;
    bool split = !PER_SEQ && p.n_chunks > 1;       // this workgroup adds a token chunk's part with atomics
    if (!PER_SEQ && p.whole_tiles > 0) {
      // Whole tiles first, then the token chunks of the remaining tiles; XCD x takes the x-th eighth of
      // each of the two lists, in id order, so a compute unit gets chunks once its whole tiles are done.
      const int x = blockIdx.x & 7, wq = p.whole_tiles >> 3;
      if (e < wq) {
        item = 0;
        tile = x * wq + e;
        split = false;
      } else {
        const int rest = p.tiles_m * p.tiles_n - p.whole_tiles, S = rest * p.n_chunks;
        const int first = (int)((long long)x * S / 8);
        const int id = first + (e - wq);
        if (id >= (int)((long long)(x + 1) * S / 8)) break;
        item = id / rest;
        tile = p.whole_tiles + id % rest;
      }
    } else if (PER_SEQ || split) {
      const int tiles = p.tiles_m * p.tiles_n;
      const int x = blockIdx.x & 7;
      if (p.xcd_start[8] > 0) {
        // XCD x (= blockIdx % 8) walks a contiguous range of the item-major (item, tile) list; the host cut
        // the list into eight ranges of equal work
        const int id = p.xcd_start[x] + e;
        if (id >= p.xcd_start[x + 1]) break;
        item = id / tiles;
        tile = id - item * tiles;
      } else {
        // XCD x owns tiles [x*tiles/8, (x+1)*tiles/8) of every sequence (or token chunk)
        const int s0 = x * tiles / 8, cs = (x + 1) * tiles / 8 - s0;
        if (cs == 0 || e >= (PER_SEQ ? p.n_seq : p.n_chunks) * cs) break;
        item = e / cs;
        tile = s0 + e % cs;
      }
    } else {
      item = 0;
      tile = xcd_contiguous(blockIdx.x, p.n_blocks);
    }
    int tile_m, tile_n;
    strip_tile_coords(tile, p.tiles_m, p.tiles_n, tile_m, tile_n);
    const int m0 = p.row0 + tile_m * BM, n0 = tile_n * BN;
    const int t0 = PER_SEQ ? p.off[item] : (split ? item * p.chunk_tokens : 0);
    const int t1 = PER_SEQ ? p.off[item + 1] : (split ? min(p.n_tokens, t0 + p.chunk_tokens) : p.n_tokens);
    const int n_rows = t1 - t0;
    int n_tiles = (n_rows + BK - 1) / BK;
    // Weighted sum over all tokens: the token range is walked segment by segment (a segment: the part of one
    // sequence inside [t0, t1), if it has tokens and a non-zero coefficient), each segment in token blocks of
    // its own, so that no block mixes two sequences (rows past a segment's end arrive as zeros).  The
    // accumulators hold the sum in units of the current segment's coefficient: tokens enter the MFMAs
    // unscaled, and where a new segment opens the accumulators are multiplied once by c_previous / c_new.
    // The epilogue multiplies by the last segment's coefficient.  No operand is scaled or rounded.
    constexpr int kMaxSeg = 1024;            // the library's limit on sequences per layer
    // What the loads take next: the address of the next token block's first row in Delta and in X, the rows
    // left of the range it lies in (<= 0: an all-zero block); weighted sum: the segment and its blocks left.
    struct Cursor { unsigned long long pa, pb; int rem, k, left; };
    [[maybe_unused]] int n_seg = 0;
    [[maybe_unused]] float last_c = 0.f;
    [[maybe_unused]] int* seg_tok = nullptr;
    [[maybe_unused]] int* seg_end = nullptr;
    [[maybe_unused]] float* seg_ratio = nullptr;
    if constexpr (WTD) {
      __shared__ int sh_seg_tok[kMaxSeg], sh_seg_end[kMaxSeg];
      __shared__ float sh_seg_c[kMaxSeg];
      __shared__ int sh_meta[2];
      __shared__ float sh_last_c;
      seg_tok = sh_seg_tok; seg_end = sh_seg_end; seg_ratio = sh_seg_c;
      if (wave == 0) {
        // the first sequence that reaches beyond t0
        int s_lo = 0;
        if (t0 > 0) {
          int lo = 0, hi = p.n_seq;
          while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (p.off[mid + 1] > t0) hi = mid; else lo = mid + 1;
          }
          s_lo = lo;
        }
        int count = 0, blocks = 0;
        for (int base = s_lo; base < p.n_seq; base += 64) {
          const int sq = base + lane;
          int a = 0, b = 0, o0 = 0x7fffffff;
          float cs = 0.f;
          if (sq < p.n_seq) {
            o0 = p.off[sq];
            a = max(o0, t0); b = min(p.off[sq + 1], t1); cs = p.c[sq];
          }
          const bool valid = b > a && cs != 0.f;          // a NaN coefficient is kept and spreads
          const unsigned long long mask = __ballot(valid);
          const int pos = count + __popcll(mask & ((1ull << lane) - 1ull));
          if (valid) {
            sh_seg_tok[pos] = a; sh_seg_end[pos] = b; sh_seg_c[pos] = cs;
            blocks += ((b - a + BK - 1) / BK + 1) & ~1;      // walked in an even number of blocks
          }
          count += __popcll(mask);
          if (__builtin_amdgcn_readfirstlane(o0) >= t1) break;    // this and all later sequences lie beyond t1
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) blocks += __shfl_xor(blocks, o, 64);
        if (lane == 0) { sh_meta[0] = count; sh_meta[1] = blocks; }
      }
      __syncthreads();
      n_seg = __builtin_amdgcn_readfirstlane(sh_meta[0]);
      n_tiles = __builtin_amdgcn_readfirstlane(sh_meta[1]);
      // coefficient -> ratio to the segment before (1 for the first), in place
      float ratio[kMaxSeg / NT];
#pragma unroll
      for (int q = 0; q < kMaxSeg / NT; ++q) {
        const int k = tid + NT * q;
        ratio[q] = (k > 0 && k < n_seg) ? sh_seg_c[k - 1] / sh_seg_c[k] : 1.f;
      }
      if (tid == 0) sh_last_c = n_seg > 0 ? sh_seg_c[n_seg - 1] : 0.f;
      __syncthreads();
#pragma unroll
      for (int q = 0; q < kMaxSeg / NT; ++q) {
        const int k = tid + NT * q;
        if (k < n_seg) sh_seg_c[k] = ratio[q];
      }
      __syncthreads();
      last_c = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, sh_last_c)));
    }
    // The loads run ahead of the multiplications.  Their cursor moves on by one token block per step with two
    // 64-bit additions (no multiplication of a token index by a row length on the way); the buffer descriptors
    // of a block cover its valid rows only.  Weighted sum: every segment is walked in an even number of blocks,
    // the last one all zero if need be, because the main loop takes two blocks per trip; one branch per block,
    // taken only where a segment ends.
    const unsigned rbA = (unsigned)p.d_out * 2u, rbB = (unsigned)p.d_in * 2u;
    auto uniform64 = [](unsigned long long a) {
      const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)a);
      const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32));
      return ((unsigned long long)hi << 32) | lo;
    };
    auto range_open = [&](Cursor& cur, int tok, int rows) {
      cur.pa = uniform64((unsigned long long)(p.Delta + (size_t)tok * p.d_out));
      cur.pb = uniform64((unsigned long long)(p.X + (size_t)tok * p.d_in));
      cur.rem = rows;
    };
    auto segment_open = [&](Cursor& cur) {
      if (cur.k < n_seg) {
        const int tok = __builtin_amdgcn_readfirstlane(seg_tok[cur.k]);
        const int len = __builtin_amdgcn_readfirstlane(seg_end[cur.k]) - tok;
        range_open(cur, tok, len);
        cur.left = ((len + BK - 1) / BK + 1) & ~1;
      } else {
        cur.rem = 0; cur.left = 0x7fffffff;                    // past the last segment: all-zero blocks
      }
    };
    // descriptors of the cursor's block, then one block on
    auto next_block = [&](Cursor& cur, v4i& ra, v4i& rb) {
      int rows;
      asm("s_max_i32 %0, %1, 0\n\ts_min_i32 %0, %0, %2" : "=s"(rows) : "s"(cur.rem), "n"(BK) : "scc");
      ra[0] = (int)(unsigned)cur.pa; ra[1] = (int)((unsigned)(cur.pa >> 32) & 0xffffu);
      ra[2] = (int)((unsigned)rows * rbA); ra[3] = 0x00020000;
      rb[0] = (int)(unsigned)cur.pb; rb[1] = (int)((unsigned)(cur.pb >> 32) & 0xffffu);
      rb[2] = (int)((unsigned)rows * rbB); rb[3] = 0x00020000;
      cur.pa += (unsigned long long)BK * rbA;
      cur.pb += (unsigned long long)BK * rbB;
      cur.rem -= BK;
      if constexpr (WTD) --cur.left;
    };
    // weighted sum, after next_block: on to the next segment once this one's blocks are out
    [[maybe_unused]] auto segment_step = [&](Cursor& cur) {
      if (__builtin_expect(cur.left == 0, 0)) {
        ++cur.k;
        segment_open(cur);
      }
    };
    Cursor ld;
    ld.k = 0; ld.left = 0;
    if constexpr (WTD) {
      ld.pa = 0; ld.pb = 0; ld.rem = 0;
      segment_open(ld);
    } else {
      range_open(ld, t0, n_rows);
    }

    // 16-byte column swizzle of token row r.  The 16x16x32 fragments (TILED) are read by lane groups whose
    // rows lie 8 apart, so that variant also moves rows 8..15 and 24..31 by two columns.
    auto swz = [](int r) { return ((r & 3) << 2) ^ (r & 2) ^ (MF16 ? ((r >> 3) & 1) << 1 : 0); };
    unsigned offA[LA], offB[LB];
#pragma unroll
    for (int q = 0; q < LA; ++q) {
      const int r = (wave * LA + q) * RA + lane / (64 / RA);
      const int g = (lane % (64 / RA)) ^ swz(r);
      offA[q] = (unsigned)r * rbA + (unsigned)(m0 * 2 + g * 16);
    }
#pragma unroll
    for (int q = 0; q < LB; ++q) {
      const int r = (wave * LB + q) * RB + lane / (64 / RB);
      const int g = (lane % (64 / RB)) ^ swz(r);
      offB[q] = (unsigned)r * rbB + (unsigned)(n0 * 2 + g * 16);
    }
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    auto issue_loads = [&](int it) {
      v4i ra, rb;
      next_block(ld, ra, rb);
      if constexpr (WTD) segment_step(ld);
      const unsigned stage = smem_base + ((unsigned)it % NSTAGE) * STAGE;
#pragma unroll
      for (int q = 0; q < LA; ++q) load_lds16(ra, stage + (unsigned)(wave_s * LA + q) * 1024, offA[q]);
#pragma unroll
      for (int q = 0; q < LB; ++q) load_lds16(rb, stage + A_BYTES + (unsigned)(wave_s * LB + q) * 1024, offB[q]);
    };

    if constexpr (MF16) {
      // ---- stash in tile order, and the sum over all tokens: the 16x16x32 MFMA, which draws less power per flop than the 32x32x16 one
      // (a loop of either on random operands in registers sustains 2.04 against 1.81 PFLOP/s under the
      // board's power cap).  A token block is one K = 32 step: 8 + 8 fragments (16 features x 32 tokens
      // each), FM16 x FN16 MFMAs row by row.  Behind row i go the next block's B fragment i (into the other
      // of two register sets) and, once the row is done with it, the next block's A fragment i (in place),
      // and a share of the eight DMA instructions of the block AHEAD ahead.  One barrier per block.
      constexpr int FM16 = WM / 16, FN16 = WN / 16, NMF16 = FM16 * FN16;
      static_assert(NMF16 - (FM16 / 2) * FN16 >= FN16 + FM16 / 2, "the second half's MFMAs carry the next block's fragment reads");
      constexpr int LPT = LA + LB, AHEAD = NSTAGE - 1;
      typedef float f32x4v __attribute__((ext_vector_type(4)));
      unsigned adA[FM16], adB[FN16];
      {
        // lane (l, g4): token rows 8 g4 + l / 4 (+ 4 for the second read), features 4 (l % 4) ..+3 of the
        // fragment's 16; the transposing read leaves lane l with tokens 8 g4 ..+7 of feature l
        const int l = lane & 15, g4 = lane >> 4;
        const int kr = 8 * g4 + (l >> 2);
        const int f = swz(kr);
#pragma unroll
        for (int i = 0; i < FM16; ++i) {
          const int ca = wm * WM + i * 16 + 4 * (l & 3);
          adA[i] = (unsigned)kr * PA + (unsigned)(((ca >> 3) ^ f) << 4) + (unsigned)((ca & 7) * 2);
        }
#pragma unroll
        for (int j = 0; j < FN16; ++j) {
          const int cb = wn * WN + j * 16 + 4 * (l & 3);
          adB[j] = A_BYTES + (unsigned)kr * PB + (unsigned)(((cb >> 3) ^ f) << 4) + (unsigned)((cb & 7) * 2);
        }
      }
      auto frag = [&](unsigned a, unsigned pitch) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(a));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(a + 4 * pitch));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      };
      f32x4v acc[FM16][FN16];
#pragma unroll
      for (int i = 0; i < FM16; ++i)
#pragma unroll
        for (int j = 0; j < FN16; ++j)
#pragma unroll
          for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
      bf16x8 fa[FM16], fb[2][FN16];
#pragma unroll
      for (int s = 0; s < AHEAD; ++s) issue_loads(s);
      if (n_tiles > 0) {
        __builtin_amdgcn_s_waitcnt(0x0f70 | (((AHEAD - 1) * LPT) & 15) | ((((AHEAD - 1) * LPT) >> 4) << 14));
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int i = 0; i < FM16; ++i) fa[i] = frag(smem_base + adA[i], PA);
#pragma unroll
        for (int j = 0; j < FN16; ++j) fb[0][j] = frag(smem_base + adB[j], PB);
        // The descriptors of the next block's loads are formed a block ahead, behind the barrier, so that this
        // scalar work issues between MFMAs and not ahead of a block's first one.
        constexpr bool PIPE = true;
        [[maybe_unused]] v4i ra_n, rb_n;
        if constexpr (PIPE) {
          next_block(ld, ra_n, rb_n);
          if constexpr (WTD) segment_step(ld);
        }
        // LATE: the two waves of the lower tile half take the other of every two read slots, so that the LDS
        // serves two waves' fragment reads at a time, not four (compile-time, as CUR, so that the bodies stay
        // straight-line code)
        // SCALE (weighted sum only): 1 in a segment's first block, 2 in its last.  The accumulators change their
        // unit from the previous segment's coefficient to this one's by a factor r; those of the first RB rows
        // take it in the last block of the segment before, behind the MFMAs of the other rows, the others in
        // this segment's first block, behind the MFMAs of the first RB rows: every accumulator is multiplied
        // once between its last MFMA of one segment and its first of the next, and the matrix pipes never wait
        // for the multiplications.
        auto token_block = [&](int it, auto cur_c, auto late_c, auto scale_c, [[maybe_unused]] float r) {
          constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1;
          constexpr bool LATE = decltype(late_c)::value;
          constexpr int SCALE = decltype(scale_c)::value;
          static_assert(SCALE == 0 || NMF16 * 4 <= 128, "the multiplications are written for accumulators in VGPRs");
          const unsigned sn = smem_base + ((unsigned)(it + 1) % NSTAGE) * STAGE;
          v4i ra, rb;                              // of block it + AHEAD
          if constexpr (PIPE) { ra = ra_n; rb = rb_n; } else next_block(ld, ra, rb);
          const unsigned stage = smem_base + ((unsigned)(it + AHEAD) % NSTAGE) * STAGE;
          // When the accumulator tile fills the AGPRs the MFMA is written as asm, so that every accumulator
          // stays where it is (left to itself the register allocator shuttles them through VGPRs).
#define ISOPO_MFMA16(i, j)                                                                                            \
  do {                                                                                                                \
    if constexpr (NMF16 * 4 > 128) {                                                                                  \
      asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fa[i]), "v"(fb[CUR][j]));       \
    } else {                                                                                                          \
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[CUR][j], acc[i][j], 0, 0, 0);                     \
    }                                                                                                                 \
  } while (0)
          // the first RB rows of the wave tile: their MFMAs carry the DMA instructions of the block AHEAD ahead
          // (its stage, that of block it - 1, was last read before the barrier of block it - 1)
          constexpr int RB = FM16 / 2, HEAD = RB * FN16, REST = NMF16 - HEAD;
#pragma unroll
          for (int i = 0; i < RB; ++i)
#pragma unroll
            for (int j = 0; j < FN16; ++j) {
              const int idx = i * FN16 + j;
              ISOPO_MFMA16(i, j);
              if constexpr (SCALE == 1) {
#pragma unroll
                for (int q = idx * REST / HEAD; q < (idx + 1) * REST / HEAD; ++q)
                  acc[RB + q / FN16][q % FN16] = acc[RB + q / FN16][q % FN16] * r;
              }
#pragma unroll
              for (int q = idx * LPT / HEAD; q < (idx + 1) * LPT / HEAD; ++q) {
                // builtin MFMAs: the scheduler would move every load to the top of the block, ahead of the MFMAs
                if constexpr (NMF16 * 4 <= 128) __builtin_amdgcn_sched_barrier(0);
                if (q < LA) load_lds16(ra, stage + (unsigned)(wave_s * LA + q) * 1024, offA[q]);
                else load_lds16(rb, stage + A_BYTES + (unsigned)(wave_s * LB + (q - LA)) * 1024, offB[q - LA]);
              }
            }
          // block it + 1 has landed (this wave's part; the barrier makes it everyone's)
          __builtin_amdgcn_s_waitcnt(0x0f70 | (((AHEAD - 1) * LPT) & 15) | ((((AHEAD - 1) * LPT) >> 4) << 14));
          __builtin_amdgcn_s_barrier();
          // the descriptors the next block's loads need: scalar work that issues between this half's MFMAs
          // instead of ahead of the next block's first one
          if constexpr (PIPE) next_block(ld, ra_n, rb_n);
          // the other rows: behind their MFMAs the fragments of block it + 1, the B ones into the other register
          // set, the A ones in place: those of the first RB rows at once, the others as their rows end
#pragma unroll
          for (int i = RB; i < FM16; ++i)
#pragma unroll
            for (int j = 0; j < FN16; ++j) {
              ISOPO_MFMA16(i, j);
              const int k = (i - RB) * FN16 + j;                      // 0 .. REST - 1
              if constexpr (SCALE == 2) {
#pragma unroll
                for (int q = k * HEAD / REST; q < (k + 1) * HEAD / REST; ++q)
                  acc[q / FN16][q % FN16] = acc[q / FN16][q % FN16] * r;
              }
              constexpr int PER = REST / (FN16 + RB);                 // MFMAs per fragment slot
              if (j == (LATE && PER > 1 ? 1 : 0) && i > RB) fa[i - 1] = frag(sn + adA[i - 1], PA);
              if (k % PER == (LATE ? 0 : PER - 1)) {
                const int f = k / PER;
                if (f < FN16) fb[NXT][f] = frag(sn + adB[f], PB);
                else if (f < FN16 + RB) fa[f - FN16] = frag(sn + adA[f - FN16], PA);
              }
            }
          fa[FM16 - 1] = frag(sn + adA[FM16 - 1], PA);
          // weighted sum: the cursor's branch (taken where a segment ends) closes the block.  Behind the barrier
          // it would cut the block in two there, with the scalar work of the second part standing between the
          // barrier and the MFMAs that follow it.
          if constexpr (WTD) segment_step(ld);
#undef ISOPO_MFMA16
        };
        // two blocks per trip (the B fragments alternate between two register sets); an odd count runs one
        // block past the end, whose rows are all out of range and arrive as zeros
        auto walk = [&](auto late_c) {
          if constexpr (WTD) {
            // segment by segment, each an even number of blocks (two at least): the first block and the last
            // carry the change of unit (ratio 1 before the first segment and after the last)
            constexpr std::integral_constant<int, 0> c0{};
            constexpr std::integral_constant<int, 1> c1{};
            constexpr std::integral_constant<int, 2> c2{};
            auto ratio_of = [&](int k) {
              return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, seg_ratio[k])));
            };
            int it = 0;
            float r_in = 1.f;
            for (int k = 0; k < n_seg; ++k) {
              const int len = __builtin_amdgcn_readfirstlane(seg_end[k]) - __builtin_amdgcn_readfirstlane(seg_tok[k]);
              const int blocks = ((len + BK - 1) / BK + 1) & ~1;
              const float r_out = k + 1 < n_seg ? ratio_of(k + 1) : 1.f;
              token_block(it, c0, late_c, c1, r_in);
              for (int b = 2; b < blocks; b += 2, it += 2) {
                token_block(it + 1, c1, late_c, c0, 0.f);
                token_block(it + 2, c0, late_c, c0, 0.f);
              }
              token_block(it + 1, c1, late_c, c2, r_out);
              it += 2;
              r_in = r_out;
            }
          } else {
            for (int it = 0; it < n_tiles; it += 2) {
              token_block(it, std::integral_constant<int, 0>{}, late_c, std::integral_constant<int, 0>{}, 0.f);
              token_block(it + 1, std::integral_constant<int, 1>{}, late_c, std::integral_constant<int, 0>{}, 0.f);
            }
          }
        };
        if (NMF16 * 4 > 128 && (wave_s & 2)) walk(std::true_type{}); else walk(std::false_type{});
      }
      __builtin_amdgcn_s_waitcnt(0x0f70);
      // Epilogue: lane l holds, of block (i, j), rows 4 (l / 16) ..+3 of column l % 16.
      asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");       // the last MFMAs have retired
      auto rd16 = [](float a) {
        if constexpr (NMF16 * 4 > 128) return acc_read(a); else return a;
      };
      (void)rd16;
      if constexpr (!PER_SEQ) {
        // dW: sixteen lanes store (or add) sixteen consecutive floats of a row
        const int col = lane & 15, rq = lane >> 4;
#pragma unroll
        for (int i = 0; i < FM16; ++i)
#pragma unroll
          for (int j = 0; j < FN16; ++j) {
            const int n = n0 + wn * WN + j * 16 + col;
            if (n >= p.d_in) continue;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const int m = m0 + wm * WM + i * 16 + 4 * rq + v;
              if (m >= p.row_end) continue;
              float* o = static_cast<float*>(p.out) + (size_t)(m - p.out_row0) * p.d_in + n;
              const float val = WTD ? last_c * rd16(acc[i][j][v]) : rd16(acc[i][j][v]);
              if (split) atomicAdd(o, val);        // beta already applied by the pass before
              else *o = (p.beta != 0.f ? p.beta * *o : 0.f) + val;
            }
          }
        if constexpr (PERSIST) continue; else break;
      }
      // Tile order: two blocks side by side make the lane's 16 bytes; a piece (two blocks, 512 elements) is
      // one 1 KiB store of the wave.
      typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
      const int tile_row = (m0 - p.out_row0) / BM;
      // the wave's quadrant of the tile, and inside each 16-row strip of the quadrant the wave's pieces (all of
      // them with four waves, the left or the right half with eight)
      constexpr int QP = (BN / 2) / 32;                        // pieces per strip of a quadrant
      const int quad = wm * 2 + wn / (WNC / 2), piece0 = (wn % (WNC / 2)) * (FN16 / 2);
      u16* tb = static_cast<u16*>(p.out) + (size_t)item * p.out_seq_stride +
                ((size_t)tile_row * p.tiles_n + tile_n) * (BM * BN) + (size_t)quad * ((BM / 2) * (BN / 2));
#pragma unroll
      for (int i = 0; i < FM16; ++i)
#pragma unroll
        for (int jp = 0; jp < FN16 / 2; ++jp) {
          u32x4 pk;
          pk[0] = pack_bf16(rd16(acc[i][2 * jp][0]), rd16(acc[i][2 * jp][1]));
          pk[1] = pack_bf16(rd16(acc[i][2 * jp][2]), rd16(acc[i][2 * jp][3]));
          pk[2] = pack_bf16(rd16(acc[i][2 * jp + 1][0]), rd16(acc[i][2 * jp + 1][1]));
          pk[3] = pack_bf16(rd16(acc[i][2 * jp + 1][2]), rd16(acc[i][2 * jp + 1][3]));
          // written once and read after the launch: non-temporal, so the stash does not push the operand
          // panels out of the L2
          __builtin_nontemporal_store(pk, (u32x4*)(tb + (i * QP + piece0 + jp) * 512 + lane * 8));
        }
      if constexpr (PERSIST) continue; else break;
    }
    // ---- row-major stash: the 32x32x16 MFMA (every other mode has left the round above)
    unsigned adA[FM], adB[FN];
    {
      const int l = lane & 15, g4 = lane >> 4;
      const int kr = 8 * (g4 >> 1) + (l >> 2);
      const int f = ((kr & 3) << 2) ^ (kr & 2);
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int ca = wm * WM + i * 32 + 16 * (g4 & 1) + 4 * (l & 3);
        adA[i] = (unsigned)kr * PA + (unsigned)(((ca >> 3) ^ f) << 4) + (unsigned)((ca & 7) * 2);
      }
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int cb = wn * WN + j * 32 + 16 * (g4 & 1) + 4 * (l & 3);
        adB[j] = A_BYTES + (unsigned)kr * PB + (unsigned)(((cb >> 3) ^ f) << 4) + (unsigned)((cb & 7) * 2);
      }
    }
    auto frA = [&](unsigned a) {
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(a));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(a + 4 * PA));
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto frB = [&](unsigned a) {
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(a));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(a + 4 * PB));
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    bf16x8 fa0[FM], fb0[FN], fa1[FM], fb1[FN];
    constexpr int LPT = LA + LB;   // loads per wave and tile
    // Token blocks in flight ahead of the one being multiplied: one less than the ring holds (the stash
    // stores compete with the operand fetches; a fourth block in flight made this mode slower).
    constexpr int AHEAD = NSTAGE - 1;
    constexpr int NMF = FM * FN;

    // Per-sequence mode, 256x256 tile: the two waves of the lower tile half read their fragments behind
    // MFMAs 8..15 of a half block instead of 0..7, in the order the next half block first uses them
    // (B0, A0, B1, B2, B3, A1, A2, A3), so the LDS serves two waves' reads at a time, not four.
    // frag_of: the fragment read behind MFMA idx (-1: none).
    auto frag_of = [](int idx, bool late, bool& is_a) -> int {
      const int k = idx - (late ? NMF - FM - FN : 0);
      if (k < 0 || k >= FM + FN) return -1;
      if (!late) { is_a = k < FM; return is_a ? k : k - FM; }
      if (k == 0) { is_a = false; return 0; }
      if (k == 1) { is_a = true; return 0; }
      if (k <= FN) { is_a = false; return k - 1; }
      is_a = true; return k - FN;
    };
    const bool late_wave = NMF >= 2 * (FM + FN) && (wave_s & 2);

#pragma unroll
    for (int s = 0; s < AHEAD; ++s) issue_loads(s);

    if (n_tiles > 0) {
      __builtin_amdgcn_s_waitcnt(0x0f70 | (((AHEAD - 1) * LPT) & 15) | ((((AHEAD - 1) * LPT) >> 4) << 14));
      __builtin_amdgcn_s_barrier();
#pragma unroll
      for (int i = 0; i < FM; ++i) fa0[i] = frA(smem_base + adA[i]);
#pragma unroll
      for (int j = 0; j < FN; ++j) fb0[j] = frB(smem_base + adB[j]);
      // one token block; LATE: this wave's fragment-read slots (compile-time, so that both bodies stay
      // straight-line code)
      auto token_block = [&](int it, auto late_c) {
        constexpr bool LATE = decltype(late_c)::value;
        const unsigned sb = smem_base + ((unsigned)it % NSTAGE) * STAGE;
        {
          // written out MFMA by MFMA: one fragment's reads behind each MFMA of this wave's read slots
#pragma unroll
          for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int j = 0; j < FN; ++j) {
              const int idx = i * FN + j;
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa0[i], fb0[j], acc[i][j], 0, 0, 0);
              bool is_a = false;
              const int f = frag_of(idx, LATE, is_a);
              if (f >= 0) {
                if (is_a) fa1[f] = frA(sb + adA[f] + 16 * PA);
                else fb1[f] = frB(sb + adB[f] + 16 * PB);
              }
            }
          }
        }
        // block it+1 has landed (this wave's part; the barrier makes it everyone's) and this wave's fragment
        // reads of block it are complete: its stage may be overwritten after the barrier
        __builtin_amdgcn_s_waitcnt(0x0f70 | (((AHEAD - 2) * LPT) & 15) | ((((AHEAD - 2) * LPT) >> 4) << 14));
        __builtin_amdgcn_s_barrier();
        const unsigned sn = smem_base + ((unsigned)(it + 1) % NSTAGE) * STAGE;
        // second half block: its 16 MFMAs carry the fragment reads of the next block's first half and the
        // DMA instructions of the block AHEAD ahead
        {
          v4i ra, rb;
          next_block(ld, ra, rb);
          const unsigned stage = smem_base + ((unsigned)(it + AHEAD) % NSTAGE) * STAGE;
#pragma unroll
          for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int j = 0; j < FN; ++j) {
              const int idx = i * FN + j;
              {
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa1[i], fb1[j], acc[i][j], 0, 0, 0);
            }
              bool is_a = false;
              const int f = frag_of(idx, LATE, is_a);
              if (f >= 0) {
                if (is_a) fa0[f] = frA(sn + adA[f]);
                else fb0[f] = frB(sn + adB[f]);
              }
              // the LPT DMA instructions spread evenly over the NMF MFMAs
#pragma unroll
              for (int q = idx * LPT / NMF; q < (idx + 1) * LPT / NMF; ++q) {
                if (q < LA) load_lds16(ra, stage + (unsigned)(wave_s * LA + q) * 1024, offA[q]);
                else load_lds16(rb, stage + A_BYTES + (unsigned)(wave_s * LB + (q - LA)) * 1024, offB[q - LA]);
              }
            }
          }
        }
      };
      if (late_wave) {
        for (int it = 0; it < n_tiles; ++it) token_block(it, std::true_type{});
      } else {
        for (int it = 0; it < n_tiles; ++it) token_block(it, std::false_type{});
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);

    // a 256-register tile lives in AGPRs (one wave per SIMD); smaller tiles stay in VGPRs
    [[maybe_unused]] auto rd = [](float a) {
      if constexpr (FM * FN * 16 > 128) return acc_read(a); else return a;
    };
    {
      __builtin_amdgcn_s_barrier();
      // the last MFMAs have retired before the accumulators are read by hand (acc_read is opaque to the
      // compiler's hazard tracking)
      asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
      constexpr unsigned PT = 80;
      const unsigned W = smem_base + (unsigned)wave * 8192;
      const int h = lane >> 5, nl = lane & 31;
      const int l = lane & 15, gq = lane >> 4;
      u16* outp = static_cast<u16*>(p.out) + (size_t)item * p.out_seq_stride;
#pragma unroll
      for (int i = 0; i < FM; ++i) {
#pragma unroll
        for (int jp = 0; jp < FN / 2; ++jp) {
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            const int j = jp * 2 + jj;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              v2u pk;
              pk.x = pack_bf16(rd(acc[i][j][4 * g]), rd(acc[i][j][4 * g + 1]));
              pk.y = pack_bf16(rd(acc[i][j][4 * g + 2]), rd(acc[i][j][4 * g + 3]));
              const unsigned a = W + (unsigned)(jj * 32 + nl) * PT + (unsigned)(8 * g + 4 * h) * 2;
              *(v2u __attribute__((address_space(3)))*)(a) = pk;
            }
          }
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            const int rb = s >> 1, pc = (s & 1) * 4 + gq;
            const unsigned a = W + (unsigned)(8 * pc + (l >> 2)) * PT + (unsigned)(16 * rb + 4 * (l & 3)) * 2;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(a));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(a + 4 * PT));
            const int m = m0 + wm * WM + i * 32 + 16 * rb + l;
            const int n = n0 + wn * WN + jp * 64 + 8 * pc;
            if (m < p.row_end && n < p.d_in)
              __builtin_nontemporal_store(__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7),
                                          (s16x8*)(outp + (size_t)(m - p.out_row0) * p.d_in + n));
          }
        }
      }
    }
    if constexpr (!PERSIST) break;
  }
}


template <int BM, int BN, int NSTAGE, int OCC, bool PER_SEQ, bool PERSIST = false, bool TILED = false, bool WTD = false>
__global__ __launch_bounds__(256, OCC) void seq_grad_stream_kernel(StreamParams p) {
  seq_grad_stream_body<BM, BN, NSTAGE, PER_SEQ, PERSIST, TILED, WTD, 4>(p);
}

template <int BM, int BN, int NSTAGE, int OCC, bool PER_SEQ, bool PERSIST = false, bool TILED = false, bool WTD = false>
__global__ __launch_bounds__(512, OCC) void seq_grad_stream_waves8_kernel(StreamParams p) {
  seq_grad_stream_body<BM, BN, NSTAGE, PER_SEQ, PERSIST, TILED, WTD, 8>(p);
}

// o[i] = beta * o[i] (0 for beta = 0, whatever o held), ahead of the atomic accumulation.
__global__ __launch_bounds__(256) void apply_beta_kernel(float* __restrict__ o, long long n, float beta) {
  const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i + 3 < n) {
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (beta != 0.f) v = *(f32x4*)(o + i) * beta;
    *(f32x4*)(o + i) = v;
  } else {
    for (long long k = i; k < n; ++k) o[k] = beta != 0.f ? beta * o[k] : 0.f;
  }
}

// The same for the 256x256 output tiles from `first_tile` on (tile order as in the contraction): the
// tiles whose token chunks are accumulated with atomics while the tiles before them are stored whole.
// One workgroup per 16 rows of a tile.
__global__ __launch_bounds__(256) void apply_beta_tiles_kernel(float* __restrict__ out, int d_in, int row0, int row_end,
                                                               int out_row0, int tiles_m, int tiles_n, int first_tile,
                                                               float beta) {
  int tile_m, tile_n;
  strip_tile_coords(first_tile + (int)(blockIdx.x >> 4), tiles_m, tiles_n, tile_m, tile_n);
  const int n = tile_n * 256 + (threadIdx.x & 63) * 4;
  if (n >= d_in) return;
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    const int m = row0 + tile_m * 256 + (int)(blockIdx.x & 15) * 16 + rr * 4 + (int)(threadIdx.x >> 6);
    if (m >= row_end) continue;
    f32x4* o = reinterpret_cast<f32x4*>(out + (size_t)(m - out_row0) * d_in + n);
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (beta != 0.f) v = *o * beta;
    *o = v;
  }
}

__global__ void queue_zero_kernel(unsigned* queue) {
  if (threadIdx.x < 8) queue[threadIdx.x] = 0u;
}

// n_wg > 0 (per-sequence mode, 256x256 tile): persistent launch of n_wg workgroups, a multiple of eight,
// pulling work from `queue` (eight device counters, zeroed here on the stream).
template <int BM, int BN, int NSTAGE, int OCC, bool PER_SEQ, bool PERSIST = false, bool TILED = false, bool WTD = false, int NW = 4>
hipError_t launch_stream(const SeqGradArgs& a, const ContractionPlan& pl, hipStream_t s, int n_wg = 0,
                         unsigned* queue = nullptr) {
  StreamParams p;
  p.queue = queue;
  p.c = a.c;
  p.X = static_cast<const u16*>(a.X); p.Delta = static_cast<const u16*>(a.Delta); p.off = a.off; p.out = a.out;
  p.d_in = a.d_in; p.d_out = a.d_out; p.n_seq = a.n_seq; p.n_tokens = a.n_tokens;
  p.row0 = a.row0; p.row_end = a.row0 + a.rows; p.out_row0 = a.out_row0;
  p.out_seq_stride = a.out_seq_stride; p.beta = a.beta;
  p.tiles_m = pl.tiles_m;
  p.tiles_n = pl.tiles_n;
  p.n_chunks = pl.n_chunks;
  p.chunk_tokens = pl.chunk_tokens;
  p.whole_tiles = pl.whole_tiles;
  for (int x = 0; x <= 8; ++x) p.xcd_start[x] = pl.xcd_start[x];
  if (pl.blocks <= 0) return hipSuccess;
  if (pl.blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  p.n_blocks = (unsigned)pl.blocks;
  constexpr size_t ring = (size_t)NSTAGE * BK * (BM + BN) * 2;
  constexpr size_t smem = ring > 32768 ? ring : 32768;      // the stash epilogue stages 8 KiB per wave
  static_assert(NW == 4 || NW == 8, "waves per workgroup");
  auto kern = [] {
    if constexpr (NW == 8) return &seq_grad_stream_waves8_kernel<BM, BN, NSTAGE, OCC, PER_SEQ, PERSIST, TILED, WTD>;
    else return &seq_grad_stream_kernel<BM, BN, NSTAGE, OCC, PER_SEQ, PERSIST, TILED, WTD>;
  }();
  // once per process (static initialisation is thread-safe); a failure is returned by every call
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr != hipSuccess) return attr;
  if (!PER_SEQ && p.whole_tiles > 0) {
    const int rest = p.tiles_m * p.tiles_n - p.whole_tiles;
    hipLaunchKernelGGL(apply_beta_tiles_kernel, dim3((unsigned)rest * 16), dim3(256), 0, s, static_cast<float*>(a.out),
                       a.d_in, a.row0, a.row0 + a.rows, a.out_row0, p.tiles_m, p.tiles_n, p.whole_tiles, a.beta);
  } else if (!PER_SEQ && p.n_chunks > 1) {
    // the band of output rows this launch owns is contiguous in dW
    float* band = static_cast<float*>(a.out) + (size_t)(a.row0 - a.out_row0) * a.d_in;
    const long long n = (long long)a.rows * a.d_in;
    hipLaunchKernelGGL(apply_beta_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, s, band, n, a.beta);
  }
  if constexpr (PERSIST) {
    hipLaunchKernelGGL(queue_zero_kernel, dim3(1), dim3(64), 0, s, queue);
    hipLaunchKernelGGL(kern, dim3((unsigned)n_wg), dim3(64 * NW), smem, s, p);
  } else {
    hipLaunchKernelGGL(kern, dim3(p.n_blocks), dim3(64 * NW), smem, s, p);
  }
  return hipGetLastError();
}

}  // namespace

// bf16: the per-sequence stash, the plain sum over all tokens, or (c != nullptr) the weighted sum.
hipError_t launch_seq_grad_stream(const SeqGradArgs& a, hipStream_t s) {
  const ContractionPlan pl = plan_contraction(a.rows, a.d_in, a.n_tokens, a.n_seq, a.off_host, a.per_sequence);
  // a workgroup budget applies to the large tile's per-sequence launches that would not fit it anyway
  if (a.per_sequence && a.tile_order) {
    // the caller has checked stash_tile_order_ok; anything else would scatter the stores
    if (a.rows % pl.tile || a.d_in % pl.tile || a.row0 % pl.tile || a.out_row0 % pl.tile) return hipErrorInvalidValue;
    if (a.max_workgroups > 0 && a.queue && pl.tile == 256 && pl.blocks > a.max_workgroups)
      return launch_stream<256, 256, 4, 1, true, true, true>(a, pl, s, a.max_workgroups / 8 * 8, a.queue);
    return pl.tile == 256 ? launch_stream<256, 256, 4, 1, true, false, true>(a, pl, s)
                          : launch_stream<128, 128, 4, 2, true, false, true>(a, pl, s);
  }
  if (a.per_sequence && a.max_workgroups > 0 && a.queue && pl.tile == 256 && pl.blocks > a.max_workgroups)
    return launch_stream<256, 256, 4, 1, true, true>(a, pl, s, a.max_workgroups / 8 * 8, a.queue);
  if (a.per_sequence)
    return pl.tile == 256 ? launch_stream<256, 256, 4, 1, true>(a, pl, s) : launch_stream<128, 128, 4, 2, true>(a, pl, s);
  if (a.c != nullptr)       // the weighted sum: segments of one sequence each, accumulators rescaled in between
    return pl.tile == 256 ? launch_stream<256, 256, 4, 1, false, false, false, true, 8>(a, pl, s)
                          : launch_stream<128, 128, 4, 2, false, false, false, true>(a, pl, s);
  return pl.tile == 256 ? launch_stream<256, 256, 4, 1, false, false, false, false, 8>(a, pl, s)
                        : launch_stream<128, 128, 4, 2, false>(a, pl, s);
}

// Schedule probe: the plain sum over all tokens on the 256x256 tile with four or eight waves per workgroup.
hipError_t launch_seq_grad_stream_waves(const SeqGradArgs& a, int waves, hipStream_t s) {
  if (a.per_sequence || a.c != nullptr || (waves != 4 && waves != 8)) return hipErrorInvalidValue;
  const ContractionPlan pl = plan_contraction(a.rows, a.d_in, a.n_tokens, a.n_seq, a.off_host, false);
  if (pl.tile != 256) return hipErrorInvalidValue;
  return waves == 8 ? launch_stream<256, 256, 4, 1, false, false, false, false, 8>(a, pl, s)
                    : launch_stream<256, 256, 4, 1, false>(a, pl, s);
}

}  // namespace isopo
