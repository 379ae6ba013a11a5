// Host-side launch plan of the streaming bf16 contraction (per-sequence gradients G_i = Delta_i^T X_i of
// both hook listings, and the unweighted dW = Delta^T X): tile size, token split, and the ranges of
// (item, tile) pairs each of the eight XCDs walks.  Pure host arithmetic, no HIP calls, so that it can be
// tested without a GPU.
#include "kernels.h"

namespace isopo {

ContractionPlan plan_contraction(int rows, int d_in, int n_tokens, int n_seq, const int32_t* off_host,
                                 bool per_sequence) {
  ContractionPlan pl;
  constexpr int kBlockTokens = 32;
  const long long big_tiles = (long long)((rows + 255) / 256) * ((d_in + 255) / 256);
  // 256x256 tiles (one workgroup per CU) when they alone fill the chip, else 128x128 (two per CU).  In the
  // sum-over-all-tokens mode the token split supplies parallelism too.
  const long long par = per_sequence ? n_seq : (n_tokens / 1024 > 1 ? n_tokens / 1024 : 1);
  const bool big = rows >= 256 && d_in >= 256 && big_tiles * par >= 256;
  pl.tile = big ? 256 : 128;
  pl.occupancy = big ? 1 : 2;
  pl.tiles_m = (rows + pl.tile - 1) / pl.tile;
  pl.tiles_n = (d_in + pl.tile - 1) / pl.tile;
  const long long tiles = (long long)pl.tiles_m * pl.tiles_n;
  pl.n_chunks = 1;
  pl.chunk_tokens = n_tokens;
  pl.whole_tiles = 0;
  for (int x = 0; x <= 8; ++x) pl.xcd_start[x] = 0;
  if (!per_sequence && big && tiles > 256 && tiles % 256 != 0 && tiles <= 0x3fffffffLL) {
    // More tiles than compute units, and the last round of one tile per compute unit would be partly idle:
    // the tiles of the full rounds stay whole (direct stores), the `rest` tiles of the last round are cut
    // into w token chunks that fill it (fp32 atomics on those tiles only).  Modelled time of the last round
    //   ceil(N / w) * t_token  +  (w > 1) * w * rest * tile outputs * t_atomic,
    // t_token a workgroup's time per token row, t_atomic the chip's time per fp32 atomic add; the split has
    // to win 5 %.  Workgroups are dispatched in id order, whole tiles first, so a compute unit takes a chunk
    // when it has finished its whole tiles.
    const long long rest = tiles % 256;
    const double t_token = 2.0e-8, t_atomic = 5.0e-12;
    long long most = 256 / rest;
    if (most > n_tokens / 512) most = n_tokens / 512;
    if (most > 64) most = 64;
    long long want = 1;
    double best = 0.95 * (double)n_tokens * t_token;
    for (long long w = 2; w <= most; ++w) {
      const double t = (double)((n_tokens + w - 1) / w) * t_token + (double)w * rest * 65536.0 * t_atomic;
      if (t < best) { best = t; want = w; }
    }
    if (want > 1) {
      pl.whole_tiles = (int)(tiles - rest);
      pl.chunk_tokens = (int)(((n_tokens + want - 1) / want + kBlockTokens - 1) / kBlockTokens * kBlockTokens);
      pl.n_chunks = (n_tokens + pl.chunk_tokens - 1) / pl.chunk_tokens;
      pl.blocks = 8LL * (pl.whole_tiles / 8 + (rest * pl.n_chunks + 7) / 8);
      return pl;
    }
  }
  if (!per_sequence) {
    // Number of token chunks: the count with the smallest modelled time
    //   rounds(w) * ceil(N / w) * t_token  +  (w > 1) * w * outputs * t_atomic,
    // rounds(w) = passes an XCD's 32 CUs make over its eighth of the tiles * w workgroups.  t_token is a
    // workgroup's time per token row, t_atomic the chip's time per fp32 atomic add (about 0.8 TB/s), both
    // measured; without the second term more chunks always look better, and the adds then cost more than
    // the idle CUs did.
    const long long slots = 32LL * pl.occupancy;                     // per XCD
    const double t_token = 2.0e-8 * (double)(pl.tile * pl.tile) / 65536.0 * pl.occupancy, t_atomic = 5.0e-12;
    const double outputs = (double)rows * d_in;
    const long long most = n_tokens / 512 > 1 ? n_tokens / 512 : 1;
    long long want = 1;
    double best = 0.0;
    for (long long w = 1; w <= most && w <= 64; ++w) {
      const long long rounds = ((tiles * w + 7) / 8 + slots - 1) / slots;
      const double t = (double)rounds * (double)((n_tokens + w - 1) / w) * t_token + (w > 1 ? w * outputs * t_atomic : 0.0);
      if (w == 1) best = 0.9 * t;                                    // a split has to win by a margin
      else if (t < best) { best = t; want = w; }
    }
    if (want > 1) {
      pl.chunk_tokens = (int)(((n_tokens + want - 1) / want + kBlockTokens - 1) / kBlockTokens * kBlockTokens);
      pl.n_chunks = (n_tokens + pl.chunk_tokens - 1) / pl.chunk_tokens;
    }
  }
  const bool mapped = per_sequence || pl.n_chunks > 1;
  const int n_items = per_sequence ? n_seq : pl.n_chunks;
  pl.blocks = mapped ? 8LL * n_items * ((tiles + 7) / 8) : tiles;
  // Per-sequence mode with a tile count that is a multiple of eight: XCD x takes the x-th eighth of the
  // tiles of every sequence (xcd_start stays zero).  Otherwise the item-major list of (item, tile) pairs is
  // cut into eight contiguous ranges of equal work.
  if (mapped && (!per_sequence || tiles % 8 != 0) && tiles * n_items <= 0x7fffffffLL) {
    // Work of item i: its tokens plus a fixed charge for the workgroup's prologue and epilogue.
    const long long fixed = per_sequence ? 192 : 64;
    auto weight = [&](int i) -> long long {
      if (per_sequence) return (off_host ? (long long)(off_host[i + 1] - off_host[i]) : 1024) + fixed;
      const long long t0 = (long long)i * pl.chunk_tokens;
      const long long t1 = t0 + pl.chunk_tokens < n_tokens ? t0 + pl.chunk_tokens : n_tokens;
      return (t1 - t0) + fixed;
    };
    long long total = 0;
    for (int i = 0; i < n_items; ++i) total += weight(i) * tiles;
    // pair (i, t) starts at work cum_i + t*w_i; XCD x's range opens at the first pair starting at or
    // beyond x/8 of the total
    long long cum = 0;
    int i = 0, most = 0;
    for (int x = 1; x < 8; ++x) {
      const long long target = (x * total + 7) / 8;
      while (i < n_items && cum + tiles * weight(i) <= target) cum += tiles * weight(i++);
      if (i == n_items) { pl.xcd_start[x] = (int)(tiles * n_items); continue; }
      const long long w = weight(i);
      pl.xcd_start[x] = (int)(i * tiles + (target - cum + w - 1) / w);
    }
    pl.xcd_start[8] = (int)(tiles * n_items);
    for (int k = 0; k < 8; ++k) most = pl.xcd_start[k + 1] - pl.xcd_start[k] > most ? pl.xcd_start[k + 1] - pl.xcd_start[k] : most;
    pl.blocks = 8LL * most;
  }
  return pl;
}

int stash_tile_order_ok(int d_out, int d_in, int n_tokens, int n_seq, const int32_t* off_host) {
  // multiples of the larger tile, so that a band of output rows may pick either tile size
  if (d_out % 256 || d_in % 256) return 0;
  return plan_contraction(d_out, d_in, n_tokens, n_seq, off_host, true).tile;
}

}  // namespace isopo
