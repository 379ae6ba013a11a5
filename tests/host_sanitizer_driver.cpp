// Replays the host-only entry points of the library (argument validation, the Gram-path cost model,
// workspace sizes, the contraction's launch plan and the stash layout) over the benchmark's shapes and a
// set of edge cases.  Built by tests/test_host_sanitizers.py with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host code; touches no GPU.  Prints one line per case so that the test
// can compare the numbers with what the regular build of the library returns.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../include/isopo.h"

static std::vector<int32_t> offsets(const std::vector<int32_t>& lengths) {
  std::vector<int32_t> off(lengths.size() + 1, 0);
  for (size_t i = 0; i < lengths.size(); ++i) off[i + 1] = off[i] + lengths[i];
  return off;
}

static unsigned long long rng_state = 88172645463325252ULL;
static unsigned rnd(unsigned lo, unsigned hi) {            // xorshift64: fixed, portable sequence
  rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
  return lo + (unsigned)(rng_state % (hi - lo + 1));
}

static int failures = 0;
#define EXPECT(cond)                                                                         \
  do {                                                                                       \
    if (!(cond)) { std::printf("FAIL %s:%d %s\n", __FILE__, __LINE__, #cond); ++failures; } \
  } while (0)

static void replay(const char* name, const std::vector<int32_t>& lengths, int d_in, int d_out, isopo_dtype dtype) {
  const std::vector<int32_t> off = offsets(lengths);
  isopo_layer l{};
  l.dtype = dtype; l.n_tokens = off.back(); l.d_in = d_in; l.d_out = d_out; l.n_seq = (int32_t)lengths.size();
  l.seq_offsets_host = off.data();
  for (int req = 0; req < 3; ++req) {
    isopo_gram_path chosen = ISOPO_GRAM_AUTO;
    size_t full = 0, mn = 0;
    const isopo_status st = isopo_layer_gram_plan(&l, (isopo_gram_path)req, &chosen, &full, &mn);
    std::printf("%s plan req=%d status=%d chosen=%d full=%zu min=%zu\n", name, req, (int)st, (int)chosen, full, mn);
    if (st == ISOPO_OK) EXPECT(mn <= full && chosen != ISOPO_GRAM_AUTO);
  }
  double tg = 0, tm = 0;
  if (isopo_gram_cost_model(&l, &tg, &tm) == ISOPO_OK) {
    std::printf("%s cost ghost=%.6e materialised=%.6e\n", name, tg, tm);
    EXPECT(tg > 0 && tm > 0);
  }
  isopo_stash_layout layout = ISOPO_STASH_ROW_MAJOR;
  int32_t tile = -1;
  if (isopo_stash_layout_of(&l, &layout, &tile) == ISOPO_OK) std::printf("%s layout=%d tile=%d\n", name, (int)layout, tile);
  for (int per_seq = 0; per_seq < 2; ++per_seq) {
    isopo_contraction_plan_info pl{};
    const isopo_status st = isopo_contraction_plan(&l, per_seq, &pl);
    if (st != ISOPO_OK) { std::printf("%s contraction per_seq=%d status=%d\n", name, per_seq, (int)st); continue; }
    std::printf("%s contraction per_seq=%d tile=%d occ=%d tiles=%d chunks=%d chunk_tokens=%d whole=%d wgs=%lld xcd=",
                name, per_seq, pl.tile, pl.workgroups_per_cu, pl.tiles, pl.n_chunks, pl.chunk_tokens, pl.whole_tiles,
                (long long)pl.workgroups);
    for (int x = 0; x <= 8; ++x) std::printf("%d%c", pl.xcd_start[x], x < 8 ? ',' : '\n');
    // what the kernel relies on: ranges in order and inside the pair list, chunks cover the tokens
    const long long items = per_seq ? l.n_seq : pl.n_chunks;
    for (int x = 0; x < 8; ++x) EXPECT(pl.xcd_start[x] <= pl.xcd_start[x + 1]);
    EXPECT(pl.xcd_start[8] == 0 || pl.xcd_start[8] == items * (long long)pl.tiles);
    EXPECT(pl.n_chunks >= 1 && (long long)pl.n_chunks * pl.chunk_tokens >= l.n_tokens);
    EXPECT(pl.whole_tiles >= 0 && pl.whole_tiles <= pl.tiles && pl.whole_tiles % 256 == 0);
    EXPECT(pl.workgroups >= 0);
  }
  std::printf("%s scratch=%zu fisher_ws=%zu fisher_group_ws=%zu fisher_block_ws=%zu\n", name, isopo_weighted_grad_scratch(&l),
              isopo_fisher_samples_workspace(&l, 32), isopo_fisher_samples_group_workspace(&l, 3, 64),
              isopo_fisher_samples_block_workspace(&l, 7, 32));
  // the block call validates on the host before it looks at any device pointer: no device offsets -> rejected
  {
    const isopo_layer* ls[3] = {&l, &l, &l};
    const int32_t sizes[2] = {2, 1};
    const int32_t too_big[1] = {ISOPO_MAX_GROUP + 1};
    EXPECT(isopo_fisher_samples_block(ls, sizes, 2, nullptr, 8, nullptr, 0.f, ISOPO_REG_ABSOLUTE, nullptr, 0.9f, nullptr, nullptr,
                                      nullptr, 0, nullptr) != ISOPO_OK);
    EXPECT(isopo_fisher_samples_block(ls, too_big, 1, nullptr, 8, nullptr, 0.f, ISOPO_REG_ABSOLUTE, nullptr, 0.9f, nullptr,
                                      nullptr, nullptr, 0, nullptr) == ISOPO_ERR_UNSUPPORTED);
    EXPECT(isopo_fisher_samples_block(ls, sizes, ISOPO_MAX_GROUPS + 1, nullptr, 8, nullptr, 0.f, ISOPO_REG_ABSOLUTE, nullptr, 0.9f,
                                      nullptr, nullptr, nullptr, 0, nullptr) == ISOPO_ERR_UNSUPPORTED);
    EXPECT(isopo_fisher_samples_block(ls, nullptr, 1, nullptr, 8, nullptr, 0.f, ISOPO_REG_ABSOLUTE, nullptr, 0.9f, nullptr, nullptr,
                                      nullptr, 0, nullptr) == ISOPO_ERR_INVALID_ARG);
  }
}

int main() {
  // the benchmark's shapes: a 1.5B-class and a 7B-class block, the 28-layer sweep's microbatch, the stress layer
  struct Shape { const char* name; int d_in, d_out; };
  const Shape small_block[] = {{"q", 1536, 1536}, {"k", 1536, 256}, {"gate", 1536, 8960}, {"down", 8960, 1536}};
  const Shape large_block[] = {{"q", 4096, 4096}, {"k", 4096, 1024}, {"gate", 4096, 14336}, {"down", 14336, 4096}};
  char name[96];
  std::vector<int32_t> c2, c3, c4(64, 2048), c5;
  for (int i = 0; i < 16; ++i) c2.push_back((int32_t)rnd(256, 1024));
  for (int i = 0; i < 32; ++i) c3.push_back((int32_t)rnd(512, 4096));
  for (int i = 0; i < 256; ++i) c5.push_back((int32_t)(i % 17 == 0 ? 16384 : rnd(128, 3000)));
  for (const Shape& s : small_block) {
    std::snprintf(name, sizeof name, "config2/%s", s.name); replay(name, c2, s.d_in, s.d_out, ISOPO_BF16);
    std::snprintf(name, sizeof name, "config4/%s", s.name); replay(name, c4, s.d_in, s.d_out, ISOPO_BF16);
  }
  for (const Shape& s : large_block) {
    std::snprintf(name, sizeof name, "config3/%s", s.name); replay(name, c3, s.d_in, s.d_out, ISOPO_BF16);
  }
  replay("config5/gate", c5, 5120, 27648, ISOPO_BF16);              // 2160 tiles of 256 x 256
  replay("config1/lin", {32, 32, 32, 32}, 64, 128, ISOPO_F32);
  // edge cases: empty sequences, one sequence, one token, one tile, widths that are no multiple of the tile
  replay("empty_all", {0, 0, 0}, 256, 256, ISOPO_BF16);
  replay("empty_some", {0, 5, 0, 700, 0}, 1536, 256, ISOPO_BF16);
  replay("one_token", {1}, 8, 8, ISOPO_BF16);
  replay("one_tile", {4096}, 256, 256, ISOPO_BF16);
  replay("odd_widths", {70, 129, 33}, 264, 520, ISOPO_BF16);
  replay("odd_widths_f32", {70, 129, 33}, 60, 36, ISOPO_F32);
  replay("long_narrow", {100000, 31072}, 256, 384, ISOPO_BF16);
  replay("max_sequences", std::vector<int32_t>(ISOPO_MAX_SEQ, 3), 512, 768, ISOPO_BF16);
  for (int k = 0; k < 24; ++k) {                                      // seeded random ragged layers
    std::vector<int32_t> len;
    const int b = (int)rnd(1, 70);
    for (int i = 0; i < b; ++i) len.push_back(rnd(0, 9) == 0 ? 0 : (int32_t)rnd(1, 5000));
    std::snprintf(name, sizeof name, "random%d", k);
    replay(name, len, 8 * (int)rnd(1, 640), 8 * (int)rnd(1, 1200), ISOPO_BF16);
  }
  // argument validation: every rejected call returns before it reads what it was not given
  {
    const std::vector<int32_t> off = {0, 3, 7};
    isopo_layer l{};
    l.dtype = ISOPO_BF16; l.n_tokens = 7; l.d_in = 64; l.d_out = 64; l.n_seq = 2; l.seq_offsets_host = off.data();
    EXPECT(isopo_layer_gram_plan(nullptr, ISOPO_GRAM_AUTO, nullptr, nullptr, nullptr) == ISOPO_ERR_INVALID_ARG);
    EXPECT(isopo_layer_gram_plan(&l, (isopo_gram_path)9, nullptr, nullptr, nullptr) == ISOPO_ERR_INVALID_ARG);
    EXPECT(isopo_layer_gram(&l, ISOPO_GRAM_AUTO, nullptr, nullptr, 0, 0, nullptr) == ISOPO_ERR_INVALID_ARG);
    EXPECT(isopo_weighted_grad(&l, nullptr, nullptr, 0.f, nullptr, nullptr) == ISOPO_ERR_INVALID_ARG);
    EXPECT(isopo_weighted_grad_stash(&l, nullptr, nullptr, (isopo_stash_layout)7, 0.f, nullptr, nullptr) == ISOPO_ERR_INVALID_ARG);
    EXPECT(isopo_weighted_grad_stash_bf16(&l, nullptr, nullptr, ISOPO_STASH_ROW_MAJOR, 0.f, nullptr, nullptr) == ISOPO_ERR_INVALID_ARG);
    EXPECT(isopo_weighted_grad_stash_bf16(nullptr, nullptr, nullptr, ISOPO_STASH_TILE_ORDER, 0.f, nullptr, nullptr) == ISOPO_ERR_INVALID_ARG);
    EXPECT(isopo_contraction_plan(&l, 1, nullptr) == ISOPO_ERR_INVALID_ARG);
    EXPECT(isopo_probe_contraction_waves(&l, 8, nullptr, nullptr) == ISOPO_ERR_INVALID_ARG);
    EXPECT(isopo_probe_contraction_waves(nullptr, 4, nullptr, nullptr) == ISOPO_ERR_INVALID_ARG);
    EXPECT(isopo_probe_lds_dma(nullptr, 8 * 32768, 4, 2, 8, 1, nullptr, nullptr) == ISOPO_ERR_INVALID_ARG);
    const std::vector<int32_t> bad1 = {1, 3, 7}, bad2 = {0, 5, 3}, bad3 = {0, 3, 6};
    for (const auto* b : {&bad1, &bad2, &bad3}) {
      l.seq_offsets_host = b->data();
      EXPECT(isopo_layer_gram_plan(&l, ISOPO_GRAM_AUTO, nullptr, nullptr, nullptr) == ISOPO_ERR_BAD_OFFSETS);
    }
    l.seq_offsets_host = off.data();
    l.d_in = 60;
    EXPECT(isopo_layer_gram_plan(&l, ISOPO_GRAM_AUTO, nullptr, nullptr, nullptr) == ISOPO_ERR_UNSUPPORTED);
    l.d_in = 64; l.n_seq = ISOPO_MAX_SEQ + 1;
    EXPECT(isopo_layer_gram_plan(&l, ISOPO_GRAM_AUTO, nullptr, nullptr, nullptr) == ISOPO_ERR_UNSUPPORTED);
    EXPECT(isopo_transform(nullptr, nullptr, 4, 1, ISOPO_VARIANT_FISHER, 0.f, ISOPO_REG_ABSOLUTE, nullptr, nullptr,
                           nullptr, 0, nullptr) == ISOPO_ERR_INVALID_ARG);
    EXPECT(isopo_transform_workspace(128, 1) == 0 && isopo_transform_workspace(256, 3) == 3u * (256 * 256 + 256) * 8);
    EXPECT(isopo_stash_gram_workspace(0) == 0 && isopo_stash_gram_workspace(256) > 0);
    EXPECT(isopo_ntk_eigh_workspace(0, 1) == 0 && isopo_ntk_eigh_workspace(300, 2) > 0);
    for (int s = 0; s <= 6; ++s) EXPECT(isopo_status_string((isopo_status)s) != nullptr);
  }
  std::printf("done failures=%d\n", failures);
  return failures ? 1 : 0;
}
