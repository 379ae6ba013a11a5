// C ABI of the ISOPO layer-step library: argument checks, the Gram-path cost
// model, workspace layout and kernel sequencing.  No arithmetic of the method
// lives here; every step runs in the kernels.
#include "../../include/isopo.h"

#include <cstring>

#include <cmath>
#include <mutex>
#include "kernels.h"

// Scratch of isopo_transform_noalloc: the fp64 work matrices and right-hand sides that isopo_transform takes
// from its workspace argument when n_seq > 128.  One copy per GPU, at its own address on each, resident
// until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the device
// address it resolves to (static_scratch below) is what kernels and copies get.
constexpr size_t kStaticScratchBytes = ISOPO_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

using namespace isopo;

constexpr size_t kAlign = 256;
constexpr int kTileRows = 256;        // output rows per tile of the contraction kernel
// the stash Gram kernels cover any bf16 batch; fp32 stashes up to 128 sequences
bool materialised_ok(int n_seq, isopo_dtype t) { return n_seq <= 128 || t == ISOPO_BF16; }

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
constexpr int kComputeUnits = 256;        // MI355X
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
size_t elem_size(isopo_dtype t) { return t == ISOPO_BF16 ? 2 : 4; }

// An enum argument arrives through a C ABI and may hold any int.  Its bytes are read as an int before
// anything touches it as the enum type (for which a value outside the enumerators' range is undefined).
template <class E>
bool enum_in(const E& e, int lo, int hi) {
  static_assert(sizeof(E) == sizeof(int), "C enums of this header are ints");
  int v;
  std::memcpy(&v, &e, sizeof v);
  return v >= lo && v <= hi;
}

isopo_status check_layer(const isopo_layer* l, bool need_dev) {
  if (!l) return ISOPO_ERR_INVALID_ARG;
  if (!enum_in(l->dtype, ISOPO_F32, ISOPO_BF16)) return ISOPO_ERR_UNSUPPORTED;
  if (l->d_in <= 0 || l->d_out <= 0 || l->n_seq <= 0 || l->n_tokens < 0) return ISOPO_ERR_INVALID_ARG;
  if (l->n_tokens >= (int64_t)1 << 31) return ISOPO_ERR_UNSUPPORTED;
  if (l->n_seq > ISOPO_MAX_SEQ) return ISOPO_ERR_UNSUPPORTED;
  const int vec = l->dtype == ISOPO_BF16 ? 8 : 4;
  if (l->d_in % vec || l->d_out % vec) return ISOPO_ERR_UNSUPPORTED;
  if (!l->seq_offsets_host) return ISOPO_ERR_INVALID_ARG;
  const int32_t* off = l->seq_offsets_host;
  if (off[0] != 0 || off[l->n_seq] != l->n_tokens) return ISOPO_ERR_BAD_OFFSETS;
  for (int i = 0; i < l->n_seq; ++i)
    if (off[i + 1] < off[i]) return ISOPO_ERR_BAD_OFFSETS;
  if (need_dev) {
    if (!l->seq_offsets_dev) return ISOPO_ERR_INVALID_ARG;
    if (l->n_tokens > 0 && (!l->X || !l->Delta)) return ISOPO_ERR_INVALID_ARG;
    if (!aligned16(l->X) || !aligned16(l->Delta)) return ISOPO_ERR_INVALID_ARG;
  }
  return ISOPO_OK;
}

// Rates of this library's own kernels, measured on one MI355X, used only to rank the two Gram paths.
// Materialised: the tiled MFMA contraction writes the stash while it computes (whichever of the two takes
// longer bounds that launch), then the Gram pass reads the stash once.  Ghost: two token-by-token Gram
// matrices over d_in + d_out features; a workgroup walks the features of its 128x128 token-tile pair
// serially (all of them, or one range of them when there are fewer tile pairs than compute units), which
// sets a floor however few tokens there are.
constexpr double kRateContraction = 1.0e15;   // flop/s, per-sequence gradient kernel
constexpr double kRateGhost = 7.0e14;         // token-pair-features/s, ghost kernel
constexpr double kRateStash = 3.7e12;         // B/s, stash write / read
constexpr double kLaunch = 6.0e-6;            // s per kernel launch in the chain

void cost_model(const isopo_layer* l, double* t_ghost, double* t_mat) {
  const double di = l->d_in, d_o = l->d_out, b = l->n_seq;
  const double D = di * d_o;
  // ghost: the kernel works on 128-token tiles, so a short batch still pays whole tiles
  const double nt = (double)((l->n_tokens + 127) / 128) * 128.0;
  // few tile pairs: the bf16 kernel cuts the features into ranges (a shorter walk) and a second kernel sums
  // the ranges' parts
  const long long tiles = (l->n_tokens + 127) / 128, tile_pairs = tiles * (tiles + 1) / 2;
  const int split = l->dtype == ISOPO_BF16 ? ghost_feature_split((int)l->n_tokens, l->d_in, l->d_out) : 1;
  const double walk = ghost_walk_time(tile_pairs, l->d_in, l->d_out, split);
  const double pairs = nt * nt * (di + d_o) / kRateGhost;
  // five short launches back to back (fill, token map, products, parts, finish) cost about three isolated ones
  *t_ghost = (walk > pairs ? walk : pairs) + 3 * kLaunch;
  // materialised: every tile is padded to whole 32-token blocks per sequence
  double n_pad = 0;
  for (int i = 0; i < l->n_seq; ++i) {
    const int len = l->seq_offsets_host[i + 1] - l->seq_offsets_host[i];
    n_pad += (double)((len + 31) / 32) * 32.0;
  }
  const double pass = b * D * (double)elem_size(l->dtype) / kRateStash;      // one pass over the stash
  const double contract = 2.0 * n_pad * D / kRateContraction;
  *t_mat = (contract > pass ? contract : pass) + pass + 3 * kLaunch;
}

size_t stash_bytes(const isopo_layer* l, int rows) {
  return (size_t)l->n_seq * (size_t)rows * (size_t)l->d_in * elem_size(l->dtype);
}

// Gram partial sums, then one aligned block holding the contraction's eight work counters.
size_t gram_partial_bytes(const isopo_layer* l) {
  return align_up(stash_gram_partial_bytes(l->n_seq, l->dtype == ISOPO_BF16));
}
size_t partial_bytes(const isopo_layer* l) { return gram_partial_bytes(l) + kAlign; }

size_t ghost_bytes(const isopo_layer* l) {
  const size_t parts = l->dtype == ISOPO_BF16 ? ghost_parts_bytes((int)l->n_tokens, l->d_in, l->d_out) : 0;
  return align_up((size_t)l->n_seq * l->n_seq * sizeof(double)) + align_up((size_t)l->n_tokens * sizeof(int32_t)) +
         align_up(parts);
}

isopo_gram_path resolve(const isopo_layer* l, isopo_gram_path req) {
  if (req != ISOPO_GRAM_AUTO) return req;
  if (!materialised_ok(l->n_seq, l->dtype)) return ISOPO_GRAM_GHOST;
  double tg, tm;
  cost_model(l, &tg, &tm);
  return tg < tm ? ISOPO_GRAM_GHOST : ISOPO_GRAM_MATERIALISED;
}

// Device address of `scratch` on the current device, resolved once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

hipError_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" {

const char* isopo_version(void) { return "0.1"; }

const char* isopo_status_string(isopo_status s) {
  switch (s) {
    case ISOPO_OK: return "ok";
    case ISOPO_ERR_INVALID_ARG: return "invalid argument";
    case ISOPO_ERR_BAD_OFFSETS: return "bad sequence offsets";
    case ISOPO_ERR_UNSUPPORTED: return "unsupported dtype or shape";
    case ISOPO_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case ISOPO_ERR_HIP: return "HIP error";
    case ISOPO_ERR_SCRATCH_LIMIT: return "problem exceeds the library's static scratch";
  }
  return "unknown status";
}

isopo_status isopo_gram_cost_model(const isopo_layer* layer, double* t_ghost, double* t_materialised) {
  isopo_status st = check_layer(layer, false);
  if (st != ISOPO_OK) return st;
  double tg, tm;
  cost_model(layer, &tg, &tm);
  if (t_ghost) *t_ghost = tg;
  if (t_materialised) *t_materialised = tm;
  return ISOPO_OK;
}

isopo_status isopo_contraction_plan(const isopo_layer* layer, int per_sequence, isopo_contraction_plan_info* plan) {
  isopo_status st = check_layer(layer, false);
  if (st != ISOPO_OK) return st;
  if (!plan) return ISOPO_ERR_INVALID_ARG;
  if (layer->dtype != ISOPO_BF16) return ISOPO_ERR_UNSUPPORTED;
  const ContractionPlan pl = plan_contraction(layer->d_out, layer->d_in, (int)layer->n_tokens, layer->n_seq,
                                              layer->seq_offsets_host, per_sequence != 0);
  plan->tile = pl.tile;
  plan->workgroups_per_cu = pl.occupancy;
  plan->tiles = pl.tiles_m * pl.tiles_n;
  plan->n_chunks = pl.n_chunks;
  plan->chunk_tokens = pl.chunk_tokens;
  plan->whole_tiles = pl.whole_tiles;
  for (int x = 0; x <= 8; ++x) plan->xcd_start[x] = pl.xcd_start[x];
  plan->workgroups = pl.blocks;
  return ISOPO_OK;
}

isopo_status isopo_layer_gram_plan(const isopo_layer* layer, isopo_gram_path requested, isopo_gram_path* chosen,
                                   size_t* ws_full, size_t* ws_min) {
  isopo_status st = check_layer(layer, false);
  if (st != ISOPO_OK) return st;
  if (!enum_in(requested, ISOPO_GRAM_AUTO, ISOPO_GRAM_MATERIALISED)) return ISOPO_ERR_INVALID_ARG;
  const isopo_gram_path path = resolve(layer, requested);
  if (path == ISOPO_GRAM_MATERIALISED && !materialised_ok(layer->n_seq, layer->dtype)) return ISOPO_ERR_UNSUPPORTED;
  if (chosen) *chosen = path;
  if (path == ISOPO_GRAM_GHOST) {
    if (ws_full) *ws_full = ghost_bytes(layer);
    if (ws_min) *ws_min = ghost_bytes(layer);
  } else {
    const int min_rows = layer->d_out < kTileRows ? layer->d_out : kTileRows;
    if (ws_full) *ws_full = align_up(stash_bytes(layer, layer->d_out)) + partial_bytes(layer);
    if (ws_min) *ws_min = align_up(stash_bytes(layer, min_rows)) + partial_bytes(layer);
  }
  return ISOPO_OK;
}

isopo_status isopo_layer_gram(const isopo_layer* layer, isopo_gram_path path, float* K, void* workspace,
                              size_t ws_bytes, int keep_stash, void* stream) {
  isopo_status st = check_layer(layer, true);
  if (st != ISOPO_OK) return st;
  if (!K || !workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1))) return ISOPO_ERR_INVALID_ARG;
  if (!enum_in(path, ISOPO_GRAM_AUTO, ISOPO_GRAM_MATERIALISED)) return ISOPO_ERR_INVALID_ARG;
  isopo_gram_path chosen;
  size_t ws_full, ws_min;
  st = isopo_layer_gram_plan(layer, path, &chosen, &ws_full, &ws_min);
  if (st != ISOPO_OK) return st;
  if (ws_bytes < ws_min) return ISOPO_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool bf16 = layer->dtype == ISOPO_BF16;
  char* ws = static_cast<char*>(workspace);

  if (chosen == ISOPO_GRAM_GHOST) {
    if (keep_stash) return ISOPO_ERR_INVALID_ARG;
    GhostArgs g;
    g.X = layer->X; g.Delta = layer->Delta; g.off = layer->seq_offsets_dev;
    g.n_tokens = (int)layer->n_tokens; g.d_in = layer->d_in; g.d_out = layer->d_out; g.n_seq = layer->n_seq;
    g.bf16 = bf16;
    g.K64 = reinterpret_cast<double*>(ws);
    g.tok_seq = reinterpret_cast<int32_t*>(ws + align_up((size_t)layer->n_seq * layer->n_seq * sizeof(double)));
    g.parts = reinterpret_cast<float*>(reinterpret_cast<char*>(g.tok_seq) +
                                       align_up((size_t)layer->n_tokens * sizeof(int32_t)));
    g.K = K;
    return launch_ghost_gram(g, s) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
  }

  if (keep_stash < 0 || keep_stash > 2) return ISOPO_ERR_INVALID_ARG;
  if (keep_stash && ws_bytes < ws_full) return ISOPO_ERR_WORKSPACE_TOO_SMALL;
  // Tile order whenever nobody asked for the row-major stash (a stash that is not kept is nobody's business).
  const bool tile_order = keep_stash != 1 && bf16 &&
                          stash_tile_order_ok(layer->d_out, layer->d_in, (int)layer->n_tokens, layer->n_seq,
                                              layer->seq_offsets_host) != 0;
  const size_t pbytes = partial_bytes(layer);
  const size_t row_bytes = stash_bytes(layer, 1);
  // rows of d_out whose gradients are formed and reduced per pass
  size_t rows_fit = (ws_bytes - pbytes) / row_bytes;
  const bool whole = rows_fit >= (size_t)layer->d_out;
  if (whole) rows_fit = layer->d_out;
  size_t chunk_rows = rows_fit;
  if (chunk_rows < (size_t)layer->d_out) {
    chunk_rows = chunk_rows / kTileRows * kTileRows;
    if (chunk_rows < (size_t)kTileRows) chunk_rows = kTileRows;
    if (chunk_rows > rows_fit) return ISOPO_ERR_WORKSPACE_TOO_SMALL;
  }
  // With the whole stash resident, chunk c lives at its final place (rows r0.. of
  // every sequence); otherwise every chunk reuses the front of the workspace.
  const long long seq_stride = whole ? (long long)layer->d_out * layer->d_in : (long long)chunk_rows * layer->d_in;
  float* partials = reinterpret_cast<float*>(ws + (whole ? align_up(stash_bytes(layer, layer->d_out))
                                                         : align_up(stash_bytes(layer, (int)chunk_rows))));
  if (reinterpret_cast<char*>(partials) + pbytes > ws + ws_bytes) return ISOPO_ERR_WORKSPACE_TOO_SMALL;

  for (int r0 = 0; r0 < layer->d_out; r0 += (int)chunk_rows) {
    const int rows = (layer->d_out - r0) < (int)chunk_rows ? (layer->d_out - r0) : (int)chunk_rows;
    SeqGradArgs a;
    a.X = layer->X; a.Delta = layer->Delta; a.off = layer->seq_offsets_dev; a.off_host = layer->seq_offsets_host; a.c = nullptr;
    a.out = ws; a.d_in = layer->d_in; a.d_out = layer->d_out; a.n_seq = layer->n_seq; a.n_tokens = (int)layer->n_tokens;
    a.row0 = r0; a.rows = rows; a.out_row0 = whole ? 0 : r0; a.out_seq_stride = seq_stride;
    a.beta = 0.f; a.per_sequence = true; a.bf16 = bf16; a.tile_order = tile_order;
    // one persistent workgroup per compute unit, fed from counters behind the Gram partials
    a.max_workgroups = kComputeUnits;
    a.queue = reinterpret_cast<unsigned*>(reinterpret_cast<char*>(partials) + gram_partial_bytes(layer));
    if (launch_seq_grad(a, s) != hipSuccess) return ISOPO_ERR_HIP;
    StashGramArgs g;
    g.stash = ws; g.seq_stride = seq_stride;
    g.p0 = whole ? (long long)r0 * layer->d_in : 0;
    g.p1 = g.p0 + (long long)rows * layer->d_in;
    g.n_seq = layer->n_seq; g.bf16 = bf16; g.first = (r0 == 0); g.partials = partials;
    if (launch_stash_gram(g, s) != hipSuccess) return ISOPO_ERR_HIP;
  }
  return launch_stash_gram_finish(partials, bf16, layer->n_seq, K, s) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

isopo_status isopo_seq_grads(const isopo_layer* layer, void* stash, void* stream) {
  return isopo_seq_grads_limited(layer, stash, 0, nullptr, stream);
}

isopo_status isopo_seq_grads_limited(const isopo_layer* layer, void* stash, int32_t max_workgroups,
                                     uint32_t* queue_dev, void* stream) {
  return isopo_seq_grads_stash(layer, stash, ISOPO_STASH_ROW_MAJOR, max_workgroups, queue_dev, stream);
}

isopo_status isopo_seq_grads_stash(const isopo_layer* layer, void* stash, isopo_stash_layout layout,
                                   int32_t max_workgroups, uint32_t* queue_dev, void* stream) {
  isopo_status st = check_layer(layer, true);
  if (st != ISOPO_OK) return st;
  if (!enum_in(layout, ISOPO_STASH_ROW_MAJOR, ISOPO_STASH_TILE_ORDER)) return ISOPO_ERR_INVALID_ARG;
  if (layout == ISOPO_STASH_TILE_ORDER) {
    isopo_stash_layout have;
    st = isopo_stash_layout_of(layer, &have, nullptr);
    if (st != ISOPO_OK) return st;
    if (have != ISOPO_STASH_TILE_ORDER) return ISOPO_ERR_UNSUPPORTED;
  }
  if (!stash || !aligned16(stash)) return ISOPO_ERR_INVALID_ARG;
  if (max_workgroups != 0 && (max_workgroups < 8 || max_workgroups > 256 || !queue_dev ||
                              (reinterpret_cast<uintptr_t>(queue_dev) & 3u)))
    return ISOPO_ERR_INVALID_ARG;
  SeqGradArgs a;
  a.max_workgroups = max_workgroups; a.queue = queue_dev;
  a.X = layer->X; a.Delta = layer->Delta; a.off = layer->seq_offsets_dev; a.off_host = layer->seq_offsets_host; a.c = nullptr;
  a.out = stash; a.d_in = layer->d_in; a.d_out = layer->d_out; a.n_seq = layer->n_seq; a.n_tokens = (int)layer->n_tokens;
  a.row0 = 0; a.rows = layer->d_out; a.out_row0 = 0;
  a.out_seq_stride = (long long)layer->d_out * layer->d_in;
  a.beta = 0.f; a.per_sequence = true; a.bf16 = layer->dtype == ISOPO_BF16;
  a.tile_order = layout == ISOPO_STASH_TILE_ORDER;
  return launch_seq_grad(a, static_cast<hipStream_t>(stream)) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

size_t isopo_stash_gram_workspace(int32_t n_seq) {
  if (n_seq <= 0) return 0;
  return align_up(stash_gram_partial_bytes(n_seq, true));
}

isopo_status isopo_stash_gram(const void* stash, isopo_dtype dtype, int32_t n_seq, int64_t n_elem, float* K,
                              void* workspace, size_t ws_bytes, void* stream) {
  if (!stash || !K || !workspace || n_seq <= 0 || n_elem <= 0 || !aligned16(stash)) return ISOPO_ERR_INVALID_ARG;
  if (!enum_in(dtype, ISOPO_F32, ISOPO_BF16)) return ISOPO_ERR_UNSUPPORTED;
  if (!materialised_ok(n_seq, dtype) || n_seq > ISOPO_MAX_SEQ || n_elem % (dtype == ISOPO_BF16 ? 8 : 4))
    return ISOPO_ERR_UNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) return ISOPO_ERR_INVALID_ARG;
  if (ws_bytes < isopo_stash_gram_workspace(n_seq)) return ISOPO_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  StashGramArgs g;
  g.stash = stash; g.seq_stride = n_elem; g.p0 = 0; g.p1 = n_elem; g.n_seq = n_seq;
  g.bf16 = dtype == ISOPO_BF16; g.first = true; g.partials = static_cast<float*>(workspace);
  if (launch_stash_gram(g, s) != hipSuccess) return ISOPO_ERR_HIP;
  return launch_stash_gram_finish(g.partials, g.bf16, n_seq, K, s) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

size_t isopo_transform_workspace(int32_t n_seq, int32_t batch) {
  if (n_seq <= kTransformLdsMax || batch <= 0) return 0;
  return (size_t)batch * ((size_t)n_seq * n_seq + n_seq) * sizeof(double);
}

isopo_status isopo_transform(const float* K, const float* A, int32_t n_seq, int32_t batch, isopo_variant variant,
                             float lambda, isopo_reg_mode reg_mode, float* c, int32_t* info_dev, void* workspace,
                             size_t ws_bytes, void* stream) {
  if (!K || !A || !c || n_seq <= 0 || batch <= 0) return ISOPO_ERR_INVALID_ARG;
  if (n_seq > ISOPO_MAX_SEQ) return ISOPO_ERR_UNSUPPORTED;
  if (!enum_in(variant, ISOPO_VARIANT_FISHER, ISOPO_VARIANT_INTERACTING)) return ISOPO_ERR_INVALID_ARG;
  if (!enum_in(reg_mode, ISOPO_REG_ABSOLUTE, ISOPO_REG_REL_TRACE)) return ISOPO_ERR_INVALID_ARG;
  if (!(lambda >= 0.f)) return ISOPO_ERR_INVALID_ARG;
  if (variant == ISOPO_VARIANT_INTERACTING) {
    const size_t need = isopo_transform_workspace(n_seq, batch);
    if (need && (!workspace || ws_bytes < need)) return ISOPO_ERR_WORKSPACE_TOO_SMALL;
    if (need && (reinterpret_cast<uintptr_t>(workspace) & 15u)) return ISOPO_ERR_INVALID_ARG;
  }
  TransformArgs t;
  t.K = K; t.A = A; t.n_seq = n_seq; t.batch = batch; t.variant = (int)variant; t.reg_mode = (int)reg_mode;
  t.lambda = lambda; t.c = c; t.info = info_dev; t.workspace = static_cast<double*>(workspace);
  return launch_transform(t, static_cast<hipStream_t>(stream)) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

isopo_status isopo_transform_noalloc(const float* K, const float* A, int32_t n_seq, int32_t batch,
                                     isopo_variant variant, float lambda, isopo_reg_mode reg_mode, float* c,
                                     int32_t* info_dev, void* stream) {
  if (!K || !A || !c || n_seq <= 0 || batch <= 0) return ISOPO_ERR_INVALID_ARG;
  if (n_seq > ISOPO_MAX_SEQ) return ISOPO_ERR_UNSUPPORTED;
  if (!enum_in(variant, ISOPO_VARIANT_FISHER, ISOPO_VARIANT_INTERACTING)) return ISOPO_ERR_INVALID_ARG;
  const size_t need = variant == ISOPO_VARIANT_INTERACTING ? isopo_transform_workspace(n_seq, batch) : 0;
  if (need > kStaticScratchBytes) return ISOPO_ERR_SCRATCH_LIMIT;
  void* ptr = nullptr;
  if (need && static_scratch(&ptr) != hipSuccess) return ISOPO_ERR_HIP;
  // Nothing in the scratch has to start at zero: the kernel writes the lower triangle of K + reg I and the
  // right-hand side before it reads them, and reads nothing else.
  return isopo_transform(K, A, n_seq, batch, variant, lambda, reg_mode, c, info_dev, ptr, need, stream);
}

isopo_status isopo_transform_ema(const float* K, const float* A, int32_t n_seq, int32_t batch, isopo_variant variant,
                                 float factor, float* ema_state, float ema_decay, float* c, int32_t* info_dev,
                                 void* workspace, size_t ws_bytes, void* stream) {
  if (!K || !A || !c || !ema_state || n_seq <= 0 || batch <= 0) return ISOPO_ERR_INVALID_ARG;
  if (n_seq > ISOPO_MAX_SEQ) return ISOPO_ERR_UNSUPPORTED;
  if (!enum_in(variant, ISOPO_VARIANT_FISHER, ISOPO_VARIANT_INTERACTING)) return ISOPO_ERR_INVALID_ARG;
  if (!(factor >= 0.f) || !(ema_decay >= 0.f && ema_decay < 1.f)) return ISOPO_ERR_INVALID_ARG;
  if (variant == ISOPO_VARIANT_INTERACTING) {
    const size_t need = isopo_transform_workspace(n_seq, batch);
    if (need && (!workspace || ws_bytes < need)) return ISOPO_ERR_WORKSPACE_TOO_SMALL;
    if (need && (reinterpret_cast<uintptr_t>(workspace) & 15u)) return ISOPO_ERR_INVALID_ARG;
  }
  TransformArgs t;
  t.K = K; t.A = A; t.n_seq = n_seq; t.batch = batch; t.variant = (int)variant; t.reg_mode = (int)ISOPO_REG_EMA_TRACE;
  t.lambda = factor; t.c = c; t.info = info_dev; t.workspace = static_cast<double*>(workspace);
  t.ema_state = ema_state; t.ema_decay = ema_decay;
  return launch_transform(t, static_cast<hipStream_t>(stream)) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

static_assert(kFisherMaxGroup == ISOPO_MAX_GROUP, "group size of the kernel and of the header");
static_assert(kFisherMaxGroups == ISOPO_MAX_GROUPS, "number of groups of the kernel and of the header");

size_t isopo_fisher_samples_group_workspace(const isopo_layer* layer, int32_t n_layers, int32_t n_samples) {
  if (!layer || n_samples < 1 || n_samples > ISOPO_MAX_SAMPLES || layer->n_seq <= 0 || layer->n_tokens < 0 ||
      n_layers < 1 || n_layers > ISOPO_MAX_GROUP)
    return 0;
  return fisher_samples_workspace((int)layer->n_tokens, layer->n_seq, n_samples, n_layers);
}

size_t isopo_fisher_samples_workspace(const isopo_layer* layer, int32_t n_samples) {
  return isopo_fisher_samples_group_workspace(layer, 1, n_samples);
}

size_t isopo_fisher_samples_block_workspace(const isopo_layer* layer, int32_t n_layers_total, int32_t n_samples) {
  if (!layer || n_samples < 1 || n_samples > ISOPO_MAX_SAMPLES || layer->n_seq <= 0 || layer->n_tokens < 0 ||
      n_layers_total < 1 || n_layers_total > ISOPO_MAX_GROUP * ISOPO_MAX_GROUPS)
    return 0;
  return fisher_samples_workspace((int)layer->n_tokens, layer->n_seq, n_samples, n_layers_total);
}

isopo_status isopo_fisher_samples_block(const isopo_layer* const* layers, const int32_t* group_sizes, int32_t n_groups,
                                        const int32_t* sample_idx_dev, int32_t n_samples, const float* A, float lambda,
                                        isopo_reg_mode reg_mode, float* ema_state, float ema_decay, float* c,
                                        float* fisher_sq, void* workspace, size_t ws_bytes, void* stream) {
  if (!layers || !group_sizes || n_groups < 1) return ISOPO_ERR_INVALID_ARG;
  if (n_groups > ISOPO_MAX_GROUPS) return ISOPO_ERR_UNSUPPORTED;
  int total = 0;
  for (int g = 0; g < n_groups; ++g) {
    if (group_sizes[g] < 1) return ISOPO_ERR_INVALID_ARG;
    if (group_sizes[g] > ISOPO_MAX_GROUP) return ISOPO_ERR_UNSUPPORTED;
    total += group_sizes[g];
  }
  for (int l = 0; l < total; ++l) {
    isopo_status st = check_layer(layers[l], true);
    if (st != ISOPO_OK) return st;
  }
  const isopo_layer* first = layers[0];
  for (int l = 1; l < total; ++l) {             // one microbatch: one dtype, one ragged layout
    const isopo_layer* o = layers[l];
    if (o->dtype != first->dtype || o->n_tokens != first->n_tokens || o->n_seq != first->n_seq ||
        o->seq_offsets_dev != first->seq_offsets_dev ||
        std::memcmp(o->seq_offsets_host, first->seq_offsets_host, sizeof(int32_t) * (size_t)(first->n_seq + 1)) != 0)
      return ISOPO_ERR_INVALID_ARG;
  }
  for (int g = 0, l0 = 0; g < n_groups; l0 += group_sizes[g], ++g)      // one input per group
    for (int l = l0 + 1; l < l0 + group_sizes[g]; ++l)
      if (layers[l]->X != layers[l0]->X || layers[l]->d_in != layers[l0]->d_in) return ISOPO_ERR_INVALID_ARG;
  if (!sample_idx_dev || !A || !c || !workspace || !(lambda >= 0.f)) return ISOPO_ERR_INVALID_ARG;
  if (n_samples < 1) return ISOPO_ERR_INVALID_ARG;
  if (n_samples > ISOPO_MAX_SAMPLES) return ISOPO_ERR_UNSUPPORTED;
  if (!enum_in(reg_mode, ISOPO_REG_ABSOLUTE, ISOPO_REG_EMA_TRACE)) return ISOPO_ERR_INVALID_ARG;
  if (reg_mode == ISOPO_REG_EMA_TRACE && (!ema_state || !(ema_decay >= 0.f && ema_decay < 1.f)))
    return ISOPO_ERR_INVALID_ARG;
  if (first->n_tokens == 0) return ISOPO_ERR_INVALID_ARG;     // nothing to sample from
  if (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) return ISOPO_ERR_INVALID_ARG;
  if (ws_bytes < isopo_fisher_samples_block_workspace(first, total, n_samples)) return ISOPO_ERR_WORKSPACE_TOO_SMALL;
  FisherSamplesArgs f;
  f.n_groups = n_groups;
  for (int g = 0, l0 = 0; g < kFisherMaxGroups; ++g) {
    FisherGroup& q = f.group[g];
    const int n = g < n_groups ? group_sizes[g] : 0;
    q.X = n ? layers[l0]->X : nullptr;
    q.d_in = n ? layers[l0]->d_in : 0;
    q.n_layers = n;
    for (int l = 0; l < kFisherMaxGroup; ++l) {
      q.Delta[l] = l < n ? layers[l0 + l]->Delta : nullptr;
      q.d_out[l] = l < n ? layers[l0 + l]->d_out : 0;
    }
    l0 += n;
  }
  f.off = first->seq_offsets_dev; f.sample_idx = sample_idx_dev;
  f.n_tokens = (int)first->n_tokens; f.n_seq = first->n_seq;
  f.n_samples = n_samples; f.bf16 = first->dtype == ISOPO_BF16; f.A = A; f.lambda = lambda;
  f.reg_mode = (int)reg_mode; f.ema_state = ema_state; f.ema_decay = ema_decay; f.c = c; f.fisher_sq = fisher_sq;
  f.workspace = workspace;
  return launch_fisher_samples(f, static_cast<hipStream_t>(stream)) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

isopo_status isopo_fisher_samples_group(const isopo_layer* const* layers, int32_t n_layers,
                                        const int32_t* sample_idx_dev, int32_t n_samples, const float* A, float lambda,
                                        isopo_reg_mode reg_mode, float* ema_state, float ema_decay, float* c,
                                        float* fisher_sq, void* workspace, size_t ws_bytes, void* stream) {
  if (n_layers < 1) return ISOPO_ERR_INVALID_ARG;
  return isopo_fisher_samples_block(layers, &n_layers, 1, sample_idx_dev, n_samples, A, lambda, reg_mode, ema_state,
                                    ema_decay, c, fisher_sq, workspace, ws_bytes, stream);
}

isopo_status isopo_fisher_samples(const isopo_layer* layer, const int32_t* sample_idx_dev, int32_t n_samples,
                                  const float* A, float lambda, isopo_reg_mode reg_mode, float* ema_state,
                                  float ema_decay, float* c, float* fisher_sq, void* workspace, size_t ws_bytes,
                                  void* stream) {
  if (!layer) return ISOPO_ERR_INVALID_ARG;
  return isopo_fisher_samples_group(&layer, 1, sample_idx_dev, n_samples, A, lambda, reg_mode, ema_state, ema_decay, c,
                                    fisher_sq, workspace, ws_bytes, stream);
}

isopo_status isopo_gram_norms(const float* K, int32_t n_seq, float* fisher_sq, float* grad_sq, void* stream) {
  if (!K || n_seq <= 0 || (!fisher_sq && !grad_sq)) return ISOPO_ERR_INVALID_ARG;
  if (n_seq > ISOPO_MAX_SEQ) return ISOPO_ERR_UNSUPPORTED;
  return launch_gram_norms(K, n_seq, fisher_sq, grad_sq, static_cast<hipStream_t>(stream)) == hipSuccess
             ? ISOPO_OK : ISOPO_ERR_HIP;
}

isopo_status isopo_rescale(const float* fisher_sq, const float* grad_sq, int64_t grad_sq_stride, int32_t n_seq,
                           const float* A, const isopo_rescale_params* params, float* c, float* batch_means,
                           void* stream) {
  if (!fisher_sq || !grad_sq || !A || !params || !c || n_seq <= 0 || grad_sq_stride < 1) return ISOPO_ERR_INVALID_ARG;
  if (n_seq > ISOPO_MAX_SEQ) return ISOPO_ERR_UNSUPPORTED;
  RescaleArgs r;
  r.fisher_sq = fisher_sq; r.grad_sq = grad_sq; r.grad_sq_stride = grad_sq_stride; r.n_seq = n_seq; r.A = A;
  r.p = params->p; r.q = params->q; r.r = params->r;
  if (!std::isfinite(r.p) || !std::isfinite(r.q) || !std::isfinite(r.r)) return ISOPO_ERR_INVALID_ARG;
  for (int k = 0; k < 3; ++k) {
    if (!(params->reg[k] >= 0.f) || std::isnan(params->expectation[k])) return ISOPO_ERR_INVALID_ARG;
    r.reg[k] = params->reg[k];
    r.expectation[k] = params->expectation[k];
  }
  r.c = c; r.batch_means = batch_means;
  return launch_rescale(r, static_cast<hipStream_t>(stream)) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

size_t isopo_ntk_eigh_workspace(int32_t n_seq, int32_t batch) {
  if (n_seq <= 0 || n_seq > ISOPO_MAX_SEQ || batch <= 0) return 0;
  return align_up((size_t)batch * eigh_workspace(n_seq));
}

isopo_status isopo_ntk_eigh(const float* K, int32_t n_seq, int32_t batch, double* D, double* U, int32_t* info,
                            void* workspace, size_t ws_bytes, void* stream) {
  if (!K || !D || !U || n_seq <= 0 || batch <= 0) return ISOPO_ERR_INVALID_ARG;
  if (n_seq > ISOPO_MAX_SEQ) return ISOPO_ERR_UNSUPPORTED;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1))) return ISOPO_ERR_INVALID_ARG;
  if (ws_bytes < isopo_ntk_eigh_workspace(n_seq, batch)) return ISOPO_ERR_WORKSPACE_TOO_SMALL;
  return launch_ntk_eigh(K, n_seq, batch, D, U, info, workspace, static_cast<hipStream_t>(stream)) == hipSuccess
             ? ISOPO_OK : ISOPO_ERR_HIP;
}

isopo_status isopo_transform_eigh(const double* D, const double* U, int32_t n_seq, int32_t batch, const float* A,
                                  const float* lambdas, int32_t n_lambda, isopo_reg_mode reg_mode, float* ema_state,
                                  float ema_decay, float* c, int32_t* info, void* stream) {
  if (!D || !U || !A || !lambdas || !c || n_seq <= 0 || batch <= 0 || n_lambda < 1) return ISOPO_ERR_INVALID_ARG;
  if (n_seq > ISOPO_MAX_SEQ || n_lambda > ISOPO_MAX_LAMBDAS) return ISOPO_ERR_UNSUPPORTED;
  if (!enum_in(reg_mode, ISOPO_REG_ABSOLUTE, ISOPO_REG_EMA_TRACE)) return ISOPO_ERR_INVALID_ARG;
  if (reg_mode == ISOPO_REG_EMA_TRACE && (!ema_state || !(ema_decay >= 0.f && ema_decay < 1.f)))
    return ISOPO_ERR_INVALID_ARG;
  EighSolveArgs e;
  e.D = D; e.U = U; e.n_seq = n_seq; e.batch = batch; e.A = A; e.n_lambda = n_lambda;
  for (int l = 0; l < kEighMaxLambdas; ++l) {
    e.lambdas[l] = l < n_lambda ? lambdas[l] : 0.f;
    if (l < n_lambda && !(lambdas[l] >= 0.f)) return ISOPO_ERR_INVALID_ARG;
  }
  e.reg_mode = (int)reg_mode; e.ema_state = ema_state; e.ema_decay = ema_decay; e.c = c; e.info = info;
  return launch_eigh_solve(e, static_cast<hipStream_t>(stream)) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

isopo_status isopo_scale_rows(const void* src, isopo_dtype dtype, int64_t n_tokens, int32_t d,
                              const int32_t* seq_offsets_dev, int32_t n_seq, const float* c, void* dst,
                              void* stream) {
  if (!src || !dst || !c || !seq_offsets_dev || src == dst || n_tokens < 0 || d <= 0 || n_seq <= 0)
    return ISOPO_ERR_INVALID_ARG;
  if (!enum_in(dtype, ISOPO_F32, ISOPO_BF16)) return ISOPO_ERR_UNSUPPORTED;
  if (d % (dtype == ISOPO_BF16 ? 8 : 4) || n_seq > ISOPO_MAX_SEQ || n_tokens >= (int64_t)1 << 31)
    return ISOPO_ERR_UNSUPPORTED;
  if (!aligned16(src) || !aligned16(dst)) return ISOPO_ERR_INVALID_ARG;
  return launch_scale_rows(src, dtype == ISOPO_BF16, n_tokens, d, seq_offsets_dev, n_seq, c, dst,
                           static_cast<hipStream_t>(stream)) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

isopo_status isopo_weighted_grad(const isopo_layer* layer, const float* c, const void* stash, float beta, float* dW,
                                 void* stream) {
  isopo_status st = check_layer(layer, true);
  if (st != ISOPO_OK) return st;
  if (!dW || !aligned16(dW) || !aligned16(stash)) return ISOPO_ERR_INVALID_ARG;
  if (!c && stash) return ISOPO_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool bf16 = layer->dtype == ISOPO_BF16;
  const long long D = (long long)layer->d_out * layer->d_in;
  if (stash) {
    return launch_stash_weighted_sum(stash, bf16, D, D, layer->n_seq, c, beta, dW, false, s) == hipSuccess ? ISOPO_OK
                                                                                                      : ISOPO_ERR_HIP;
  }
  SeqGradArgs a;
  a.X = layer->X; a.Delta = layer->Delta; a.off = layer->seq_offsets_dev; a.off_host = layer->seq_offsets_host; a.c = c; a.out = dW;
  a.d_in = layer->d_in; a.d_out = layer->d_out; a.n_seq = layer->n_seq; a.n_tokens = (int)layer->n_tokens;
  a.row0 = 0; a.rows = layer->d_out; a.out_row0 = 0; a.out_seq_stride = 0;
  a.beta = beta; a.per_sequence = false; a.bf16 = bf16;
  return launch_seq_grad(a, s) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

isopo_status isopo_stash_layout_of(const isopo_layer* layer, isopo_stash_layout* layout, int32_t* tile) {
  isopo_status st = check_layer(layer, false);
  if (st != ISOPO_OK) return st;
  const int t = layer->dtype == ISOPO_BF16
                    ? stash_tile_order_ok(layer->d_out, layer->d_in, (int)layer->n_tokens, layer->n_seq,
                                          layer->seq_offsets_host)
                    : 0;
  if (layout) *layout = t ? ISOPO_STASH_TILE_ORDER : ISOPO_STASH_ROW_MAJOR;
  if (tile) *tile = t;
  return ISOPO_OK;
}

// dW = beta dW + sum_i c_i G_i from a kept stash in either layout, dW in fp32 or bf16
static isopo_status weighted_grad_from_stash(const isopo_layer* layer, const float* c, const void* stash,
                                             bool tile_order, float beta, void* dW, bool dw_bf16, void* stream) {
  isopo_status st = check_layer(layer, true);
  if (st != ISOPO_OK) return st;
  if (!c || !stash || !dW || !aligned16(dW) || !aligned16(stash)) return ISOPO_ERR_INVALID_ARG;
  const bool bf16 = layer->dtype == ISOPO_BF16;
  if (dw_bf16 && !bf16) return ISOPO_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!tile_order) {
    const long long D = (long long)layer->d_out * layer->d_in;
    return launch_stash_weighted_sum(stash, bf16, D, D, layer->n_seq, c, beta, dW, dw_bf16, s) == hipSuccess
               ? ISOPO_OK : ISOPO_ERR_HIP;
  }
  isopo_stash_layout have;
  int32_t tile;
  st = isopo_stash_layout_of(layer, &have, &tile);
  if (st != ISOPO_OK) return st;
  if (have != ISOPO_STASH_TILE_ORDER) return ISOPO_ERR_UNSUPPORTED;      // this layer's kept stash is row-major
  return launch_stash_weighted_sum_tiled(stash, tile, layer->d_out, layer->d_in, layer->n_seq, c, beta, dW, dw_bf16,
                                         s) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

isopo_status isopo_weighted_grad_stash(const isopo_layer* layer, const float* c, const void* stash,
                                       isopo_stash_layout layout, float beta, float* dW, void* stream) {
  if (!enum_in(layout, ISOPO_STASH_ROW_MAJOR, ISOPO_STASH_TILE_ORDER)) return ISOPO_ERR_INVALID_ARG;
  return weighted_grad_from_stash(layer, c, stash, layout == ISOPO_STASH_TILE_ORDER, beta, dW, false, stream);
}

isopo_status isopo_weighted_grad_stash_bf16(const isopo_layer* layer, const float* c, const void* stash,
                                            isopo_stash_layout layout, float beta, void* dW_bf16, void* stream) {
  if (!enum_in(layout, ISOPO_STASH_ROW_MAJOR, ISOPO_STASH_TILE_ORDER)) return ISOPO_ERR_INVALID_ARG;
  return weighted_grad_from_stash(layer, c, stash, layout == ISOPO_STASH_TILE_ORDER, beta, dW_bf16, true, stream);
}

size_t isopo_weighted_grad_scratch(const isopo_layer* layer) {
  if (check_layer(layer, false) != ISOPO_OK) return 0;
  const int d = layer->d_in <= layer->d_out ? layer->d_in : layer->d_out;
  return (size_t)layer->n_tokens * (size_t)d * elem_size(layer->dtype);
}

isopo_status isopo_weighted_grad_prescaled(const isopo_layer* layer, const float* c, float beta, float* dW,
                                           void* scratch, size_t scratch_bytes, void* stream) {
  isopo_status st = check_layer(layer, true);
  if (st != ISOPO_OK) return st;
  if (!c || !dW || !aligned16(dW)) return ISOPO_ERR_INVALID_ARG;
  if (layer->n_tokens == 0) return isopo_weighted_grad(layer, nullptr, nullptr, beta, dW, stream);
  if (!scratch || !aligned16(scratch)) return ISOPO_ERR_INVALID_ARG;
  if (scratch_bytes < isopo_weighted_grad_scratch(layer)) return ISOPO_ERR_WORKSPACE_TOO_SMALL;
  const bool narrow_x = layer->d_in <= layer->d_out;
  st = isopo_scale_rows(narrow_x ? layer->X : layer->Delta, layer->dtype, layer->n_tokens,
                        narrow_x ? layer->d_in : layer->d_out, layer->seq_offsets_dev, layer->n_seq, c, scratch, stream);
  if (st != ISOPO_OK) return st;
  isopo_layer scaled = *layer;
  if (narrow_x) scaled.X = scratch; else scaled.Delta = scratch;
  return isopo_weighted_grad(&scaled, nullptr, nullptr, beta, dW, stream);
}

isopo_status isopo_probe_mfma_loop(int32_t shape, const void* operands, float* sink, int32_t iters, void* stream) {
  if (!operands || !sink || iters < 1 || !aligned16(operands)) return ISOPO_ERR_INVALID_ARG;
  if (shape != 16 && shape != 32) return ISOPO_ERR_INVALID_ARG;
  return launch_mfma_loop(shape, operands, sink, iters, static_cast<hipStream_t>(stream)) == hipSuccess ? ISOPO_OK
                                                                                                         : ISOPO_ERR_HIP;
}

isopo_status isopo_probe_lds_dma(const void* buf, size_t bytes, int32_t waves, int32_t stages, int32_t workgroups,
                                 int32_t iters, float* sink, void* stream) {
  if (!buf || !sink || !aligned16(buf) || iters < 1 || workgroups < 1 || workgroups > 4096) return ISOPO_ERR_INVALID_ARG;
  if (bytes == 0 || bytes % (8 * 32768)) return ISOPO_ERR_INVALID_ARG;
  if ((waves != 2 && waves != 4 && waves != 8 && waves != 16) || (stages != 2 && stages != 4)) return ISOPO_ERR_INVALID_ARG;
  return launch_lds_dma_ring(buf, bytes, waves, stages, workgroups, iters, sink, static_cast<hipStream_t>(stream)) ==
                 hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

isopo_status isopo_probe_contraction_waves(const isopo_layer* layer, int32_t waves, float* dW, void* stream) {
  isopo_status st = check_layer(layer, true);
  if (st != ISOPO_OK) return st;
  if (!dW || !aligned16(dW) || (waves != 4 && waves != 8)) return ISOPO_ERR_INVALID_ARG;
  if (layer->dtype != ISOPO_BF16 || layer->n_tokens == 0) return ISOPO_ERR_UNSUPPORTED;
  if (plan_contraction(layer->d_out, layer->d_in, (int)layer->n_tokens, layer->n_seq, layer->seq_offsets_host, false).tile != 256)
    return ISOPO_ERR_UNSUPPORTED;
  SeqGradArgs a;
  a.X = layer->X; a.Delta = layer->Delta; a.off = layer->seq_offsets_dev; a.off_host = layer->seq_offsets_host; a.c = nullptr; a.out = dW;
  a.d_in = layer->d_in; a.d_out = layer->d_out; a.n_seq = layer->n_seq; a.n_tokens = (int)layer->n_tokens;
  a.row0 = 0; a.rows = layer->d_out; a.out_row0 = 0; a.out_seq_stride = 0;
  a.beta = 0.f; a.per_sequence = false; a.bf16 = true;
  return launch_seq_grad_stream_waves(a, waves, static_cast<hipStream_t>(stream)) == hipSuccess ? ISOPO_OK : ISOPO_ERR_HIP;
}

}  // extern "C"
