// Host-callable launchers of the gfx950 kernels.  Internal to the library: the
// public surface is include/isopo.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace isopo {

// Token-reduction contraction  out[o][k] = sum_t scale(t) * Delta[t][o] * X[t][k].
//   per_sequence = true :  one output per sequence (the stash of G_i), scale = 1
//   per_sequence = false:  one output (dW), scale = c[seq(t)], out = beta*out + sum
struct SeqGradArgs {
  const void* X;
  const void* Delta;
  const int32_t* off;        // device [n_seq+1]
  const int32_t* off_host = nullptr;   // the same values on the host, if the caller has them (work balancing)
  const float* c;            // device [n_seq]; nullptr = unweighted (all ones)
  void* out;                 // stash (input dtype) or dW (fp32)
  int d_in, d_out, n_seq, n_tokens;
  int row0, rows;            // output rows [row0, row0+rows) of d_out handled by this launch
  int out_row0;              // output row o is stored at row (o - out_row0)
  long long out_seq_stride;  // elements between consecutive sequences' outputs (per_sequence)
  float beta;
  bool per_sequence;
  bool bf16;
  // per_sequence, bf16: at most this many workgroups resident at a time (0: no limit), fed from `queue`,
  // eight device counters the launch zeroes; the other compute units stay free for other streams
  int max_workgroups = 0;
  unsigned* queue = nullptr;
  // per_sequence, bf16: store every sequence's gradient in the order the accumulators hold it (see
  // stash_tile_order_ok) instead of row-major
  bool tile_order = false;
};
// The per-sequence bf16 contraction can leave its result in tile order: tiles of T x T outputs (T the plan's
// tile, 256 or 128) in row-major tile order; inside a tile its four (T/2 x T/2) quadrants one after the
// other (upper left, upper right, lower left, lower right); inside a quadrant its strips of 16 rows, top down,
// each strip as pieces of 16 rows x 32 columns, left to right; a piece is 1 KiB, 16 bytes per lane l: its
// element 8 l + q (q = 0..7) is row 4 (l / 16) + q % 4, column l % 16 + 16 (q / 4) of the piece.  That is what
// the 16x16 accumulator blocks of two neighbouring MFMA outputs hold, so the epilogue stores 16 bytes per lane
// without a transpose.  Possible when d_out and d_in are multiples of 256: returns T, else 0.
int stash_tile_order_ok(int d_out, int d_in, int n_tokens, int n_seq, const int32_t* off_host);
// Launch plan of the streaming bf16 contraction (host arithmetic only).
struct ContractionPlan {
  int tile;                    // 256 (one workgroup per CU) or 128 (two)
  int occupancy;
  int tiles_m, tiles_n;
  int n_chunks, chunk_tokens;  // sum-over-all-tokens mode: token chunks (1: no split)
  int whole_tiles;             // sum-over-all-tokens mode: tiles [0, whole_tiles) of the tile order are not split
                               // (one workgroup each, all tokens); the chunks apply to the tiles after them
  int xcd_start[9];            // XCD x walks (item, tile) pairs [xcd_start[x], xcd_start[x+1]) of the item-major
                               // list (items: sequences or chunks); all zero: the x-th eighth of every item's
                               // tiles (per-sequence mode), or no items at all (unsplit)
  long long blocks;            // workgroups to launch
};
ContractionPlan plan_contraction(int rows, int d_in, int n_tokens, int n_seq, const int32_t* off_host,
                                 bool per_sequence);
hipError_t launch_seq_grad(const SeqGradArgs& a, hipStream_t s);
// bf16 only, c == nullptr only: the direct-to-LDS streaming kernel (launch_seq_grad routes to it).
hipError_t launch_seq_grad_stream(const SeqGradArgs& a, hipStream_t s);
// Schedule probe: the plain sum over all tokens (c == nullptr, not per sequence) on the 256x256 tile with four or
// eight waves per workgroup; hipErrorInvalidValue where the plan would take the 128x128 tile.
hipError_t launch_seq_grad_stream_waves(const SeqGradArgs& a, int waves, hipStream_t s);

// K partials from the stash:  for p in [p0, p1):  acc[i][j] += S[i][p] * S[j][p].
struct StashGramArgs {
  const void* stash;         // [n_seq][seq_stride] elements, input dtype
  long long seq_stride;
  long long p0, p1;          // element range inside each sequence's gradient
  int n_seq;
  bool bf16;
  bool first;                // overwrite the partial slots instead of adding to them
  float* partials;           // [stash_gram_slots()][stash_gram_slot_floats(n_seq)]
};
int stash_gram_slots();
// bytes of partial-sum scratch the Gram reduction needs (0 = shape not covered)
size_t stash_gram_partial_bytes(int n_seq, bool bf16);
// n_seq > 128 (bf16): 128x128 super-block pairs
int stash_gram_large_slots(int n_seq);
size_t stash_gram_large_slot_floats(int n_seq);
hipError_t launch_stash_gram_large(const StashGramArgs& a, hipStream_t s);
hipError_t launch_stash_gram_large_finish(const float* partials, int n_seq, float* K, hipStream_t s);
size_t stash_gram_slot_floats(int n_seq);
hipError_t launch_stash_gram(const StashGramArgs& a, hipStream_t s);
// K[i][j] = K[j][i] = sum over slots (fixed order) of the (i<=j) entry.
hipError_t launch_stash_gram_finish(const float* partials, bool bf16, int n_seq, float* K, hipStream_t s);
// bf16 stash: row-contiguous DMA into an LDS ring (launch_stash_gram routes to it); uses fewer slots.
int stash_gram_stream_slots();
hipError_t launch_stash_gram_stream(const StashGramArgs& a, hipStream_t s);

// dW[p] = beta*dW[p] + sum_i c[i] * stash[i][p],  p in [0, n_elem).  dW fp32, or bf16 (dw_bf16; bf16 stash only:
// fp32 sums, one rounding).
hipError_t launch_stash_weighted_sum(const void* stash, bool bf16, long long seq_stride, long long n_elem,
                                     int n_seq, const float* c, float beta, void* dW, bool dw_bf16, hipStream_t s);
// The same from a bf16 stash in tile order (tile 256 or 128, d_out and d_in multiples of it); dW row-major.
hipError_t launch_stash_weighted_sum_tiled(const void* stash, int tile, int d_out, int d_in, int n_seq, const float* c,
                                           float beta, void* dW, bool dw_bf16, hipStream_t s);

// Ghost Gram: K_ij = sum_{t in i, s in j} (x_t.x_s)(delta_t.delta_s).
struct GhostArgs {
  const void* X;
  const void* Delta;
  const int32_t* off;
  int n_tokens, d_in, d_out, n_seq;
  bool bf16;
  int32_t* tok_seq;          // workspace [n_tokens]
  double* K64;               // workspace [n_seq*n_seq]
  float* parts;              // workspace [ghost_parts_bytes / 4], bf16 with ghost_feature_split > 1 only
  float* K;
};
hipError_t launch_ghost_gram(const GhostArgs& a, hipStream_t s);
// bf16 ghost kernel: ranges the 64-feature slices of X and Delta are cut into when the microbatch has too few
// 128x128 token-tile pairs to fill the compute units (1: no split).  A workgroup then forms the two
// token-by-token products over one range, and a second kernel sums the ranges' fp32 parts.  The count is the
// one with the smallest modelled time: a workgroup's serial walk over its features against the pass over the
// parts (rates measured on one MI355X).  Host arithmetic, shared by the launcher, the workspace size and the
// cost model.
constexpr double kGhostParts = 4.0e-6;        // s, the kernel that sums the ranges ...
constexpr double kRateGhostParts = 2.5e12;    // ... plus B/s over the parts
constexpr size_t kGhostPartBytes = 2 * 128 * 128 * sizeof(float);   // P and Q of one (tile pair, range)
// s per 64-feature ring stage of one workgroup while `wgs` of them run: the stages stream through the L2s,
// whose bandwidth the workgroups share (two fit a compute unit; beyond 512 they queue)
inline double ghost_stage_time(long long wgs) {
  const double w = wgs > 512 ? 512.0 : (double)wgs;
  if (w <= 128.0) return 0.6e-6;
  if (w <= 256.0) return 0.6e-6 + 0.4e-6 * (w - 128.0) / 128.0;
  return 1.0e-6 + 0.32e-6 * (w - 256.0) / 256.0;
}
inline double ghost_walk_time(long long pairs, int d_in, int d_out, int split) {
  const double stages = (double)((d_in + 63) / 64 + (d_out + 63) / 64) / split;
  const double walk = stages * ghost_stage_time(pairs * split);
  return split > 1 ? walk + kGhostParts + (double)pairs * split * kGhostPartBytes / kRateGhostParts : walk;
}
inline int ghost_feature_split(int n_tokens, int d_in, int d_out) {
  const long long nt = (n_tokens + 127) / 128, pairs = nt * (nt + 1) / 2;
  if (pairs <= 0) return 1;
  const long long slices = (d_in + 63) / 64 + (d_out + 63) / 64;
  long long most = 512 / pairs;                        // two workgroups per compute unit (LDS ring: 64 KiB)
  if (most > slices / 16) most = slices / 16;          // a range is worth its prologue from 16 slices on
  if (most > 32) most = 32;
  int best = 1;
  for (int s = 2; s <= most; ++s)
    if (ghost_walk_time(pairs, d_in, d_out, s) < ghost_walk_time(pairs, d_in, d_out, best)) best = s;
  return best;
}
inline size_t ghost_parts_bytes(int n_tokens, int d_in, int d_out) {
  const int split = ghost_feature_split(n_tokens, d_in, d_out);
  if (split <= 1) return 0;
  const size_t nt = (size_t)(n_tokens + 127) / 128;
  return nt * (nt + 1) / 2 * (size_t)split * kGhostPartBytes;
}

// dst[t][:] = c[seq(t)] * src[t][:] (rounded to the storage type).
hipError_t launch_scale_rows(const void* src, bool bf16, long long n_tokens, int d, const int32_t* off, int n_seq,
                             const float* c, void* dst, hipStream_t s);

// Token-position-sample Fisher norms and the coefficients c_i = A_i / sqrt(F_i^2 + reg), for a group of
// layers that share their input X (q/k/v, gate/up): X is streamed once for the whole group.
// Several such groups of one microbatch (a transformer block's {q,k,v}, {o}, {gate,up}, {down}) go in one
// launch, so that only the last group's last round of workgroups leaves compute units idle.
constexpr int kFisherMaxGroup = 4;
constexpr int kFisherMaxGroups = 8;
struct FisherGroup {
  const void* X;
  const void* Delta[kFisherMaxGroup];
  int d_out[kFisherMaxGroup];
  int d_in, n_layers;
};
struct FisherSamplesArgs {
  FisherGroup group[kFisherMaxGroups];
  int n_groups;
  const int32_t* off;
  const int32_t* sample_idx;   // device [n_samples], token rows
  int n_tokens, n_seq, n_samples;
  bool bf16;
  const float* A;
  float lambda;
  int reg_mode;                // 0 absolute, 1 times this batch's mean F^2, 2 times its trailing mean
  float* ema_state;            // [layers of all groups][2]: trailing mean, number of minibatches seen (reg_mode 2)
  float ema_decay;
  float* c;                    // [layers of all groups][n_seq], group after group
  float* fisher_sq;            // optional, same shape
  void* workspace;
};
size_t fisher_samples_workspace(int n_tokens, int n_seq, int n_samples, int n_layers);
hipError_t launch_fisher_samples(const FisherSamplesArgs& a, hipStream_t s);

struct TransformArgs {
  const float* K;
  const float* A;
  int n_seq, batch;
  int variant, reg_mode;
  float lambda;
  float* c;
  int32_t* info;
  double* workspace;         // [batch][n_seq*n_seq + n_seq] when n_seq > kTransformLdsMax, else unused
  float* ema_state = nullptr;  // reg_mode 2: [batch][2] trailing mean of tr(K)/m, number of minibatches seen
  float ema_decay = 0.f;
};
constexpr int kTransformLdsMax = 128;
constexpr int kTransformWidePanelMax = 512;   // larger problems factor panels of 16 columns instead of 32 (the panel has to fit in LDS)
hipError_t launch_transform(const TransformArgs& a, hipStream_t s);

// Generalised (p, q, r) re-scaling of the per-sequence coefficients.
struct RescaleArgs {
  const float* fisher_sq;      // [n_seq] F_norm^2
  const float* grad_sq;        // ||G_i||^2 at grad_sq[i * grad_sq_stride]
  long long grad_sq_stride;
  int n_seq;
  const float* A;
  float p, q, r;
  float reg[3];                // regularisation factors for (F_norm, ||G||, rel_F_norm)
  float expectation[3];        // E[val^2] for each; negative: this batch's mean
  float* c;
  float* batch_means;          // optional [3]
};
hipError_t launch_rescale(const RescaleArgs& a, hipStream_t s);
hipError_t launch_gram_norms(const float* K, int m, float* fisher_sq, float* grad_sq, hipStream_t s);

// Eigendecomposition route of the interacting variant.
constexpr int kEighMaxSeq = 1024;
constexpr size_t kEighLdsBytes = 144 * 1024;     // work matrix + eigenvectors in LDS up to this size
constexpr int kEighMaxLambdas = 16;
struct EighSolveArgs {
  const double* D;             // [batch][n_seq]
  const double* U;             // [batch][n_seq][n_seq]
  int n_seq, batch;
  const float* A;              // [batch][n_seq]
  float lambdas[kEighMaxLambdas];
  int n_lambda;
  int reg_mode;                // 0 absolute, 1 times mean(D), 2 times the trailing mean of mean(D)
  float* ema_state;            // [batch][2]: trailing mean, number of minibatches seen
  float ema_decay;
  float* c;                    // [batch][n_lambda][n_seq]
  int32_t* info;               // [batch]
};
size_t eigh_workspace(int m);           // bytes per problem
hipError_t launch_ntk_eigh(const float* K, int m, int batch, double* D, double* U, int32_t* info, void* workspace,
                           hipStream_t s);
hipError_t launch_eigh_solve(const EighSolveArgs& a, hipStream_t s);

// Diagnostic: a loop of nothing but bf16 MFMAs (shape 32: 32x32x16, shape 16: 16x16x32) on register operands,
// kProbeWorkgroups workgroups of 256 threads; 2 * 128 * 128 * 32 flop per wave and trip.
constexpr int kProbeWorkgroups = 256;
hipError_t launch_mfma_loop(int shape, const void* operands, float* sink, int iters, hipStream_t s);
// `workgroups` workgroups of `waves` waves (2, 4, 8 or 16) stream the buffer (bytes: a multiple of 8 * 32 KiB,
// workgroup b walks its (b mod 8)-th eighth) into a ring of `stages` (2 or 4) LDS stages of 32 KiB, `iters`
// stages each; sink: float [workgroups].
hipError_t launch_lds_dma_ring(const void* buf, size_t bytes, int waves, int stages, int workgroups, int iters,
                               float* sink, hipStream_t s);

}  // namespace isopo
