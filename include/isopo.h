/*
 * isopo.h - C ABI of the MI355X (gfx950) ISOPO layer-step library.
 *
 * One linear layer of a policy network sees, per microbatch, token activations
 * X = act_in [N, d_in] and back-propagated output gradients Delta = grad_out
 * [N, d_out] of sum(log_prob), grouped into m = n_seq contiguous sequences.
 * The per-sequence log-probability gradient is G_i = Delta_i^T X_i
 * [d_out, d_in] (both hook listings: `grad_out.T @ act_in`).  The layer step is
 *
 *   1. isopo_layer_gram     K_ij = <G_i, G_j>_F          (K = J J^T, interacting-
 *                                                         variant section)
 *   2. isopo_transform      c from K and the advantages A: Fisher-normalised
 *                           (non-interacting update u_l with eq. F-norm-basic)
 *                           or c = (K + reg I)^-1 A (interacting update)
 *   3. isopo_weighted_grad  dW = beta dW + sum_i c_i G_i
 *                              = beta dW + Delta^T diag(c_tok) X
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless the name ends in _host.
 *     The caller owns every buffer; the library never allocates or frees
 *     device memory and never synchronises the stream or the device.
 *   - Matrices are dense row-major.  X, Delta are fp32 or bf16 (isopo_dtype);
 *     K, A, c, dW are fp32.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream);
 *     all work is enqueued on it in order.
 *   - Errors a host check can see return a non-zero isopo_status and enqueue
 *     nothing.  Conditions only the device can see are reported through
 *     info_dev (isopo_transform).
 *   - d_in and d_out must be multiples of 8 (bf16) or 4 (fp32) so token rows
 *     are 16-byte aligned; X, Delta, stash and workspace pointers must be
 *     16-byte aligned (256 for workspace).
 *   - n_seq <= ISOPO_MAX_SEQ.  A zero-length sequence is legal: its G_i is 0,
 *     its row and column of K are 0.
 */
#ifndef ISOPO_H
#define ISOPO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ISOPO_MAX_SEQ 1024

typedef enum {
  ISOPO_OK = 0,
  ISOPO_ERR_INVALID_ARG = 1,        /* null pointer, non-positive size, bad enum, misalignment */
  ISOPO_ERR_BAD_OFFSETS = 2,        /* host offsets not 0-based, not non-decreasing or not ending at n_tokens */
  ISOPO_ERR_UNSUPPORTED = 3,        /* dtype / shape the kernels do not cover */
  ISOPO_ERR_WORKSPACE_TOO_SMALL = 4,
  ISOPO_ERR_HIP = 5,                /* a HIP launch or query failed */
  ISOPO_ERR_SCRATCH_LIMIT = 6       /* isopo_transform_noalloc: the problem needs more than the library's static scratch */
} isopo_status;

typedef enum { ISOPO_F32 = 0, ISOPO_BF16 = 1 } isopo_dtype;

/* How K is formed.  GHOST: K_ij = sum_{t in i, s in j} (x_t.x_s)(delta_t.delta_s),
 * from the rank-one structure of token gradients (efficient-implementation
 * paragraph); no G_i exists.  MATERIALISED: every G_i is written to a stash and
 * K is its Gram matrix (interacting listing).  AUTO lets the cost model pick. */
typedef enum { ISOPO_GRAM_AUTO = 0, ISOPO_GRAM_GHOST = 1, ISOPO_GRAM_MATERIALISED = 2 } isopo_gram_path;

typedef enum {
  ISOPO_VARIANT_FISHER = 0,         /* c_i = A_i / sqrt((1/m) sum_j K_ij^2 + reg) */
  ISOPO_VARIANT_INTERACTING = 1     /* c = (K + reg I)^-1 A */
} isopo_variant;

typedef enum {
  ISOPO_REG_ABSOLUTE = 0,           /* reg = lambda (the Tikhonov constant as printed; reg_l of the update u_l) */
  ISOPO_REG_REL_TRACE = 1,          /* reg = lambda * this batch's typical value of the quantity reg is added to:
                                       INTERACTING: tr(K)/m, the mean eigenvalue of K (as the interacting
                                       experiment's regulariser is relative to);
                                       FISHER: mean_i ||g_i||_F^2 (the non-interacting derivation compares reg_l
                                       with the typical value of ||.||_F^2).  Either way c scales like 1/K under a
                                       rescaling of Delta, whatever lambda is */
  ISOPO_REG_EMA_TRACE = 2           /* reg = lambda * trailing mean over minibatches of the same value
                                       (interacting experiment: factor * E[mean(D)], decay 0.9);
                                       isopo_transform_ema, isopo_transform_eigh and
                                       isopo_fisher_samples (there: of the batch mean of F^2) */
} isopo_reg_mode;

/* One ragged layer problem.  All pointers caller-owned. */
typedef struct {
  const void* X;                    /* device [n_tokens, d_in]  */
  const void* Delta;                /* device [n_tokens, d_out] */
  isopo_dtype dtype;                /* of X and Delta */
  int64_t n_tokens;                 /* N, < 2^31 */
  int32_t d_in, d_out, n_seq;
  const int32_t* seq_offsets_dev;   /* device [n_seq+1]: 0 = off[0] <= ... <= off[n_seq] = n_tokens */
  const int32_t* seq_offsets_host;  /* the same values on the host (validation, path choice, grid sizing) */
} isopo_layer;

/* What isopo_layer_gram would do for `requested` and how much workspace it
 * wants.  Pure host function.
 *   *chosen       the path taken (never AUTO)
 *   *ws_full      bytes that hold the whole stash [n_seq, d_out, d_in] (needed for keep_stash)
 *   *ws_min       the smallest workspace the call accepts (the stash is then
 *                 formed and consumed in chunks of output rows)
 * Any out pointer may be NULL. */
isopo_status isopo_layer_gram_plan(const isopo_layer* layer, isopo_gram_path requested,
                                   isopo_gram_path* chosen, size_t* ws_full, size_t* ws_min);

/* Modelled cost (seconds on one MI355X) of forming K by each path; the AUTO
 * choice is the smaller.  Pure host function; exposed for tests. */
isopo_status isopo_gram_cost_model(const isopo_layer* layer, double* t_ghost, double* t_materialised);

/* How the bf16 contraction behind isopo_seq_grads (per_sequence != 0; `grad_out.T @ act_in` per sequence,
 * both hook listings) or the unweighted isopo_weighted_grad (per_sequence == 0) would be launched for
 * this layer.  Pure host function; needs seq_offsets_host; exposed for tests of the launch logic.
 *   tile               square output tile edge, 256 or 128
 *   workgroups_per_cu  resident workgroups per compute unit for that tile (1 or 2)
 *   tiles              output tiles of one item (item: a sequence, or a token chunk)
 *   n_chunks, chunk_tokens   token split of the unweighted mode (1, n_tokens: none); partial tiles of a
 *                      split are added to dW with fp32 atomics
 *   whole_tiles        unweighted mode with more 256x256 tiles than compute units: the first whole_tiles
 *                      tiles (a multiple of 256, the full rounds of one tile per compute unit) are not
 *                      split; the chunks apply to the tiles of the last, partial round only.  0: the
 *                      split, if any, applies to every tile
 *   xcd_start[9]       the item-major list of (item, tile) pairs is cut into 8 contiguous ranges of equal
 *                      work, XCD x walks [xcd_start[x], xcd_start[x+1]).  All zero: no list - per-sequence
 *                      mode with tiles % 8 == 0 gives XCD x the x-th eighth of every sequence's tiles,
 *                      the unsplit unweighted mode has one item
 *   workgroups         grid size of the one-workgroup-per-pair launch (some workgroups may find their XCD's
 *                      range exhausted and exit); isopo_layer_gram and isopo_seq_grads_limited launch at most
 *                      256 (or the budget) persistent workgroups over the same list instead */
typedef struct {
  int32_t tile, workgroups_per_cu, tiles, n_chunks, chunk_tokens;
  int32_t xcd_start[9];
  int64_t workgroups;
  int32_t whole_tiles;
} isopo_contraction_plan_info;
isopo_status isopo_contraction_plan(const isopo_layer* layer, int per_sequence, isopo_contraction_plan_info* plan);

/* Layout of a stash that isopo_layer_gram keeps.
 *   ROW_MAJOR   [n_seq, d_out, d_in], what `torch.stack(seq_grads)` of the interacting listing holds.
 *   TILE_ORDER  per sequence the same d_out * d_in elements in the order the matrix cores' accumulators
 *               hold them, so that the contraction stores them without a transpose (bf16 layers whose
 *               d_out and d_in are multiples of 256): T x T tiles (T = 256 or 128, as the contraction
 *               plan chooses) in row-major tile order; inside a tile its four (T/2 x T/2) quadrants (upper
 *               left, upper right, lower left, lower right); inside a quadrant its strips of 16 rows, top
 *               down, each strip as pieces of 16 rows x 32 columns, left to right; element 8 l + q
 *               (l = 0..63, q = 0..7) of a piece is its row 4 (l / 16) + q % 4, column l % 16 + 16 (q / 4).
 * isopo_stash_layout_of tells which of the two keep_stash = 2 leaves for a layer (a pure host function of
 * dtype, shape and sequence offsets; *tile = T, or 0 for ROW_MAJOR).  The Gram matrix does not depend on
 * the order of the elements; isopo_weighted_grad_stash forms dW (row-major, as always) from either. */
typedef enum { ISOPO_STASH_ROW_MAJOR = 0, ISOPO_STASH_TILE_ORDER = 1 } isopo_stash_layout;
isopo_status isopo_stash_layout_of(const isopo_layer* layer, isopo_stash_layout* layout, int32_t* tile);

/* K [n_seq, n_seq] fp32, both triangles written, bit-symmetric.
 *   workspace/ws_bytes  device scratch, >= ws_min of the plan.
 *   keep_stash          non-zero: leave the per-sequence gradients in the
 *                       workspace, starting at its first byte, in the stash dtype
 *                       (bf16 for bf16 inputs, fp32 for fp32 inputs).
 *                       1: as [n_seq, d_out, d_in], for isopo_weighted_grad;
 *                       2: in the layout isopo_stash_layout_of reports for the
 *                       layer (the faster one), for isopo_weighted_grad_stash.
 *                       Needs ws_bytes >= ws_full and the MATERIALISED path
 *                       (forced, or AUTO resolving to it); otherwise
 *                       ISOPO_ERR_WORKSPACE_TOO_SMALL / ISOPO_ERR_INVALID_ARG. */
isopo_status isopo_layer_gram(const isopo_layer* layer, isopo_gram_path path, float* K,
                              void* workspace, size_t ws_bytes, int keep_stash, void* stream);

/* The two halves of the MATERIALISED path on their own.
 *
 * isopo_seq_grads: stash[i] = G_i = Delta_i^T X_i for every sequence
 * (`seq_grads.append(grad_out.T @ act_in)`), [n_seq, d_out, d_in] in the input
 * dtype (fp32 accumulation, one rounding for bf16).
 *
 * isopo_stash_gram: K_ij = sum(G_i * G_j) from such a stash
 * (`ntk[i, j] = torch.sum(seq_grads[i] * seq_grads[j])`), n_elem = d_out * d_in
 * elements per sequence.  workspace >= isopo_stash_gram_workspace(n_seq). */
isopo_status isopo_seq_grads(const isopo_layer* layer, void* stash, void* stream);

/* isopo_seq_grads on a budget of compute units, for callers that overlap this layer's contraction with
 * bandwidth-bound work queued on another stream (the Gram pass and the stash-weighted sum of the layer
 * before): at most max_workgroups workgroups are resident at a time, each on a compute unit of its own,
 * and the other units stay free.  The result is the same stash, bit for bit.
 *   max_workgroups  0: no limit (isopo_seq_grads).  Otherwise 8..256, rounded down to a multiple of 8
 *                   (the workgroups are dealt evenly to the 8 accelerator dies).  Honoured for bf16
 *                   layers large enough for the 256x256 tile with more tiles than the budget; smaller
 *                   problems and fp32 inputs run as isopo_seq_grads does.
 *   queue_dev       device uint32[8], 4-byte aligned, caller-owned scratch; zeroed and used by the call
 *                   (work counters); must not be shared by launches that may run concurrently */
isopo_status isopo_seq_grads_limited(const isopo_layer* layer, void* stash, int32_t max_workgroups,
                                     uint32_t* queue_dev, void* stream);

/* isopo_seq_grads_limited with the layout of the stash as an argument: ROW_MAJOR is that call; TILE_ORDER
 * writes the same per-sequence gradients (`grad_out.T @ act_in`) in the order isopo_layer_gram(keep_stash =
 * 2) leaves them (ISOPO_ERR_UNSUPPORTED where isopo_stash_layout_of reports ROW_MAJOR for the layer).
 * max_workgroups = 0 and queue_dev = NULL: no budget. */
isopo_status isopo_seq_grads_stash(const isopo_layer* layer, void* stash, isopo_stash_layout layout,
                                   int32_t max_workgroups, uint32_t* queue_dev, void* stream);
size_t isopo_stash_gram_workspace(int32_t n_seq);
isopo_status isopo_stash_gram(const void* stash, isopo_dtype dtype, int32_t n_seq, int64_t n_elem, float* K,
                              void* workspace, size_t ws_bytes, void* stream);

/* Bytes of device workspace isopo_transform needs (0 for n_seq <= 128). */
size_t isopo_transform_workspace(int32_t n_seq, int32_t batch);

/* Coefficients from K and A, for `batch` independent problems laid out
 * back to back: K [batch, n_seq, n_seq], A [batch, n_seq] -> c [batch, n_seq].
 *   info_dev  device int32 [batch] or NULL.  0: ok.  k > 0 (INTERACTING only):
 *             the k-th pivot of K + reg I was not positive; c of that problem
 *             is then filled with NaN.  FISHER: a zero denominator gives
 *             c_i = 0. */
isopo_status isopo_transform(const float* K, const float* A, int32_t n_seq, int32_t batch,
                             isopo_variant variant, float lambda, isopo_reg_mode reg_mode,
                             float* c, int32_t* info_dev, void* workspace, size_t ws_bytes,
                             void* stream);

/* isopo_transform for callers that cannot allocate or pass device scratch: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace, same kernels,
 * same results bit for bit.  The fp64 work matrices that n_seq > 128 needs live in an array the library
 * holds on each GPU it runs on (ISOPO_NOALLOC_SCRATCH_BYTES per GPU, until the process ends); the call
 * allocates and frees nothing.
 *   limit   isopo_transform_workspace(n_seq, batch) <= ISOPO_NOALLOC_SCRATCH_BYTES, e.g. a block's seven
 *           256-sequence problems, or one problem of 1024 sequences; beyond it ISOPO_ERR_SCRATCH_LIMIT,
 *           nothing enqueued
 *   device  the array of the device that is current at the call is used: the stream must belong to it.  The
 *           first call on a device looks the array's address up (make it outside stream capture)
 *   races   all calls on one GPU share that GPU's array: calls that may overlap in time (two streams, two
 *           threads) race on it; order them, or use isopo_transform with workspaces of their own.  The
 *           array keeps the last call's contents; no call depends on them */
#define ISOPO_NOALLOC_SCRATCH_BYTES ((size_t)16 << 20)
isopo_status isopo_transform_noalloc(const float* K, const float* A, int32_t n_seq, int32_t batch,
                                     isopo_variant variant, float lambda, isopo_reg_mode reg_mode,
                                     float* c, int32_t* info_dev, void* stream);

/* isopo_transform with the interacting experiment's regulariser, reg = factor * E[mean(D)]: the
 * trailing mean over minibatches (this one included) of the Gram matrix's mean eigenvalue, which is
 * tr(K)/n_seq, so the fast factorisation route serves it too.  For FISHER the value averaged is the batch
 * mean of the Fisher norms, mean_i (1/m) sum_j K_ij^2, as under ISOPO_REG_REL_TRACE.
 *   ema_state  device float [batch, 2] per problem {E, number of minibatches seen}; zero it before the
 *              first minibatch.  Updated by the call: E <- this batch's value v on the first minibatch,
 *              E <- decay E + (1 - decay) v after (decay 0.9 in the experiment)
 *   factor     >= 0 (1.0 in the experiment);  0 <= ema_decay < 1
 * Everything else as isopo_transform. */
isopo_status isopo_transform_ema(const float* K, const float* A, int32_t n_seq, int32_t batch,
                                 isopo_variant variant, float factor, float* ema_state, float ema_decay,
                                 float* c, int32_t* info_dev, void* workspace, size_t ws_bytes, void* stream);

/* dW [d_out, d_in] fp32 = beta * dW + sum_i c_i G_i.
 *   stash  NULL: contract X and Delta again, dW = Delta^T diag(c_tok) X
 *          (`grad += advantages[seq_id] * rescaling(...) * seq_logprob_grad`, summed over the sequences).
 *          bf16 inputs: one launch of the matrix-core contraction that walks the tokens sequence by
 *          sequence; the tokens enter unscaled and the fp32 accumulators are re-expressed in units of each
 *          sequence's coefficient where a sequence ends, so no operand is scaled, copied or rounded and no
 *          scratch is needed.  A sequence with c_i = 0 is skipped (it contributes exactly 0, whatever its
 *          rows hold); the ratios c_i / c_j of the non-zero coefficients must be representable in fp32
 *          next to the sums (a span of 2^60 is safe).  fp32 inputs: the rows of Delta are scaled in
 *          registers.
 *          non-NULL: the stash isopo_layer_gram left (keep_stash), read once.
 *   c      device [n_seq].  NULL (only with stash == NULL) means all ones:
 *          dW = beta dW + Delta^T X with no scaling at all.  That is the
 *          plain REINFORCE weight gradient when the advantages were folded into
 *          the loss (so Delta already carries them), and it is the baseline the
 *          layer step's overhead is measured against.
 * Reproducibility: from the stash the sum runs in a fixed order (bit-identical from run to run).
 * From X and Delta with few output tiles and many tokens the token range is split and the partial
 * tiles are added with fp32 atomics, so dW can then differ between runs by fp32 rounding. */
isopo_status isopo_weighted_grad(const isopo_layer* layer, const float* c, const void* stash,
                                 float beta, float* dW, void* stream);

/* The same sum over a kept stash, `stack(seq_grads) @ coef` of the interacting listing, from a stash in
 * either layout: ROW_MAJOR is isopo_weighted_grad with that stash; TILE_ORDER reads the stash that
 * isopo_layer_gram(keep_stash = 2) left for this layer (ISOPO_ERR_UNSUPPORTED if isopo_stash_layout_of
 * reports ROW_MAJOR for it).  c and stash must not be NULL.  dW is row-major [d_out, d_in] in both cases;
 * fixed summation order, bit-identical from run to run. */
isopo_status isopo_weighted_grad_stash(const isopo_layer* layer, const float* c, const void* stash,
                                       isopo_stash_layout layout, float beta, float* dW, void* stream);

/* isopo_weighted_grad_stash with dW [d_out, d_in] in bf16, the gradient buffer of a bf16 model's parameter
 * (`mod.grad += ...` of both listings where `mod.weight` is bf16): the sums run in fp32 as before and
 * dW = bf16(beta * dW + sum_i c_i G_i) is rounded once, to nearest even; with beta = 0 the result is the
 * fp32 call's result rounded.  The pass is bound by HBM and by the lines of dW it writes back, of which
 * there are half as many.  bf16 layers only (ISOPO_ERR_UNSUPPORTED otherwise); dW_bf16 device, 16-byte
 * aligned, caller-owned; everything else as isopo_weighted_grad_stash. */
isopo_status isopo_weighted_grad_stash_bf16(const isopo_layer* layer, const float* c, const void* stash,
                                            isopo_stash_layout layout, float beta, void* dW_bf16, void* stream);

/* The non-interacting update's coefficients with the paper's own Fisher-norm estimate (eq.
 * formal-F-norm; F_norm of the non-interacting listing): from n_samples sampled token rows j of the
 * microbatch (a0 = act_in[samples], g0 = grad_out[samples]),
 *     F_i^2 = sum_j (g0_j . G_i a0_j)^2 / sum_j (||g0_j|| ||a0_j||)^2,   c_i = A_i / sqrt(F_i^2 + reg).
 * Evaluated in ghost form, G_i a0_j = sum_{t in i} delta_t (x_t . a0_j) (eq. (one)): no per-sequence
 * gradient is formed, the cost is 2 N n_samples (d_in + d_out) flop, and c is known before any
 * contraction, so the whole update is one weighted contraction (isopo_weighted_grad with c and no stash).
 *   sample_idx_dev  device int32 [n_samples], token row indices in [0, n_tokens) (the caller draws
 *                   them, e.g. randperm(N)[:n_samples]; an index outside the range is clamped
 *                   into it); 1 <= n_samples <= ISOPO_MAX_SAMPLES
 *   reg_mode        ABSOLUTE: reg = lambda.  REL_TRACE: reg = lambda * mean_i F_i^2 of this batch.
 *                   EMA_TRACE: reg = lambda * E[mean_i F_i^2], the listing's "trailing minibatch
 *                   means": E <- the batch mean on the first call, E <- decay E + (1 - decay) mean
 *                   after, this batch included
 *   ema_state       device float[2] {E, number of minibatches seen}; zero it before the first
 *                   minibatch; required for EMA_TRACE, ignored otherwise
 *   fisher_sq       optional device [n_seq]: F_i^2
 * A zero denominator (empty sequence, reg = 0) gives c_i = 0. */
#define ISOPO_MAX_SAMPLES 128
size_t isopo_fisher_samples_workspace(const isopo_layer* layer, int32_t n_samples);
isopo_status isopo_fisher_samples(const isopo_layer* layer, const int32_t* sample_idx_dev, int32_t n_samples,
                                  const float* A, float lambda, isopo_reg_mode reg_mode, float* ema_state,
                                  float ema_decay, float* c, float* fisher_sq, void* workspace, size_t ws_bytes,
                                  void* stream);

/* The same for up to ISOPO_MAX_GROUP layers that share their input (q/k/v, gate/up of a transformer
 * block): every layers[l] must have the same X pointer, dtype, n_tokens, d_in, n_seq and offsets; only
 * Delta and d_out differ.  X is streamed once for the group (its token-by-sample product is common),
 * each Delta once.  One set of samples and one advantage vector serve the group.
 *   c, fisher_sq   device [n_layers, n_seq]
 *   ema_state      device float[n_layers][2] (EMA_TRACE), one trailing mean per layer */
#define ISOPO_MAX_GROUP 4
size_t isopo_fisher_samples_group_workspace(const isopo_layer* layer, int32_t n_layers, int32_t n_samples);
isopo_status isopo_fisher_samples_group(const isopo_layer* const* layers, int32_t n_layers,
                                        const int32_t* sample_idx_dev, int32_t n_samples, const float* A, float lambda,
                                        isopo_reg_mode reg_mode, float* ema_state, float ema_decay, float* c,
                                        float* fisher_sq, void* workspace, size_t ws_bytes, void* stream);

/* The same for several such groups of one microbatch in one launch - the projections of a transformer
 * block, {q, k, v}, {o}, {gate, up}, {down}: the non-interacting update is formed "in each layer
 * individually", but nothing in one layer's estimate waits for another's, and launched together the groups'
 * workgroups fill the chip one after the other, so that only the last group's last round leaves compute
 * units idle (a quarter of a launch per group otherwise, at 7e4 tokens).
 *   layers        the groups' layers back to back (group 0's first); within a group as for
 *                 isopo_fisher_samples_group (one X, one d_in); all layers share dtype, n_tokens, n_seq
 *                 and the offsets
 *   group_sizes   host [n_groups], each 1..ISOPO_MAX_GROUP; 1 <= n_groups <= ISOPO_MAX_GROUPS
 *   c, fisher_sq  device [sum of group_sizes, n_seq], in the order of `layers`
 *   ema_state     device float[sum of group_sizes][2] (EMA_TRACE)
 *   workspace     isopo_fisher_samples_block_workspace(layers[0], sum of group_sizes, n_samples) bytes */
#define ISOPO_MAX_GROUPS 8
size_t isopo_fisher_samples_block_workspace(const isopo_layer* layer, int32_t n_layers_total, int32_t n_samples);
isopo_status isopo_fisher_samples_block(const isopo_layer* const* layers, const int32_t* group_sizes, int32_t n_groups,
                                        const int32_t* sample_idx_dev, int32_t n_samples, const float* A, float lambda,
                                        isopo_reg_mode reg_mode, float* ema_state, float ema_decay, float* c,
                                        float* fisher_sq, void* workspace, size_t ws_bytes, void* stream);

/* Norms the re-scalings are built from, read off the Gram matrix: fisher_sq[i] = (1/m) sum_j K_ij^2
 * (eq. F-norm-basic with the batch's reduced gradients as samples) and grad_sq[i] = K_ii = ||G_i||^2.
 * Device pointers, either output may be NULL. */
isopo_status isopo_gram_norms(const float* K, int32_t n_seq, float* fisher_sq, float* grad_sq, void* stream);

/* Generalised re-scaling (alternative re-scalings listing):
 *     rel_F_norm = F_norm / ||G||
 *     c_i = A_i * reg2(F_norm_i)^p * reg2(||G_i||)^q * reg2(rel_F_norm_i)^r
 *     reg2(val) = sqrt(val^2 + regularization * E[val^2] + 1e-8)
 * p = -1 (q = r = 0): the KL-bounding re-scaling; r = -2: the multiple of G_i closest to the natural
 * gradient in the Fisher metric; q = -1, r = -2: the headline experiment's setting.
 *   fisher_sq      device [n_seq], F_norm^2 (from isopo_gram_norms or isopo_fisher_samples)
 *   grad_sq        device, ||G_i||^2 at grad_sq[i * grad_sq_stride] (pass K with stride n_seq + 1 to
 *                  read its diagonal in place)
 *   reg[3]         host: regularisation factors for (F_norm, ||G||, rel_F_norm), each >= 0
 *   expectation[3] host: E[val^2] for the same three, e.g. the caller's trailing mean over
 *                  minibatches; a negative entry means "this batch's mean"
 *   batch_means    optional device [3]: this batch's means of F^2, ||G||^2, rel^2, for the caller's
 *                  trailing mean
 * A sequence with ||G_i|| = 0 takes rel_F_norm = 0; its c_i is finite and multiplies a zero gradient. */
typedef struct isopo_rescale_params {
  float p, q, r;
  float reg[3];
  float expectation[3];
} isopo_rescale_params;
isopo_status isopo_rescale(const float* fisher_sq, const float* grad_sq, int64_t grad_sq_stride, int32_t n_seq,
                           const float* A, const isopo_rescale_params* params, float* c, float* batch_means,
                           void* stream);

/* Eigendecomposition of the layers' Gram matrices (interacting listing: D, U = eigh(ntk)), so that a
 * sweep over regularisers costs one decomposition.  `batch` independent problems laid out back to back
 * (the projections of a block), one workgroup each, in fp64: cyclic Jacobi in LDS up to 94 sequences,
 * Householder tridiagonalisation and implicit QL in the workspace from 95.
 *   K     device fp32 [batch, n_seq, n_seq], symmetric (the mean of K and K^T is decomposed)
 *   D     device fp64 [batch, n_seq], ascending
 *   U     device fp64 [batch, n_seq, n_seq] row-major, eigenvectors as columns: K = U diag(D) U^T
 *   info  optional device int32 [batch]: 0 converged, 1 not converged within the iteration limit (40 Jacobi
 *         sweeps, 60 QL steps per eigenvalue; a K with NaN or infinite entries ends there)
 *   workspace  device, isopo_ntk_eigh_workspace(n_seq, batch) bytes, 256-byte aligned (the work matrices
 *              of problems with 95 sequences and more) */
size_t isopo_ntk_eigh_workspace(int32_t n_seq, int32_t batch);
isopo_status isopo_ntk_eigh(const float* K, int32_t n_seq, int32_t batch, double* D, double* U, int32_t* info,
                            void* workspace, size_t ws_bytes, void* stream);

/* c_l = U ((U^T A) / (D + reg_l)) for l < n_lambda (interacting listing: preconditioner and
 * advantages_preconditioned), all from one decomposition, for each of `batch` problems
 * (D [batch, n_seq], U [batch, n_seq, n_seq], A [batch, n_seq]).
 *   lambdas    host [n_lambda], 1 <= n_lambda <= ISOPO_MAX_LAMBDAS, each >= 0
 *   reg_mode   ABSOLUTE: reg_l = lambda_l.  REL_TRACE: reg_l = lambda_l * mean(D).
 *              EMA_TRACE: reg_l = lambda_l * E[mean(D)], the trailing mean over minibatches (this one
 *              included) kept in ema_state and updated by this call:
 *              E <- mean(D) on the first call, E <- decay E + (1 - decay) mean(D) after
 *   ema_state  device float [batch, 2] {E, number of minibatches seen} per problem; zero it before the
 *              first minibatch; required for EMA_TRACE, ignored otherwise
 *   c          device fp32 [batch, n_lambda, n_seq]
 *   info       optional device int32 [batch]: number of (lambda, eigenvalue) pairs with D + reg <= 0;
 *              those components are left out of c (0 for a positive definite K + reg I) */
#define ISOPO_MAX_LAMBDAS 16
isopo_status isopo_transform_eigh(const double* D, const double* U, int32_t n_seq, int32_t batch, const float* A,
                                  const float* lambdas, int32_t n_lambda, isopo_reg_mode reg_mode, float* ema_state,
                                  float ema_decay, float* c, int32_t* info, void* stream);

/* dst[t, :] = c[seq(t)] * src[t, :] for a token-major matrix [n_tokens, d] (X or Delta), rounded to
 * the storage type; dst may not alias src.  Since Delta^T diag(c_tok) X = (diag(c_tok) Delta)^T X =
 * Delta^T (diag(c_tok) X), scaling the narrower operand once and then calling isopo_weighted_grad with
 * c = NULL gives the weighted update (`grad += advantages[i] * scale_i * seq_logprob_grad`) from a
 * scaled copy; the scaled rows are rounded to the storage type once.  isopo_weighted_grad(c != NULL) needs
 * no such copy. */
isopo_status isopo_scale_rows(const void* src, isopo_dtype dtype, int64_t n_tokens, int32_t d,
                              const int32_t* seq_offsets_dev, int32_t n_seq, const float* c, void* dst,
                              void* stream);

/* The weighted update from X and Delta (no stash) in two launches: isopo_scale_rows on the narrower of
 * X and Delta into `scratch`, then the unweighted contraction on the scaled copy:
 *     dW = beta dW + Delta^T diag(c_tok) X      (`grad += advantages[i] * scale_i * seq_logprob_grad`).
 * For callers that have no stash (coefficients from isopo_fisher_samples, or a workspace too small to
 * keep one).  scratch: device, 16-byte aligned, isopo_weighted_grad_scratch(layer) bytes
 * (n_tokens * min(d_in, d_out) elements of the input dtype). */
size_t isopo_weighted_grad_scratch(const isopo_layer* layer);
isopo_status isopo_weighted_grad_prescaled(const isopo_layer* layer, const float* c, float beta, float* dW,
                                           void* scratch, size_t scratch_bytes, void* stream);

/* Diagnostic, not a step of the method: a loop of nothing but bf16 matrix-core instructions on operands held
 * in registers, one wave per SIMD with 256 accumulator registers per lane (the register shape of the
 * contraction behind isopo_layer_gram).  The benchmark times it on random and on zero operands to find the
 * rate the board sustains at its power limit, against which the contraction's own rate is to be read.
 *   shape     32: v_mfma_f32_32x32x16_bf16, 16: v_mfma_f32_16x16x32_bf16
 *   operands  device, ISOPO_PROBE_THREADS * 256 bytes, 16-byte aligned (16 vectors of 8 bf16 per thread)
 *   sink      device float [ISOPO_PROBE_THREADS], overwritten
 *   iters     trips; each is 2 * 128 * 128 * 32 flop per wave, ISOPO_PROBE_THREADS / 64 waves */
#define ISOPO_PROBE_THREADS (256 * 256)
isopo_status isopo_probe_mfma_loop(int32_t shape, const void* operands, float* sink, int32_t iters, void* stream);

/* Diagnostic: the rate at which workgroups stream global memory into LDS with the 16-byte-per-lane DMA loads
 * of the contraction kernels, against the number of waves that issue them.  Every workgroup keeps a ring of
 * `stages` stages of 32 KiB filled (it waits for a stage, meets, requests the next) for `iters` stages and
 * computes nothing; workgroup b walks the (b mod 8)-th eighth of buf round and round.
 *   buf         device, 16-byte aligned, `bytes` a multiple of 8 * 32768 (16 MiB stays in the L2s)
 *   waves       2, 4, 8 or 16 per workgroup;  stages 2 or 4;  workgroups 1 .. 4096 (256: one per compute unit)
 *   sink        device float [workgroups], overwritten
 * Bytes moved: workgroups * iters * 32768. */
isopo_status isopo_probe_lds_dma(const void* buf, size_t bytes, int32_t waves, int32_t stages, int32_t workgroups,
                                 int32_t iters, float* sink, void* stream);

/* Diagnostic: dW [d_out, d_in] fp32 = Delta^T X (isopo_weighted_grad with c = NULL, stash = NULL, beta = 0) by
 * the matrix-core contraction on its 256 x 256 tile with 4 waves per workgroup (a 2 x 2 arrangement of
 * 128 x 128 wave tiles, one wave per SIMD, 256 accumulators per lane: what the per-sequence launch behind
 * isopo_layer_gram uses) or with 8 (2 x 4, 128 x 64 wave tiles, two waves per SIMD, twice as many waves issuing
 * the operand loads: what isopo_weighted_grad launches for the sums over all tokens).  Same result; the
 * benchmark times both on the workload and on zero operands.  bf16 layers whose launch plan takes the
 * 256 x 256 tile (isopo_contraction_plan), else ISOPO_ERR_UNSUPPORTED. */
isopo_status isopo_probe_contraction_waves(const isopo_layer* layer, int32_t waves, float* dW, void* stream);

const char* isopo_status_string(isopo_status s);

/* Library version, "major.minor". */
const char* isopo_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ISOPO_H */
