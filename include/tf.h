/*
 * tf.h - C ABI of the freeze-aware stage-backward library for MI355X (gfx950).
 *
 * The library computes what TimelyFreeze's per-stage freeze ratios speed up
 * (TimelyFreeze, arxiv 2602.05754):
 *   - the backward of a pipeline stage's linear layers, split as in Sec. 3.2.1
 *     into the input-gradient part (always computed) and the parameter-gradient
 *     part (computed only for tensors that are not frozen);
 *   - the masked parameter update of App. D.1 (mask convention: 1 = frozen =
 *     no update; update rule Delta_t = (1/M) sum_m U_{t,m} (.) g_{t,m}) with
 *     the AdamW optimizer named in Table exp_setup;
 *   - the APF stability recurrences and score of Sec. 2.3.
 * To those three the freeze ratio r and the freeze masks are inputs.  The steps
 * that produce them are offered beside the hot path: the metric-aware selection
 * statistics (APF scores, AutoFreeze norms, the budget reconciliation of Alg. 2,
 * row-block draws) and, host only, the schedule DAG, its longest paths and the
 * linear program of Sec. 3.2 that turns measured action times into ratios.
 *
 * General conventions
 *   - Every function returns an int: TF_OK (0) or a negative tf_status.
 *     Nothing throws, aborts or prints.
 *   - "host" / "device" on a pointer says where the memory it points to lives.
 *     Arrays of pointers (W, X, dY, ...) are HOST arrays whose entries are
 *     DEVICE pointers.  Host arrays are consumed before the call returns.
 *   - The caller owns every device buffer and the stream.  The library keeps no
 *     caller pointer after a call returns.  Calls only enqueue work on
 *     `hip_stream` (a hipStream_t passed as void*, NULL = the default stream);
 *     they never synchronise the device.  Outputs are valid once the caller
 *     has synchronised the stream.
 *   - All argument validation happens before the first HIP call of a function,
 *     so argument errors are reported identically on a machine without a GPU.
 *   - Device pointers must be 16-byte aligned (TF_ERR_ALIGN otherwise).
 *   - Inputs may alias each other (q/k/v may share one X).  An output must not
 *     overlap any input or any other output of the same call, with one
 *     exception: the members of an input group of tf_stage_backward_shared pass
 *     the same dX pointer.  The stage-backward entry points check this on the
 *     host (byte ranges from the shapes) and return TF_ERR_ALIAS.
 *   - A tf_ctx serves one stream at a time and is not re-entrant.
 *   - Matrices are dense row-major with no padding.  A linear layer l has
 *     K_l input features and N_l output features, forward Y_l = X_l W_l with
 *     W_l stored [K_l x N_l]; X_l is [T x K_l], dY_l is [T x N_l], T = tokens
 *     in the microbatch.
 */
#ifndef TF_H_
#define TF_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tf_ctx tf_ctx;                    /* opaque */

typedef enum { TF_F32 = 0, TF_BF16 = 1 } tf_dtype;

typedef struct { int64_t K, N; } tf_shape;       /* in_features, out_features */

typedef enum {
    TF_OK              =  0,
    TF_ERR_INVALID_ARG = -1,   /* NULL where a pointer is required, negative count, bad scalar */
    TF_ERR_SHAPE       = -2,   /* non-positive K/N/T/numel, or a size the kernels cannot index */
    TF_ERR_DTYPE       = -3,   /* unknown dtype or an unsupported combination */
    TF_ERR_ALIGN       = -4,   /* a device pointer is not 16-byte aligned */
    TF_ERR_WORKSPACE   = -5,   /* internal staging could not be allocated */
    TF_ERR_HIP         = -6,   /* a HIP call failed; see tf_last_hip_error */
    TF_ERR_NO_DEVICE   = -7,   /* tf_create: no usable gfx950 device with that id */
    TF_ERR_ALIAS       = -8    /* an output overlaps an input or another output of the call */
} tf_status;

/* Create / destroy a context bound to HIP device `device_id`.  tf_create makes
 * that device current for the calling thread and queries its properties; it
 * fails with TF_ERR_NO_DEVICE when there is no such device.  The context owns
 * its host-side bookkeeping (timing events) and two small device allocations, made
 * here: the 8.2 KB rank-search state of tf_reconcile_mask and 128 KB of partial
 * sums for tf_masked_adamw / tf_stability_update / tf_autofreeze_norms
 * (TF_ERR_WORKSPACE if either fails).  No call allocates device memory afterwards.  Every later call on the
 * context makes device_id current for the calling thread before it launches. */
int tf_create(tf_ctx** out, int device_id);
int tf_destroy(tf_ctx* ctx);

/* Static, never-NULL description of a status code. */
const char* tf_strerror(int code);

/* Raw hipError_t of the most recent TF_ERR_HIP on this context (0 if none). */
int tf_last_hip_error(const tf_ctx* ctx);

/*
 * Optional per-kernel timing (the analogue of the paper's monitoring of action
 * times, Sec. 3.1, at kernel granularity).  While enabled, every kernel the
 * library launches is bracketed by a HIP event pair recorded on the launch
 * stream.  tf_profile_collect waits for the recorded events, writes up to
 * `capacity` (kind, milliseconds) pairs in launch order into the HOST arrays
 * `kinds` and `ms`, stores the count in *n_out and forgets all records.
 * Disabled by default; costs nothing when disabled.
 */
typedef enum {
    TF_KERNEL_DX_MFMA = 0,      /* input-gradient GEMMs on the matrix cores   */
    TF_KERNEL_DW_MFMA = 1,      /* weight-gradient GEMMs on the matrix cores  */
    TF_KERNEL_DX_GENERIC = 2,   /* input-gradient GEMMs, fp32-FMA kernel      */
    TF_KERNEL_DW_GENERIC = 3,   /* weight-gradient GEMMs, fp32-FMA kernel     */
    TF_KERNEL_ADAMW = 4,        /* fused masked AdamW (+ stability EMAs)      */
    TF_KERNEL_STABILITY = 5,    /* stand-alone stability update               */
    TF_KERNEL_AUTOFREEZE = 6,   /* norms of the cumulative updates            */
    TF_KERNEL_RECONCILE = 7     /* every kernel of tf_reconcile_mask          */
} tf_kernel_kind;
int tf_profile_enable(tf_ctx* ctx, int enable);
int tf_profile_collect(tf_ctx* ctx, int32_t capacity, int32_t* kinds, float* ms, int32_t* n_out);

/* Library version, "major.minor.patch". */
const char* tf_version(void);

/*
 * Freeze-aware backward of n_layers independent linear layers (Sec. 3.2.1:
 * activation-gradient component always runs, parameter-gradient component
 * shrinks with the freeze ratio; App. D.1: mask value 1 = frozen).
 *
 *   for every l:                     dX_l = dY_l * W_l^T          [T x K_l]
 *   for every l, freeze_mask[l]==0:  dW_l  = X_l^T * dY_l         [K_l x N_l]   (accumulate == 0)
 *                                    dW_l += X_l^T * dY_l                       (accumulate == 1)
 *   for every l, freeze_mask[l]==1:  dW_l is neither read nor written; dW[l]
 *                                    and X[l] may be NULL.
 *
 *   shapes       host, n_layers entries.
 *   io_dtype     element type of W, X, dY and dX (TF_F32 or TF_BF16).
 *   W, X, dY     host arrays of n_layers device pointers (read only).
 *   freeze_mask  host, n_layers bytes, or NULL (= nothing frozen).
 *   dX           host array of n_layers device pointers, written for all l.
 *   dW           host array of n_layers device pointers; dw_dtype is its element
 *                type.  accumulate == 1 sums over the microbatches of a step
 *                (the 1/M of the update rule is applied by tf_masked_adamw's
 *                grad_scale) and requires dw_dtype == TF_F32.
 *   Products accumulate in fp32; bf16 outputs are rounded to nearest even once.
 *   n_layers == 0 is a no-op.  With io_dtype TF_F32 the arithmetic is true fp32.
 */
int tf_stage_backward(tf_ctx* ctx, void* hip_stream,
                      int32_t n_layers, const tf_shape* shapes,
                      int64_t T, tf_dtype io_dtype,
                      const void* const* W, const void* const* X, const void* const* dY,
                      const uint8_t* freeze_mask,
                      void* const* dX,
                      void* const* dW, tf_dtype dw_dtype,
                      int accumulate);

/*
 * One microbatch of a step in which every microbatch has its own freeze mask
 * (App. D.1, update rule: Delta_t = (1/M) sum_m U_{t,m} (.) g_{t,m}, the sum running
 * over the microbatches in which a parameter is not frozen).  As
 * tf_stage_backward, but whether a weight gradient is added to dW_l or
 * overwrites it is said layer by layer:
 *
 *   for every l:                                           dX_l = dY_l * W_l^T
 *   freeze_mask[l]==0 and accumulate_mask[l]==0:           dW_l  = X_l^T * dY_l
 *   freeze_mask[l]==0 and accumulate_mask[l]==1:           dW_l += X_l^T * dY_l
 *   freeze_mask[l]==1:                                     dW_l untouched
 *
 *   accumulate_mask  host, n_layers bytes (0 or 1), required.  The caller sets
 *                    entry l to 0 in the first microbatch of the step in which
 *                    layer l is not frozen and to 1 afterwards: the accumulators
 *                    then need no clearing between steps and the first product
 *                    of a step is written without the old values being read.
 *                    Entries of frozen layers are ignored.
 *   dw_dtype         TF_F32 as soon as one unfrozen layer adds (TF_ERR_DTYPE
 *                    otherwise).
 * Everything else, errors included, as tf_stage_backward.  The layers that add
 * and the layers that overwrite go to separate launches.
 */
int tf_stage_backward_microbatch(tf_ctx* ctx, void* hip_stream,
                                 int32_t n_layers, const tf_shape* shapes,
                                 int64_t T, tf_dtype io_dtype,
                                 const void* const* W, const void* const* X, const void* const* dY,
                                 const uint8_t* freeze_mask,
                                 void* const* dX,
                                 void* const* dW, tf_dtype dw_dtype,
                                 const uint8_t* accumulate_mask);

/*
 * Host-only bookkeeping for such a step (App. D.1, update rule).  freeze_masks
 * is host memory, n_microbatches rows of n_layers bytes (row m = the mask of
 * microbatch m, 1 = frozen).  Outputs, host memory:
 *   accumulate_masks  n_microbatches x n_layers: the accumulate_mask of call m
 *                     (1 where layer l was unfrozen in an earlier microbatch);
 *   step_freeze_mask  n_layers: 1 where layer l was frozen in EVERY microbatch -
 *                     the tensor_freeze_mask of the step's tf_masked_adamw call
 *                     (its grad_scale is 1 / n_microbatches whatever the masks).
 * TF_ERR_INVALID_ARG for NULL pointers, negative sizes or mask bytes above 1.
 */
int tf_microbatch_plan(int32_t n_microbatches, int32_t n_layers, const uint8_t* freeze_masks,
                       uint8_t* accumulate_masks, uint8_t* step_freeze_mask);

/*
 * Masked AdamW step over n_tensors tensors, optionally fused with the APF
 * stability recurrences (App. D.1 update rule with U = 1 - I; optimizer from
 * Table exp_setup; Sec. 2.3 for E, E^abs).  For every element j of tensor i that
 * is NOT frozen, with t = step[i] and g = grad_scale * grad_j:
 *     m <- beta1 m + (1-beta1) g          v <- beta2 v + (1-beta2) g^2
 *     u  = -lr*wd*p - lr * (m/(1-beta1^t)) / (sqrt(v/(1-beta2^t)) + eps)
 *     p <- p + u                          p_lowp <- bf16_rne(p)
 *     E <- a E + (1-a) u                  A <- a A + (1-a) |u|        (a = ema_decay)
 * A frozen element (tensor_freeze_mask[i] == 1, or its bit set in
 * elem_freeze_bits[i]) keeps every one of p, m, v, p_lowp, E, A bit-identical;
 * a frozen tensor's buffers are not even read.
 *
 *   numel               host, n_tensors element counts (> 0).
 *   p_master, m, v      host arrays of device pointers to fp32 buffers (read/write).
 *   grad, grad_dtype    host array of device pointers, TF_BF16 or TF_F32 (read only).
 *   p_lowp              NULL, or host array of device pointers to bf16 buffers
 *                       (entries may be NULL individually).
 *   tensor_freeze_mask  NULL or host, n_tensors bytes, 1 = skip the tensor.
 *   elem_freeze_bits    NULL, or host array whose entries are NULL or device
 *                       pointers to ceil(numel/32) uint32 words; element j is
 *                       bit (j & 31) of word (j >> 5), 1 = frozen.
 *   step                host, n_tensors ints >= 1: the bias-correction exponent
 *                       of each tensor (the caller advances it only for tensors
 *                       it updates).
 *   ema, ema_abs        both NULL (stability off) or both host arrays of device
 *                       pointers to fp32 buffers.
 *   score_sums          NULL or device, 2*n_tensors doubles: on return
 *                       score_sums[2i] = sum_j |E_j| and score_sums[2i+1] =
 *                       sum_j A_j over ALL elements of tensor i (frozen elements
 *                       contribute their unchanged values).  Entries of frozen
 *                       tensors are left as they were.  Requires ema/ema_abs.
 *   Arithmetic is fp32; sums are accumulated in fp64.
 *   numel[i] <= 2^37 (TF_ERR_SHAPE beyond).
 *
 * Element masks are applied per mask word (32 elements, one 128-byte line of each
 * fp32 buffer): a word of all ones is skipped altogether; in any other word the
 * frozen elements are written back with the bits that were read, and their stored
 * bf16 copy is read in order to be written back unchanged.
 *
 * tf_assume_lowp_is_rounded_master(ctx, 1): the caller promises that on entry to
 * every later tf_masked_adamw on this context p_lowp[i][j] == bf16_rne(p_master[i][j])
 * for all elements (true whenever the copies were produced by this function, or by
 * rounding the master weights, and not changed since).  Frozen elements of a partly
 * frozen word then get their copy from the unchanged p instead of a second read:
 * the same bits under the promise, 2 bytes per element less traffic.  Off by default.
 */
int tf_assume_lowp_is_rounded_master(tf_ctx* ctx, int on);
int tf_masked_adamw(tf_ctx* ctx, void* hip_stream,
                    int32_t n_tensors, const int64_t* numel,
                    void* const* p_master, void* const* m, void* const* v,
                    const void* const* grad, tf_dtype grad_dtype, float grad_scale,
                    void* const* p_lowp,
                    const uint8_t* tensor_freeze_mask,
                    const uint32_t* const* elem_freeze_bits,
                    const int32_t* step,
                    float lr, float beta1, float beta2, float eps, float weight_decay,
                    void* const* ema, void* const* ema_abs, float ema_decay,
                    double* score_sums);

/*
 * Stand-alone APF stability update (Sec. 2.3) for stability checks that are
 * more than one optimizer step apart: Delta is given explicitly.
 *     E <- a E + (1-a) Delta      A <- a A + (1-a) |Delta|     on unfrozen elements
 * Arguments as in tf_masked_adamw; delta entries are device fp32 buffers.
 */
int tf_stability_update(tf_ctx* ctx, void* hip_stream,
                        int32_t n_tensors, const int64_t* numel,
                        const void* const* delta,
                        void* const* ema, void* const* ema_abs, float ema_decay,
                        const uint8_t* tensor_freeze_mask,
                        const uint32_t* const* elem_freeze_bits,
                        double* score_sums);

/*
 * Host-only helpers for the score -> mask step (Sec. 2.3: low score = stable).
 *
 * tf_stability_scores: scores[i] = score_sums[2i] / score_sums[2i+1], or 1 when
 * the denominator is 0 (never updated: not evidence of stability).  Both
 * arrays are HOST memory (copy score_sums back first).
 *
 * tf_select_lowest: out_mask[i] = 1 for the n_freeze tensors with the lowest
 * score, ordered by (score ascending, index ascending); 0 elsewhere.
 * TF_ERR_INVALID_ARG if n_freeze is outside [0, n] or a score is NaN.
 *
 * tf_num_frozen: number of tensors frozen at ratio r out of n: ceil(r*n),
 * computed so that r*n a rounding error above an integer does not round up;
 * clamped to [0, n].
 */
int tf_stability_scores(const double* score_sums, int32_t n, double* scores);
int tf_select_lowest(const double* scores, int32_t n, int32_t n_freeze, uint8_t* out_mask);
int32_t tf_num_frozen(double r, int32_t n);

/*
 * Sub-tensor freezing (Sec. 3.2.1: the parameter-gradient time shrinks with the
 * fraction of parameters frozen; Alg. 1: a random subset I_i of the stage's
 * parameters with |I_i| = AFR |P_s| in expectation).  The unit is a block of
 * block_rows consecutive rows of a weight tensor W_l [K_l x N_l] (rows = input
 * features), so that the frozen fraction of the parameters follows the freeze
 * ratio to within one block instead of one tensor.
 *
 * tf_stage_backward_blocks: as tf_stage_backward, and in addition, for a layer l
 * with freeze_mask[l] == 0 and row_block_mask[l] != NULL, only the row blocks b
 * with row_block_mask[l][b] == 0 are computed:
 *     dW_l[b*block_rows .. (b+1)*block_rows) (+)= X_l[:, those columns]^T * dY_l
 * Rows of frozen blocks of dW_l are neither read nor written; dX is always
 * computed in full.  Runs of unfrozen blocks are single GEMM problems; on the
 * matrix cores when the run has a multiple of 256 rows (and N_l % 256 == 0,
 * T % 64 == 0, bf16 inputs), otherwise on the fp32-FMA kernel.
 *   row_block_mask   host array of n_layers HOST pointers (entries may be NULL: layer
 *                    without row mask), each K_l / block_rows bytes, 1 = frozen; or NULL
 *   block_rows       > 0; must divide K_l of every layer that has a row mask
 * Errors as tf_stage_backward, plus TF_ERR_SHAPE when block_rows does not divide K_l.
 *
 * tf_select_row_blocks (host only): seeded draw of row blocks whose parameters add
 * up to at most floor(r * P).  Units are numbered layer by layer, block by block;
 * they are visited in the order of the keys perm32(unit number, seed) (the keyed
 * permutation described at tf_reconcile_mask) and frozen if they still fit into
 * what is left of the budget.  masks: sum_l K_l / block_rows bytes, layer after
 * layer; frozen_params (optional): parameters frozen.
 *
 * tf_row_blocks_to_bits: element masks (the elem_freeze_bits of tf_masked_adamw)
 * of row-block masks: bit j of elem_bits[l] = row_block_mask[l][(j / N_l) / block_rows],
 * all zero for a layer without row mask.  elem_bits: host array of n_layers DEVICE
 * pointers, ceil(K_l N_l / 32) words each, written.  block_rows * N_l must be a
 * multiple of 32 for layers with a row mask (TF_ERR_SHAPE).  Only enqueues.
 */
int tf_stage_backward_blocks(tf_ctx* ctx, void* hip_stream,
                             int32_t n_layers, const tf_shape* shapes,
                             int64_t T, tf_dtype io_dtype,
                             const void* const* W, const void* const* X, const void* const* dY,
                             const uint8_t* freeze_mask,
                             const uint8_t* const* row_block_mask, int32_t block_rows,
                             void* const* dX,
                             void* const* dW, tf_dtype dw_dtype,
                             int accumulate);
/*
 * Layers that share their input (in a transformer block q, k, v read the same
 * activations, gate and up too): the gradient with respect to that input is the
 * sum of the members' products,
 *     dX_g = sum over l with input_group[l] == g of  dY_l * W_l^T,
 * i.e. the product with the members' weights concatenated along the output
 * features.  tf_stage_backward_shared is tf_stage_backward_blocks plus
 *   input_group   host, n_layers, or NULL: -1 = a layer of its own; g >= 0 = member of group g
 *                 (g < n_layers).  Members must have the same K_l and pass the SAME dX pointer;
 *                 the sum is formed in the fp32 accumulators and rounded once.
 * On the matrix cores the members are contraction segments of one problem (bf16, shapes as
 * for tf_stage_backward); an fp32 stage falls back to one launch per member adding onto the
 * previous one; a bf16 group with shapes the matrix-core kernel cannot take is TF_ERR_SHAPE.
 * dW is per layer as before (each member has its own X pointer; they may be equal).
 */
int tf_stage_backward_shared(tf_ctx* ctx, void* hip_stream,
                             int32_t n_layers, const tf_shape* shapes,
                             int64_t T, tf_dtype io_dtype,
                             const void* const* W, const void* const* X, const void* const* dY,
                             const uint8_t* freeze_mask,
                             const uint8_t* const* row_block_mask, int32_t block_rows,
                             const int32_t* input_group,
                             void* const* dX,
                             void* const* dW, tf_dtype dw_dtype,
                             int accumulate);
int tf_select_row_blocks(int32_t n_layers, const tf_shape* shapes, int32_t block_rows,
                         double r, uint64_t seed, uint8_t* masks, int64_t* frozen_params);
int tf_row_blocks_to_bits(tf_ctx* ctx, void* hip_stream,
                          int32_t n_layers, const tf_shape* shapes,
                          const uint8_t* const* row_block_mask, int32_t block_rows,
                          uint32_t* const* elem_bits);

/*
 * AutoFreeze stability statistic (Sec. 2.3, "AutoFreeze"): the score of a layer
 * at the K-th check is | ||D_{K-1}|| - ||D_K|| | / ||D_{K-1}|| with D_K the
 * cumulative parameter update since the previous check, D_K = p_now - snapshot.
 *
 * tf_autofreeze_norms, per tensor i with tensor_freeze_mask[i] == 0 (or no mask):
 *     sq_norms[i] = sum_j (p_master[i][j] - snapshot[i][j])^2      (fp64 sum)
 *     snapshot[i] <- p_master[i]                  if update_snapshot != 0
 * Tensors with mask 1 are skipped: sq_norms[i] and snapshot[i] stay as they are.
 * Call it once per stability check; nothing is paid between checks.
 *
 *   numel            host, n_tensors
 *   p_master_f32     host array of n_tensors DEVICE pointers, fp32, read only
 *   snapshot_f32     host array of n_tensors DEVICE pointers, fp32, read (and written)
 *   sq_norms         DEVICE, n_tensors doubles, 8-byte aligned; valid after the stream is synchronised
 * Errors as for tf_masked_adamw.  Only enqueues.
 *
 * tf_autofreeze_scores (host only): scores[i] from sq_prev[i], sq_cur[i] (the
 * squared norms of two consecutive checks); a zero previous norm gives 0 if
 * the current one is zero too and +infinity otherwise.
 *
 * tf_autofreeze_select (host only): layers [0, n_already_frozen) are frozen.
 * The threshold is the nearest-rank `percentile`-th percentile (P_Auto, Table
 * exp_setup: 80) of the scores of the layers still trained; from the first
 * trained layer on, layers are frozen while their score does not exceed it
 * (a layer is frozen only if all layers before it are).  out_mask[i] = 1 frozen.
 * TF_ERR_INVALID_ARG for NaN scores, percentile outside [0, 100] or
 * n_already_frozen outside [0, n].
 */
int tf_autofreeze_norms(tf_ctx* ctx, void* hip_stream,
                        int32_t n_tensors, const int64_t* numel,
                        const void* const* p_master_f32, void* const* snapshot_f32,
                        const uint8_t* tensor_freeze_mask, int update_snapshot,
                        double* sq_norms);
int tf_autofreeze_scores(const double* sq_prev, const double* sq_cur, int32_t n, double* scores);
int tf_autofreeze_select(const double* scores, int32_t n, int32_t n_already_frozen,
                         double percentile, uint8_t* out_mask);

/*
 * Metric-aware parameter selection of the hybrid variants (App. "Hybrid
 * Variants Algorithm", Alg. 2): bring a base element mask over the N_s
 * parameters of a stage to exactly n_freeze = floor(r N_s) ones.
 *
 *   ||base||_1 == n_freeze : the mask is left as it is
 *   ||base||_1 <  n_freeze : n_freeze - ||base||_1 of its zeros, drawn uniformly, become ones
 *   ||base||_1 >  n_freeze : ||base||_1 - n_freeze of its ones, drawn uniformly, become zeros
 *
 * The tensors are taken as one index space, concatenated in the order given.
 * Drawing: candidates are ranked by the image of their stage-wide index under
 * a permutation of [0, 2^32) keyed by `seed` (6-round Feistel network on 16-bit
 * halves; round function: top 16 bits of ((half ^ key) + 1) * 0x9E3779B1 mod
 * 2^32; round keys: the four 16-bit pieces of seed, low first, then bits 32..47
 * and 48..63 of seed * 0xD1342543DE82EF95 mod 2^64) and the lowest ranks are
 * drawn, so the result is a function of (mask, n_freeze, seed) alone.
 *
 *   numel            host, n_tensors; sum < 2^32
 *   elem_bits        host array of n_tensors DEVICE pointers; bit j & 31 of word j >> 5
 *                    is element j, 1 = frozen; updated in place; bits past numel are kept
 *   n_freeze         0 <= n_freeze <= sum(numel)
 *   stats            optional DEVICE, 3 x int64, 8-byte aligned: {||base||_1, case (0 kept,
 *                    1 added, 2 removed), largest key drawn}; valid after the stream is synchronised
 * Only enqueues (the rank search runs on the device).  Uses device memory owned by the
 * context: calls on one context must not overlap.
 * Errors: TF_ERR_INVALID_ARG, TF_ERR_SHAPE (numel <= 0, sum >= 2^32), TF_ERR_ALIGN
 * (mask pointers not 4-byte, stats not 8-byte aligned), TF_ERR_HIP.
 */
int tf_reconcile_mask(tf_ctx* ctx, void* hip_stream,
                      int32_t n_tensors, const int64_t* numel,
                      uint32_t* const* elem_bits,
                      int64_t n_freeze, uint64_t seed,
                      int64_t* stats);

/*
 * tf_reconcile_mask for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result, bit for bit.
 * The call allocates nothing, on the device or on the host, and creates no events (it is not
 * timed by tf_profile_*): its rank-search state lives in a static device array of 8448 bytes
 * that is part of the library's code object, one copy per GPU, held until the process ends;
 * tf_create looks up its address on the context's device.  Limit: as tf_reconcile_mask,
 * sum(numel) < 2^32 (TF_ERR_SHAPE beyond).  Every call on one GPU, from whatever context or
 * stream, uses that GPU's one array: the call clears it first with a kernel, and calls that
 * overlap in time on one GPU race.
 */
int tf_reconcile_mask_static(tf_ctx* ctx, void* hip_stream,
                             int32_t n_tensors, const int64_t* numel,
                             uint32_t* const* elem_bits,
                             int64_t n_freeze, uint64_t seed,
                             int64_t* stats);

/*
 * From measured action times to freeze ratios (Sec. 3.2), host only.
 *
 * Nodes: action (a, m, s) - a = 0 forward / 1 backward, microbatch m in [0, M),
 * stage s in [0, S) - has id (a M + m) S + s; the source node is 2 M S, the
 * destination 2 M S + 1 (both of duration 0).
 *
 * tf_pipeline_dag: the edges of one batch's schedule (App. "Edge Construction
 * Rules"): source -> f(0,0) and b(M-1,0) -> destination; within a stage the
 * microbatch order of forwards and of backwards and forward before its
 * backward; forward s -> s+1 and backward s+1 -> s of the same microbatch; and
 * the order in which a rank runs its actions - GPipe: all forwards, then all
 * backwards; 1F1B: min(M, S-1-s) forwards, then one forward / one backward in
 * turn, then the remaining backwards.  These two keep one stage per rank.
 * Interleaved 1F1B and ZBV (Sec. 4.2 "Pipeline Schedules") place TWO stages on
 * each of R = S / 2 ranks (S even, TF_ERR_SHAPE otherwise), and a rank's chain
 * of edges runs through the actions of both:
 *   interleaved 1F1B - rank r owns stages r and r + R; it takes g = M / max(1,
 *     M div R) microbatches per visit of a stage (M must be a multiple of
 *     max(1, M div R), TF_ERR_SHAPE otherwise), forwards from its first stage
 *     on, backwards from its last, runs g + 2 (R-1-r) forwards ahead, then
 *     alternates, then finishes the backwards;
 *   ZBV - rank r owns stages r and 2R-1-r (V-shaped placement) and follows the
 *     zero-bubble V schedule; that schedule splits a backward into an
 *     input-gradient and a weight-gradient pass, the DAG's backward node is
 *     both and stands where the input-gradient pass runs.
 * Writes min(capacity, *n_edges) pairs
 * (from, to), sorted, without duplicates; *n_edges is the full count.
 *
 * tf_dag_start_times: P_i = max over predecessors j of (P_j + w_j), 0 for nodes
 * without predecessor.  TF_ERR_INVALID_ARG for a graph with a cycle.
 *
 * tf_freeze_ratio_lp: the linear program of Sec. 3.2.2,
 *     min  P_d - lambda * sum_i delta_i w_i
 *     s.t. P_j >= P_i + w_i for every edge, w_min_i <= w_i <= w_max_i, P_source = 0,
 *          for every stage: mean over its freezable nodes of r_i <= r_max,
 * with delta_i = 1 / (w_max_i - w_min_i) (0 when the two are equal: not
 * freezable) and r_i = delta_i (w_max_i - w_i).  w_min / w_max: 2 M S measured
 * durations (all parameters frozen / none frozen).  Outputs (r required, the
 * others optional): r and w per action, P per node (2 M S + 2, the longest-path
 * start times at w), the batch time at w_max and at w.  The optimum's batch
 * time is unique, its r need not be; the solver (dense two-phase simplex,
 * Bland's rule) is deterministic.  S * M <= 4096.
 *
 * tf_actual_freeze_ratio: the progressive ratio of the freezing phase (Sec. 3.3):
 * 0 for t <= T_m, min(r, r (t - T_m) / (T_f - T_m)) after.
 */
typedef enum { TF_SCHEDULE_GPIPE = 0, TF_SCHEDULE_1F1B = 1, TF_SCHEDULE_INTERLEAVED_1F1B = 2, TF_SCHEDULE_ZBV = 3 } tf_schedule;
int tf_pipeline_dag(int32_t n_stages, int32_t n_microbatches, tf_schedule schedule,
                    int32_t capacity, int32_t* edges, int32_t* n_edges);
int tf_dag_start_times(int32_t n_nodes, int32_t n_edges, const int32_t* edges, const double* w, double* P);
int tf_freeze_ratio_lp(int32_t n_stages, int32_t n_microbatches, tf_schedule schedule,
                       const double* w_min, const double* w_max, double r_max, double lambda,
                       double* r, double* w, double* P, double* batch_time_max, double* batch_time);
double tf_actual_freeze_ratio(double r, int64_t t, int64_t T_m, int64_t T_f);

#ifdef __cplusplus
}
#endif
#endif /* TF_H_ */
