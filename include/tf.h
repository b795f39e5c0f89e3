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
 * The freeze ratio r and the freeze masks are inputs; the schedule DAG and the
 * linear program that produce r are not part of this library.
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
 *   - Inputs may alias each other (q/k/v may share one X).  Outputs must not
 *     alias anything else.
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
    TF_ERR_NO_DEVICE   = -7    /* tf_create: no usable gfx950 device with that id */
} tf_status;

/* Create / destroy a context bound to HIP device `device_id`.  tf_create makes
 * that device current for the calling thread and queries its properties; it
 * fails with TF_ERR_NO_DEVICE when there is no such device.  The context owns
 * only small internal bookkeeping; no per-call allocation happens later. */
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
    TF_KERNEL_STABILITY = 5     /* stand-alone stability update               */
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
 */
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

#ifdef __cplusplus
}
#endif
#endif /* TF_H_ */
