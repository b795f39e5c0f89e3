/*
 * TEST INFRASTRUCTURE - NOT PART OF THE PRODUCT.
 *
 * Plain, slow, fp64 CPU definitions of what the freeze-aware stage backward,
 * the masked AdamW step and the APF stability statistics compute.  Only tests,
 * the smoke check and the CPU-baseline leg of the benchmark may call this.
 * It shares no code with the HIP library and never includes its headers.
 *
 * Sources (TimelyFreeze, arxiv 2602.05754):
 *   - Sec. 3.2.1 "Node weight" paragraph after Fig. fwdbwd_ratio: a backward
 *     action = gradient w.r.t. input activations (always) + gradient w.r.t.
 *     parameters (the only part freezing removes).
 *   - App. D.1 "Freezing and Update Masks": I = 1 means frozen (no update),
 *     U = 1 - I; eq. (update_rule): Delta_t = (1/M) sum_m U_{t,m} (.) g_{t,m}.
 *   - Sec. 2.3 "APF": E_K = a E_{K-1} + (1-a) Delta_K,
 *     E^abs_K = a E^abs_{K-1} + (1-a)|Delta_K|, Score = |E_K| / E^abs_K.
 *   - Table exp_setup, Optimizer row: AdamW (no equations in the paper; the
 *     decoupled-weight-decay form of Loshchilov & Hutter with Adam's bias
 *     correction is used, eps added outside the square root).
 *
 * Every loop below is the definition written out: no blocking, no fusion,
 * no reordering.  OpenMP only splits independent output rows / elements.
 *
 * Parity pins (tests/test_oracle_*.py): central finite differences of the
 * bilinear form, adjoint identities, numpy matmul, outer-product / identity /
 * one-hot special cases, closed-form AdamW steps (first step, constant and
 * alternating gradients), closed-form EMAs, brute-force selection.
 * Paper-printed worked values for these operations: none exist.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------------- */
/* O1: stage backward of L independent linear layers Y_l = X_l W_l,       */
/*     W_l is [K_l x N_l] row-major, X_l [T x K_l], dY_l [T x N_l].       */
/* ---------------------------------------------------------------------- */

/* dX[t,k] = sum_n dY[t,n] * W[k,n]   (Sec. 3.2.1, component (1): always) */
static void input_grad(int64_t T, int64_t K, int64_t N,
                       const double *dY, const double *W, double *dX)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t k = 0; k < K; ++k) {
            double s = 0.0;
            for (int64_t n = 0; n < N; ++n)
                s += dY[t * N + n] * W[k * N + n];
            dX[t * K + k] = s;
        }
    }
}

/* G[k,n] = sum_t X[t,k] * dY[t,n]    (Sec. 3.2.1, component (2))
 * accumulate == 0: dW = G ; accumulate != 0: dW += G (sum over microbatches
 * of U (.) g, App. D.1 eq. update_rule; the 1/M lives in the optimizer). */
static int weight_grad(int64_t T, int64_t K, int64_t N,
                       const double *X, const double *dY, double *dW,
                       int accumulate)
{
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; ++k) {
        double *row = (double *)calloc((size_t)(N > 0 ? N : 1), sizeof(double));
        if (!row) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        for (int64_t t = 0; t < T; ++t) {
            const double x = X[t * K + k];
            for (int64_t n = 0; n < N; ++n)
                row[n] += x * dY[t * N + n];
        }
        for (int64_t n = 0; n < N; ++n) {
            if (accumulate)
                dW[k * N + n] += row[n];
            else
                dW[k * N + n] = row[n];
        }
        free(row);
    }
    return fail;
}

/* freeze_mask[l] == 1: tensor l frozen -> dW[l] is neither read nor written
 * (App. D.1: frozen = no update).  dX is produced for every layer. */
int oracle_stage_backward(int32_t n_layers, const int64_t *K, const int64_t *N,
                          int64_t T,
                          const double *const *W, const double *const *X,
                          const double *const *dY,
                          const uint8_t *freeze_mask,
                          double *const *dX, double *const *dW,
                          int accumulate)
{
    for (int32_t l = 0; l < n_layers; ++l) {
        input_grad(T, K[l], N[l], dY[l], W[l], dX[l]);
        if (freeze_mask && freeze_mask[l])
            continue;
        if (weight_grad(T, K[l], N[l], X[l], dY[l], dW[l], accumulate))
            return -1;
    }
    return 0;
}

/* ---------------------------------------------------------------------- */
/* bf16 round-to-nearest-even of a double, returned as a double.          */
/* bf16 = 1 sign, 8 exponent, 7 fraction bits; subnormals kept.           */
/* ---------------------------------------------------------------------- */
double oracle_bf16_rne(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x))
        return x;
    int e = ilogb(x);
    if (e < -126)
        e = -126;                       /* subnormal spacing 2^-133 */
    const double q = ldexp(1.0, e - 7); /* spacing of bf16 numbers near x */
    double r = nearbyint(x / q) * q;    /* default rounding mode: ties-to-even */
    if (fabs(r) >= ldexp(1.0, 128))
        r = copysign(INFINITY, x);
    return r;
}

/* ---------------------------------------------------------------------- */
/* O2 + O3: masked AdamW step with the APF EMAs of the applied update.    */
/* One tensor per call.                                                   */
/*   elem_frozen: NULL or numel bytes, 1 = frozen element (untouched).    */
/*   ema/ema_abs: both NULL (stability off) or both numel doubles.        */
/*   p_lowp: NULL or numel doubles receiving bf16_rne(p) for updated      */
/*           elements only.                                               */
/* ---------------------------------------------------------------------- */
int oracle_masked_adamw(int64_t numel,
                        double *p, double *m, double *v,
                        const double *grad, double grad_scale,
                        double *p_lowp,
                        const uint8_t *elem_frozen,
                        int32_t step,
                        double lr, double beta1, double beta2, double eps,
                        double weight_decay,
                        double *ema, double *ema_abs, double ema_decay)
{
    if (step < 1)
        return -1;
    if ((ema == NULL) != (ema_abs == NULL))
        return -1;
    const double bc1 = 1.0 - pow(beta1, (double)step);
    const double bc2 = 1.0 - pow(beta2, (double)step);
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < numel; ++j) {
        if (elem_frozen && elem_frozen[j])
            continue;                               /* I = 1: no update at all */
        const double g = grad_scale * grad[j];
        const double mj = beta1 * m[j] + (1.0 - beta1) * g;
        const double vj = beta2 * v[j] + (1.0 - beta2) * g * g;
        const double mhat = mj / bc1;
        const double vhat = vj / bc2;
        /* applied update u = p_new - p_old; decay acts on the old p */
        const double u = -lr * weight_decay * p[j] - lr * mhat / (sqrt(vhat) + eps);
        m[j] = mj;
        v[j] = vj;
        p[j] = p[j] + u;
        if (p_lowp)
            p_lowp[j] = oracle_bf16_rne(p[j]);
        if (ema) {                                   /* Sec. 2.3, Delta_K = u */
            ema[j] = ema_decay * ema[j] + (1.0 - ema_decay) * u;
            ema_abs[j] = ema_decay * ema_abs[j] + (1.0 - ema_decay) * fabs(u);
        }
    }
    return 0;
}

/* O3 standalone: the same two recurrences with Delta supplied by the caller
 * (stability checks spaced more than one step apart). */
int oracle_stability_update(int64_t numel, const double *delta,
                            double *ema, double *ema_abs, double ema_decay,
                            const uint8_t *elem_frozen)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < numel; ++j) {
        if (elem_frozen && elem_frozen[j])
            continue;
        ema[j] = ema_decay * ema[j] + (1.0 - ema_decay) * delta[j];
        ema_abs[j] = ema_decay * ema_abs[j] + (1.0 - ema_decay) * fabs(delta[j]);
    }
    return 0;
}

/* Per-tensor sums feeding the tensor-level score: out[0] = sum_j |E_j|,
 * out[1] = sum_j A_j, over ALL elements (serial, index order). */
void oracle_score_sums(int64_t numel, const double *ema, const double *ema_abs,
                       double *out)
{
    double se = 0.0, sa = 0.0;
    for (int64_t j = 0; j < numel; ++j) {
        se += fabs(ema[j]);
        sa += ema_abs[j];
    }
    out[0] = se;
    out[1] = sa;
}

/* Per-element APF score |E| / E^abs (Sec. 2.3); E^abs == 0 (never updated)
 * scores 1, i.e. "not known to be stable". */
void oracle_elem_scores(int64_t numel, const double *ema, const double *ema_abs,
                        double *score)
{
    for (int64_t j = 0; j < numel; ++j)
        score[j] = (ema_abs[j] == 0.0) ? 1.0 : fabs(ema[j]) / ema_abs[j];
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
