/*
 * CPU oracle for the mixed-batch LoRA linear layer.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain, fp64 statement of what the layer computes.  It exists so
 * that the GPU library can be checked against something written independently of it; it is
 * linked only by the tests, the smoke check and the benchmark's CPU-baseline leg.  It shares
 * no code, header, table or helper with the GPU library and must never be called from it.
 *
 * What it follows:
 *   - LoRA parameterisation (paper section 4.2, "FL PEFT process"): a frozen base weight
 *     W_pre plus a trainable low-rank update Delta W = B_g A_g, h = W_pre x + B_g A_g x.
 *     Here everything is written for row vectors:  W = W_pre^T is [d_in, d_out],
 *     A_a = A_g^T is [d_in, r_a] (down-projection), B_a = B_g^T is [r_a, d_out]
 *     (up-projection), and a scalar `scale` multiplies the low-rank term.
 *   - Model sharing (paper section 2.1, "CoLLM's model sharing"): inference and fine-tuning
 *     run on one copy of W and of the adapters at the same time.  Here that is one batch of
 *     tokens split into segments; each segment names its adapter and whether it trains.
 *   - Only the adapters train (section 4.2): there is no gradient for W.
 *
 * Every loop below is the definition written out: sums run over the contracted index in
 * ascending order, one token at a time, nothing is blocked, fused or reordered.  OpenMP
 * only hands different tokens (forward) or different output entries (gradients) to
 * different threads; the order of additions into any one output entry never changes.
 *
 * All matrices are row-major, all floating point is double.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------ *
 * Integer bookkeeping, kept apart from the arithmetic.
 * Segment k owns tokens seg_start[k] .. seg_start[k+1]-1; every token inherits its
 * segment's adapter index (-1 = base weights only) and training flag.
 * ------------------------------------------------------------------------------------ */
void oracle_token_map(int32_t n_segments, const int32_t *seg_start, const int32_t *seg_adapter,
                      const uint8_t *seg_is_train, int32_t *tok_segment, int32_t *tok_adapter,
                      uint8_t *tok_is_train)
{
    for (int32_t k = 0; k < n_segments; ++k) {
        for (int32_t t = seg_start[k]; t < seg_start[k + 1]; ++t) {
            tok_segment[t] = k;
            tok_adapter[t] = seg_adapter[k];
            tok_is_train[t] = seg_is_train[k];
        }
    }
}

/* ------------------------------------------------------------------------------------ *
 * Plain product of the batch with the base weight, y0 = x W.  Used on its own by the
 * checks that pin the base term.
 * ------------------------------------------------------------------------------------ */
void oracle_base_matmul(int32_t n_tokens, int32_t d_in, int32_t d_out, const double *x,
                        const double *W, double *y0)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t t = 0; t < n_tokens; ++t) {
        double *yt = y0 + (size_t)t * d_out;
        for (int32_t j = 0; j < d_out; ++j) yt[j] = 0.0;
        for (int32_t i = 0; i < d_in; ++i) {
            const double xi = x[(size_t)t * d_in + i];
            const double *Wi = W + (size_t)i * d_out;
            for (int32_t j = 0; j < d_out; ++j) yt[j] += xi * Wi[j];
        }
    }
}

/* ------------------------------------------------------------------------------------ *
 * Forward.  For token t with adapter a = tok_adapter[t]:
 *     y[t,j]  = sum_i x[t,i] W[i,j]
 *     h[t,q]  = sum_i x[t,i] A_a[i,q]                      (a >= 0, q < rank[a])
 *     y[t,j] += scale * sum_q h[t,q] B_a[q,j]
 * h is [n_tokens, h_stride]; entries with q >= rank[a], and whole rows of base-only
 * tokens, are set to zero.  h may be NULL.
 * ------------------------------------------------------------------------------------ */
void oracle_lora_linear_fwd(int32_t n_tokens, int32_t d_in, int32_t d_out, const double *x,
                            const double *W, const double *const *A, const double *const *B,
                            const int32_t *rank, const int32_t *tok_adapter, double scale,
                            double *y, double *h, int32_t h_stride)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t t = 0; t < n_tokens; ++t) {
        const double *xt = x + (size_t)t * d_in;
        double *yt = y + (size_t)t * d_out;
        for (int32_t j = 0; j < d_out; ++j) yt[j] = 0.0;
        for (int32_t i = 0; i < d_in; ++i) {
            const double xi = xt[i];
            const double *Wi = W + (size_t)i * d_out;
            for (int32_t j = 0; j < d_out; ++j) yt[j] += xi * Wi[j];
        }
        if (h) {
            for (int32_t q = 0; q < h_stride; ++q) h[(size_t)t * h_stride + q] = 0.0;
        }
        const int32_t a = tok_adapter[t];
        if (a < 0) continue;
        const int32_t r = rank[a];
        const double *Aa = A[a];
        const double *Ba = B[a];
        double *ht = (double *)malloc(sizeof(double) * (size_t)r);
        for (int32_t q = 0; q < r; ++q) {
            double acc = 0.0;
            for (int32_t i = 0; i < d_in; ++i) acc += xt[i] * Aa[(size_t)i * r + q];
            ht[q] = acc;
        }
        for (int32_t j = 0; j < d_out; ++j) {
            double acc = 0.0;
            for (int32_t q = 0; q < r; ++q) acc += ht[q] * Ba[(size_t)q * d_out + j];
            yt[j] += scale * acc;
        }
        if (h) {
            for (int32_t q = 0; q < r; ++q) h[(size_t)t * h_stride + q] = ht[q];
        }
        free(ht);
    }
}

/* ------------------------------------------------------------------------------------ *
 * Backward for the training tokens, given the upstream gradient dy = dL/dy.
 * For a training token t with adapter a (training tokens always have one):
 *     h[t,q]   = sum_i x[t,i] A_a[i,q]
 *     dh[t,q]  = scale * sum_j dy[t,j] B_a[q,j]
 *     dB_a[q,j] += scale * h[t,q] dy[t,j]          (t ascending over the adapter's tokens)
 *     dA_a[i,q] += x[t,i] dh[t,q]                  (t ascending)
 *     dx[t,i]  = sum_j dy[t,j] W[i,j] + sum_q dh[t,q] A_a[i,q]
 * dA[a], dB[a] are zeroed first for every adapter that owns at least one training token;
 * pointers of other adapters are never touched (they may be NULL).  Rows of dx that belong
 * to inference tokens are never touched.  dx (and then W) may be NULL to skip the two
 * W-sized contractions; dA/dB may be NULL to skip the adapter gradients.
 * ------------------------------------------------------------------------------------ */
void oracle_lora_linear_bwd(int32_t n_tokens, int32_t d_in, int32_t d_out, int32_t n_adapters,
                            const double *x, const double *W, const double *const *A,
                            const double *const *B, const int32_t *rank,
                            const int32_t *tok_adapter, const uint8_t *tok_is_train, double scale,
                            const double *dy, double *dx, double *const *dA, double *const *dB)
{
    int32_t rmax = 1;
    for (int32_t a = 0; a < n_adapters; ++a)
        if (rank[a] > rmax) rmax = rank[a];
    double *h = (double *)calloc((size_t)n_tokens * rmax, sizeof(double));
    double *dh = (double *)calloc((size_t)n_tokens * rmax, sizeof(double));

    /* per-token low-rank activations and their gradients */
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t t = 0; t < n_tokens; ++t) {
        if (!tok_is_train[t]) continue;
        const int32_t a = tok_adapter[t];
        const int32_t r = rank[a];
        const double *xt = x + (size_t)t * d_in;
        const double *dyt = dy + (size_t)t * d_out;
        for (int32_t q = 0; q < r; ++q) {
            double acc = 0.0;
            for (int32_t i = 0; i < d_in; ++i) acc += xt[i] * A[a][(size_t)i * r + q];
            h[(size_t)t * rmax + q] = acc;
            double g = 0.0;
            for (int32_t j = 0; j < d_out; ++j) g += dyt[j] * B[a][(size_t)q * d_out + j];
            dh[(size_t)t * rmax + q] = scale * g;
        }
    }

    /* gradient with respect to the layer input */
    if (dx) {
#pragma omp parallel for schedule(dynamic, 1)
        for (int32_t t = 0; t < n_tokens; ++t) {
            if (!tok_is_train[t]) continue;
            const int32_t a = tok_adapter[t];
            const int32_t r = rank[a];
            const double *dyt = dy + (size_t)t * d_out;
            double *dxt = dx + (size_t)t * d_in;
            for (int32_t i = 0; i < d_in; ++i) {
                const double *Wi = W + (size_t)i * d_out;
                double acc = 0.0;
                for (int32_t j = 0; j < d_out; ++j) acc += dyt[j] * Wi[j];
                double lo = 0.0;
                for (int32_t q = 0; q < r; ++q)
                    lo += dh[(size_t)t * rmax + q] * A[a][(size_t)i * r + q];
                dxt[i] = acc + lo;
            }
        }
    }

    /* adapter gradients, summed over the adapter's training tokens in ascending order */
    if (dA && dB) {
        for (int32_t a = 0; a < n_adapters; ++a) {
            int trained = 0;
            for (int32_t t = 0; t < n_tokens; ++t)
                if (tok_is_train[t] && tok_adapter[t] == a) { trained = 1; break; }
            if (!trained) continue;
            const int32_t r = rank[a];
            double *dAa = dA[a];
            double *dBa = dB[a];
            memset(dAa, 0, sizeof(double) * (size_t)d_in * r);
            memset(dBa, 0, sizeof(double) * (size_t)r * d_out);
#pragma omp parallel for schedule(static)
            for (int32_t q = 0; q < r; ++q) {
                for (int32_t t = 0; t < n_tokens; ++t) {
                    if (!tok_is_train[t] || tok_adapter[t] != a) continue;
                    const double sh = scale * h[(size_t)t * rmax + q];
                    const double *dyt = dy + (size_t)t * d_out;
                    for (int32_t j = 0; j < d_out; ++j) dBa[(size_t)q * d_out + j] += sh * dyt[j];
                }
            }
#pragma omp parallel for schedule(static)
            for (int32_t i = 0; i < d_in; ++i) {
                for (int32_t t = 0; t < n_tokens; ++t) {
                    if (!tok_is_train[t] || tok_adapter[t] != a) continue;
                    const double xi = x[(size_t)t * d_in + i];
                    for (int32_t q = 0; q < r; ++q)
                        dAa[(size_t)i * r + q] += xi * dh[(size_t)t * rmax + q];
                }
            }
        }
    }
    free(h);
    free(dh);
}
