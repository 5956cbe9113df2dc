/* Host-only driver for a sanitizer build of the CPU oracle (tests/test_host_abi.py compiles it together with
 * oracle/collm_oracle.c under -fsanitize=address,undefined and runs it): random small batches with exactly sized
 * buffers, so that any access outside them is reported; checks the hand-worked one-token example on the way.
 * Prints "oracle ok <cases>" and returns 0. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_token_map(int32_t n_segments, const int32_t *seg_start, const int32_t *seg_adapter,
                      const uint8_t *seg_is_train, int32_t *tok_segment, int32_t *tok_adapter, uint8_t *tok_is_train);
void oracle_base_matmul(int32_t n_tokens, int32_t d_in, int32_t d_out, const double *x, const double *W, double *y0);
void oracle_lora_linear_fwd(int32_t n_tokens, int32_t d_in, int32_t d_out, const double *x, const double *W,
                            const double *const *A, const double *const *B, const int32_t *rank,
                            const int32_t *tok_adapter, double scale, double *y, double *h, int32_t h_stride);
void oracle_lora_linear_bwd(int32_t n_tokens, int32_t d_in, int32_t d_out, int32_t n_adapters, const double *x,
                            const double *W, const double *const *A, const double *const *B, const int32_t *rank,
                            const int32_t *tok_adapter, const uint8_t *tok_is_train, double scale, const double *dy,
                            double *dx, double *const *dA, double *const *dB);

static uint64_t g_state = 20260416u;
static uint32_t rnd(void)
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(g_state >> 33);
}
static int uni(int lo, int hi) { return (int)(rnd() % (uint32_t)(hi - lo + 1)) + lo; }
static double *fill(size_t n)
{
    double *p = (double *)malloc((n ? n : 1) * sizeof(double));
    for (size_t i = 0; i < n; ++i) p[i] = (double)uni(-1000, 1000) / 500.0;
    return p;
}
#define REQUIRE(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main(int argc, char **argv)
{
    const int n_cases = argc > 1 ? atoi(argv[1]) : 300;
    {
        /* one token, d = 2, rank 1, scale 2: h = 3, y = [7, -4]; dy = [1, 0]: dh = 2, dB = [6, 0], dA = [2, 4], dx = [3, 2] */
        const double x[2] = {1, 2}, W[4] = {1, 0, 0, 1}, A0[2] = {1, 1}, B0[2] = {1, -1}, dy[2] = {1, 0};
        const double *A[1] = {A0}, *B[1] = {B0};
        const int32_t rank[1] = {1}, ta[1] = {0};
        const uint8_t tt[1] = {1};
        double y[2], h[1], dx[2], dA0[2], dB0[2];
        double *dA[1] = {dA0}, *dB[1] = {dB0};
        oracle_lora_linear_fwd(1, 2, 2, x, W, A, B, rank, ta, 2.0, y, h, 1);
        REQUIRE(h[0] == 3.0 && y[0] == 7.0 && y[1] == -4.0);
        oracle_lora_linear_bwd(1, 2, 2, 1, x, W, A, B, rank, ta, tt, 2.0, dy, dx, dA, dB);
        REQUIRE(dB0[0] == 6.0 && dB0[1] == 0.0 && dA0[0] == 2.0 && dA0[1] == 4.0 && dx[0] == 3.0 && dx[1] == 2.0);
    }
    for (int c = 0; c < n_cases; ++c) {
        const int N = uni(0, 5), S = uni(0, 8), d_in = uni(1, 24), d_out = uni(1, 24);
        int32_t rank[8], seg_start[16], seg_adapter[16];
        uint8_t seg_train[16];
        double *A[8], *B[8], *dA[8], *dB[8];
        for (int a = 0; a < N; ++a) rank[a] = uni(1, 9);
        seg_start[0] = 0;
        for (int k = 0; k < S; ++k) {
            seg_start[k + 1] = seg_start[k] + (uni(0, 4) ? uni(1, 6) : 0);
            seg_adapter[k] = (N == 0 || uni(0, 5) == 0) ? -1 : uni(0, N - 1);
            seg_train[k] = (uint8_t)(seg_adapter[k] >= 0 && uni(0, 1));
        }
        const int T = seg_start[S];
        int32_t *ts = (int32_t *)malloc((T ? T : 1) * sizeof(int32_t)), *ta = (int32_t *)malloc((T ? T : 1) * sizeof(int32_t));
        uint8_t *tt = (uint8_t *)malloc(T ? T : 1);
        oracle_token_map(S, seg_start, seg_adapter, seg_train, ts, ta, tt);
        for (int k = 0; k < S; ++k)
            for (int t = seg_start[k]; t < seg_start[k + 1]; ++t) REQUIRE(ts[t] == k && ta[t] == seg_adapter[k] && tt[t] == seg_train[k]);
        int rmax = 1;
        for (int a = 0; a < N; ++a) {
            A[a] = fill((size_t)d_in * rank[a]);
            B[a] = fill((size_t)rank[a] * d_out);
            dA[a] = fill((size_t)d_in * rank[a]);
            dB[a] = fill((size_t)rank[a] * d_out);
            if (rank[a] > rmax) rmax = rank[a];
        }
        double *x = fill((size_t)T * d_in), *W = fill((size_t)d_in * d_out), *dy = fill((size_t)T * d_out);
        double *y = fill((size_t)T * d_out), *y0 = fill((size_t)T * d_out), *h = fill((size_t)T * rmax), *dx = fill((size_t)T * d_in);
        oracle_base_matmul(T, d_in, d_out, x, W, y0);
        oracle_lora_linear_fwd(T, d_in, d_out, x, W, (const double *const *)A, (const double *const *)B, rank, ta, 0.5, y, h, rmax);
        oracle_lora_linear_fwd(T, d_in, d_out, x, W, (const double *const *)A, (const double *const *)B, rank, ta, 0.5, y, NULL, rmax);
        for (int t = 0; t < T; ++t)
            if (ta[t] < 0)
                for (int j = 0; j < d_out; ++j) REQUIRE(y[(size_t)t * d_out + j] == y0[(size_t)t * d_out + j]);
        oracle_lora_linear_bwd(T, d_in, d_out, N, x, W, (const double *const *)A, (const double *const *)B, rank, ta, tt, 0.5, dy, dx, dA, dB);
        oracle_lora_linear_bwd(T, d_in, d_out, N, x, NULL, (const double *const *)A, (const double *const *)B, rank, ta, tt, 0.5, dy, NULL, dA, dB);
        oracle_lora_linear_bwd(T, d_in, d_out, N, x, W, (const double *const *)A, (const double *const *)B, rank, ta, tt, 0.5, dy, dx, NULL, NULL);
        for (size_t i = 0; i < (size_t)T * d_out; ++i) REQUIRE(isfinite(y[i]));
        for (int a = 0; a < N; ++a) { free(A[a]); free(B[a]); free(dA[a]); free(dB[a]); }
        free(x); free(W); free(dy); free(y); free(y0); free(h); free(dx); free(ts); free(ta); free(tt);
    }
    printf("oracle ok %d\n", n_cases);
    return 0;
}
