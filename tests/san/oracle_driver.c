/* Calls every function of the CPU oracle on small heap buffers of exactly the documented sizes.
 * Built with -fsanitize=address,undefined by tests/test_sanitizers.py: an out-of-bounds access, a
 * leak or undefined behaviour in the oracle makes the run fail.  Test infrastructure only. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int clada_oracle_set_sigma(int);
int clada_oracle_num_threads(void);
int clada_oracle_prefix_stats(const float *, const float *, const float *, int, int, const float *, int, double *,
                              double *, double *, double *, double *, double *, double *);
int64_t clada_oracle_quantile_rank(int64_t, float);
int clada_oracle_calibrate(const double *, int64_t, float, double *);
int clada_oracle_signals(const float *, int, int, const int32_t *, double *, double *);
int clada_oracle_threshold(const double *, const double *, const double *, int, const double *, const double *, int,
                           double, double, double *);
int clada_oracle_gate_act(const float *, int, int, const float *, int, double *);
int clada_oracle_sparse_decode(const float *, const float *, const float *, int, int, const float *, int,
                               const double *, double *, double *, uint8_t *, int32_t *, int32_t *);
int clada_oracle_decode_given_mask(const float *, const float *, const float *, int, int, const float *, int,
                                   const uint8_t *, double *);
int clada_oracle_dense_decode(const float *, const float *, const float *, int, int, const float *, int, double *);
int clada_oracle_cett(const float *, const float *, const float *, int, int, const float *, int, double, double *,
                      double *);
int clada_oracle_cett_search(const float *, const float *, const float *, int, int, const float *, int, double,
                             double *, double *);
int clada_oracle_static_mask_threshold(const double *, int, double, uint8_t *, int32_t *, int32_t *);
int clada_oracle_static_mask_topk(const double *, int, int, uint8_t *, int32_t *, int32_t *);
int clada_oracle_relu_decode(const float *, const float *, const float *, const float *, int, int, const float *, int,
                             const double *, const uint8_t *, double *, double *, uint8_t *, int32_t *, int32_t *);
int clada_oracle_relu_prefix_stats(const float *, const float *, const float *, const float *, int, int, const float *,
                                   int, double *, double *, double *, double *, double *, double *, double *);

static unsigned int g_s = 12345u;
static float rnd(void) { g_s = g_s * 1664525u + 1013904223u; return (float)((g_s >> 8) & 0xffff) / 65536.0f - 0.5f; }
static float *fbuf(size_t n, float scale) { float *p = malloc(sizeof(float) * (n ? n : 1)); for (size_t i = 0; i < n; ++i) p[i] = rnd() * scale; return p; }
static double *dbuf(size_t n) { return malloc(sizeof(double) * (n ? n : 1)); }
#define CHECK(call) do { int rc_ = (call); if (rc_ != 0) { printf("%s -> %d\n", #call, rc_); fails++; } } while (0)

int main(void)
{
    int fails = 0;
    static const int shapes[][4] = {{8, 5, 1, 1}, {24, 40, 3, 7}, {16, 33, 2, 64}, {7, 1, 4, 2}};   /* d, F, B, T */
    for (unsigned s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s)
        for (int sigma = 0; sigma < 2; ++sigma) {
            const int d = shapes[s][0], F = shapes[s][1], B = shapes[s][2], T = shapes[s][3];
            CHECK(clada_oracle_set_sigma(sigma));
            float *wg = fbuf((size_t)F * d, 1.0f), *wu = fbuf((size_t)F * d, 1.0f), *wd = fbuf((size_t)F * d, 1.0f);
            float *x = fbuf((size_t)B * d, 2.0f), *X = fbuf((size_t)T * d, 2.0f), *bi = fbuf(F, 0.5f), *bo = fbuf(d, 0.5f);
            double *y = dbuf((size_t)B * d), *act = dbuf((size_t)B * F), *tau = dbuf(B), *Y = dbuf((size_t)T * d);
            double *agg[5], *pool = dbuf((size_t)T * F), *ce = dbuf(T);
            for (int i = 0; i < 5; ++i) agg[i] = dbuf(F);
            uint8_t *mask = malloc((size_t)B * F);
            int32_t *idx = malloc(sizeof(int32_t) * F), *na = malloc(sizeof(int32_t) * (1 + B));
            for (int b = 0; b < B; ++b) tau[b] = 0.05 * (b + 1);
            CHECK(clada_oracle_gate_act(wg, d, F, x, B, act));
            CHECK(clada_oracle_sparse_decode(wg, wu, wd, d, F, x, B, tau, y, act, mask, idx, na));
            CHECK(clada_oracle_decode_given_mask(wg, wu, wd, d, F, x, B, mask, y));
            CHECK(clada_oracle_dense_decode(wg, wu, wd, d, F, x, B, y));
            CHECK(clada_oracle_prefix_stats(wg, wu, wd, d, F, X, T, Y, agg[0], agg[1], agg[2], agg[3], agg[4], pool));
            CHECK(clada_oracle_prefix_stats(wg, wu, wd, d, F, X, T, NULL, NULL, NULL, NULL, NULL, agg[4], NULL));
            double tb = 0, mean = 0;
            CHECK(clada_oracle_calibrate(pool, (int64_t)T * F, 0.4f, &tb));
            (void)clada_oracle_quantile_rank((int64_t)T * F, 0.4f);
            CHECK(clada_oracle_cett(wg, wu, wd, d, F, X, T, tb, ce, &mean));
            { int rc = clada_oracle_cett_search(wg, wu, wd, d, F, X, T, 0.2, &tb, &mean); if (rc != 0 && rc != 3 && rc != 4) { printf("cett_search -> %d\n", rc); fails++; } }
            CHECK(clada_oracle_static_mask_threshold(agg[4], F, tb, mask, idx, na));
            CHECK(clada_oracle_static_mask_topk(agg[4], F, F / 2, mask, idx, na));
            CHECK(clada_oracle_static_mask_topk(agg[4], F, 0, mask, idx, na));
            CHECK(clada_oracle_relu_decode(wg, bi, wd, bo, d, F, x, B, tau, NULL, y, act, mask, idx, na));
            CHECK(clada_oracle_relu_decode(wg, NULL, wd, NULL, d, F, x, B, NULL, mask, y, act, NULL, NULL, NULL));
            CHECK(clada_oracle_relu_prefix_stats(wg, bi, wd, bo, d, F, X, T, Y, agg[0], agg[1], agg[2], agg[3], agg[4], pool));
            CHECK(clada_oracle_relu_cett(wg, bi, wd, bo, d, F, X, T, 0.3, ce, &mean));
            CHECK(clada_oracle_relu_cett(wg, NULL, wd, NULL, d, F, X, T, INFINITY, ce, NULL));
            { int rc = clada_oracle_relu_cett_search(wg, bi, wd, bo, d, F, X, T, 0.2, &tb, &mean); if (rc != 0 && rc != 3 && rc != 4) { printf("relu_cett_search -> %d\n", rc); fails++; } }
            free(wg); free(wu); free(wd); free(x); free(X); free(bi); free(bo); free(y); free(act); free(tau); free(Y);
            for (int i = 0; i < 5; ++i) free(agg[i]);
            free(pool); free(ce); free(mask); free(idx); free(na);
        }
    {   /* signals and thresholds */
        const int B = 3, V = 37, L = 4;
        float *z = fbuf((size_t)B * V, 6.0f);
        z[5] = -INFINITY;
        int32_t tok[3] = {0, 36, 5};
        double s[3], h[3], tb[4] = {0.1, 0.2, 0.3, 0.4}, lam[4] = {0.8, -0.8, 0, 1}, gam[4] = {0.12, 0, -0.12, 1}, out[12];
        CHECK(clada_oracle_signals(z, B, V, tok, s, h));
        CHECK(clada_oracle_threshold(tb, lam, gam, L, s, h, B, 3.0, 3.0, out));
        free(z);
    }
    /* rejected arguments return codes, they do not touch the buffers */
    if (clada_oracle_dense_decode(NULL, NULL, NULL, 1, 1, NULL, 1, NULL) == 0) fails++;
    if (clada_oracle_set_sigma(7) == 0) fails++;
    clada_oracle_set_sigma(0);
    printf("oracle sanitizer driver: %d failures, %d threads\n", fails, clada_oracle_num_threads());
    return fails ? 1 : 0;
}
