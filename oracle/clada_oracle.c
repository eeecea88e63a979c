/*
 * CLADA fp64 CPU oracle  --  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of the thresholded sparse
 * SwiGLU FFN path of CLADA (arXiv 2502.19078), written straight from the
 * paper's definitions.  It exists so that the GPU library can be checked
 * against something that shares no code with it.  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it; the product never does.
 *
 * Conventions
 *   - every input is the exact stored value (fp32, or bf16 widened to fp32,
 *     which is exact), passed as float; every arithmetic step is fp64 with no
 *     intermediate rounding, no blocking, no reordering beyond what the
 *     definition states (sums run over ascending index).
 *   - weights are neuron-major: row j of W_gate / W_up is neuron j's input
 *     projection row, row j of W_down is neuron j's output-projection column
 *     (section 3.2.1, text under the neuron-activation equation).
 *   - OpenMP only splits loops whose iterations are independent, so results
 *     do not depend on the thread count.
 *
 * Pins (see tests/test_oracle_*.py): library fp64 matmul, scalar hand cases,
 * tau=0 => dense, tau=+inf => zero, pure-Python brute force on 8-neuron toys,
 * closed forms for entropy/surprisal, the printed lambda/gamma factor table,
 * numpy.partition order statistics; for the CETT evaluation and search a
 * hand-worked three-neuron example, brute force over every candidate threshold,
 * dense-minus-sparse decode outputs, the closed form for orthogonal output rows
 * and a constructed non-monotone case; for the static masks hand cases with
 * ties / NaN / signed zeros and numpy's lexsort / partition; for the non-gated
 * ReLU FFN a hand case and numpy fp64 matmul.  No function here is "parity
 * unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* sigma in the neuron-activation equation, read as SiLU for gated (SwiGLU)
 * FFNs: sigma(g) = g * sigmoid(g) = g / (1 + exp(-g)). */
static double silu(double g) { return g / (1.0 + exp(-g)); }

/* sigma of the GELU-gated FFN (the Gemma model of the paper's experiments), in the tanh
 * form that model's public configuration names:
 *   GELU(g) = g/2 * (1 + tanh(sqrt(2/pi) * (g + 0.044715 g^3))). */
static double gelu_tanh(double g)
{
    return 0.5 * g * (1.0 + tanh(0.7978845608028654 * (g + 0.044715 * g * g * g)));
}

/* Which sigma the gated functions below use: 0 = SiLU (default), 1 = tanh-form GELU.
 * Set by the Python wrapper before every call from its own `sigma` argument. */
static int g_sigma = 0;
int clada_oracle_set_sigma(int kind)
{
    if (kind != 0 && kind != 1) return 1;
    g_sigma = kind;
    return 0;
}
static double sigma_act(double g) { return g_sigma == 1 ? gelu_tanh(g) : silu(g); }

static double dot_fd(const float *w, const float *x, int n)
{
    double s = 0.0;
    for (int i = 0; i < n; ++i) s += (double)w[i] * (double)x[i];
    return s;
}

int clada_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------
 * Prefill: dense FFN over the prefix plus per-neuron aggregates.
 * (section 3.2.1, neuron-activation equation; Algorithm "CLADA Inference",
 * prefill phase.)
 *
 *   g_tj = W_gate[j,:] . X[t,:]      u_tj = W_up[j,:] . X[t,:]
 *   a_tj = sigma(g_tj)               h_tj = a_tj * u_tj
 *   Y[t,:] = sum_j h_tj * W_down[j,:]
 *   sum_abs_act[j] = sum_t |a_tj|    sum_sq_act[j] = sum_t a_tj^2
 *   max_abs_act[j] = max_t |a_tj|    sum_sq_h[j]   = sum_t h_tj^2
 *   A[j] = || h_{:,j} W_down[j,:] ||_F = sqrt(sum_sq_h[j]) * ||W_down[j,:]||_2
 *   pool[t][j] = |a_tj|
 * Any output pointer may be NULL.
 * ---------------------------------------------------------------------- */
int clada_oracle_prefix_stats(const float *w_gate, const float *w_up,
                              const float *w_down, int d, int d_ff,
                              const float *x, int T, double *y,
                              double *sum_abs_act, double *sum_sq_act,
                              double *max_abs_act, double *sum_sq_h, double *A,
                              double *pool)
{
    if (!w_gate || !w_up || !w_down || !x || d <= 0 || d_ff <= 0 || T < 0) return 1;
    double *h = NULL;
    if (y) {
        h = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * (size_t)d_ff);
        if (!h) return 2;
    }
#pragma omp parallel for schedule(static)
    for (int j = 0; j < d_ff; ++j) {
        const float *wg = w_gate + (size_t)j * d;
        const float *wu = w_up + (size_t)j * d;
        const float *wd = w_down + (size_t)j * d;
        double s_abs = 0.0, s_sq = 0.0, mx = 0.0, s_h2 = 0.0;
        for (int t = 0; t < T; ++t) {
            const float *xt = x + (size_t)t * d;
            double g = dot_fd(wg, xt, d);
            double u = dot_fd(wu, xt, d);
            double a = sigma_act(g);
            double hv = a * u;
            double aa = fabs(a);
            s_abs += aa;
            s_sq += a * a;
            if (aa != aa) mx = aa;                       /* a NaN sticks */
            else if (mx == mx && aa > mx) mx = aa;
            s_h2 += hv * hv;
            if (pool) pool[(size_t)t * d_ff + j] = aa;
            if (h) h[(size_t)t * d_ff + j] = hv;
        }
        double wn2 = 0.0;
        for (int i = 0; i < d; ++i) wn2 += (double)wd[i] * (double)wd[i];
        if (sum_abs_act) sum_abs_act[j] = s_abs;
        if (sum_sq_act) sum_sq_act[j] = s_sq;
        if (max_abs_act) max_abs_act[j] = mx;
        if (sum_sq_h) sum_sq_h[j] = s_h2;
        if (A) A[j] = sqrt(s_h2) * sqrt(wn2);
    }
    if (y) {
#pragma omp parallel for schedule(static)
        for (int t = 0; t < T; ++t) {
            double *yt = y + (size_t)t * d;
            for (int i = 0; i < d; ++i) yt[i] = 0.0;
            for (int j = 0; j < d_ff; ++j) {
                double hv = h[(size_t)t * d_ff + j];
                const float *wd = w_down + (size_t)j * d;
                for (int i = 0; i < d; ++i) yt[i] += hv * (double)wd[i];
            }
        }
        free(h);
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Base-threshold calibration, percentile stand-in for the CETT search of
 * section 3.2.2: tau_base = the k-th smallest of the pooled prefix magnitudes,
 * k = max(1, ceil(q * n)) (nearest-rank quantile).  q is the fp32 value the
 * caller holds, widened; the rank is taken in fp64.
 * ---------------------------------------------------------------------- */
static int cmp_double(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    return (x > y) - (x < y);
}

int64_t clada_oracle_quantile_rank(int64_t n, float q)
{
    double r = ceil((double)q * (double)n);
    int64_t k = (int64_t)r;
    if (k < 1) k = 1;
    if (k > n) k = n;
    return k;
}

int clada_oracle_calibrate(const double *pool, int64_t n, float q, double *tau_base)
{
    if (!pool || !tau_base || n <= 0 || !(q >= 0.0f) || !(q < 1.0f)) return 1;
    double *tmp = (double *)malloc(sizeof(double) * (size_t)n);
    if (!tmp) return 2;
    memcpy(tmp, pool, sizeof(double) * (size_t)n);
    qsort(tmp, (size_t)n, sizeof(double), cmp_double);
    *tau_base = tmp[clada_oracle_quantile_rank(n, q) - 1];
    free(tmp);
    return 0;
}

/* ------------------------------------------------------------------------
 * Cognitive-load signals (section 2.3.1, surprisal and entropy equations):
 *   P = softmax(z) over the vocabulary (natural log, raw nats)
 *   s = -log P[tok] = lse - z_tok
 *   H = -sum_v P_v log P_v, terms with P_v = 0 contribute 0
 * A row holding NaN or +inf, or nothing but -inf, has no distribution:
 * s = H = NaN.  A token id outside [0, V) gives s = NaN, H still defined.
 * ---------------------------------------------------------------------- */
int clada_oracle_signals(const float *logits, int B, int V, const int32_t *tok,
                         double *surprisal, double *entropy)
{
    if (!logits || !tok || !surprisal || !entropy || B < 0 || V <= 0) return 1;
    for (int b = 0; b < B; ++b) {
        const float *z = logits + (size_t)b * V;
        double m = -INFINITY;
        int bad = 0;
        for (int v = 0; v < V; ++v) {
            double zv = (double)z[v];
            if (zv != zv || zv == INFINITY) bad = 1;
            if (zv > m) m = zv;
        }
        if (bad || m == -INFINITY) {
            surprisal[b] = NAN;
            entropy[b] = NAN;
            continue;
        }
        double Z = 0.0;
        for (int v = 0; v < V; ++v) Z += exp((double)z[v] - m);
        double lse = m + log(Z);
        double H = 0.0;
        for (int v = 0; v < V; ++v) {
            double logp = (double)z[v] - lse;
            double p = exp(logp);
            if (p > 0.0) H -= p * logp;
        }
        entropy[b] = H;
        surprisal[b] = (tok[b] >= 0 && tok[b] < V) ? lse - (double)z[tok[b]] : NAN;
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Token-aware threshold (section 3.2.3, final-threshold equation):
 *   tau_final[l][b] = tau_base[l] * (1 + lambda[l]*[s_b > tau_s]
 *                                      + gamma[l]*[H_b > tau_H])
 * Strict '>' as printed; signed coefficients, no clamp.
 * ---------------------------------------------------------------------- */
int clada_oracle_threshold(const double *tau_base, const double *lambda,
                           const double *gamma, int L, const double *surprisal,
                           const double *entropy, int B, double tau_s,
                           double tau_H, double *tau_final)
{
    if (!tau_base || !lambda || !gamma || !surprisal || !entropy || !tau_final ||
        L < 0 || B < 0)
        return 1;
    for (int l = 0; l < L; ++l)
        for (int b = 0; b < B; ++b) {
            double is = surprisal[b] > tau_s ? 1.0 : 0.0;
            double ih = entropy[b] > tau_H ? 1.0 : 0.0;
            tau_final[(size_t)l * B + b] = tau_base[l] * (1.0 + lambda[l] * is + gamma[l] * ih);
        }
    return 0;
}

/* ------------------------------------------------------------------------
 * Decode-time activations of one layer: a_bj = SiLU(W_gate[j,:] . x_b).
 * ---------------------------------------------------------------------- */
int clada_oracle_gate_act(const float *w_gate, int d, int d_ff, const float *x,
                          int B, double *act /* [B][d_ff] */)
{
    if (!w_gate || !x || !act || d <= 0 || d_ff <= 0 || B < 0) return 1;
    for (int b = 0; b < B; ++b) {
        const float *xb = x + (size_t)b * d;
#pragma omp parallel for schedule(static)
        for (int j = 0; j < d_ff; ++j)
            act[(size_t)b * d_ff + j] = sigma_act(dot_fd(w_gate + (size_t)j * d, xb, d));
    }
    return 0;
}

/* y_b = sum over kept j (ascending) of a_bj * (W_up[j,:] . x_b) * W_down[j,:]
 * with the kept set given per token.  mask == NULL keeps every neuron. */
static void ffn_given_mask(const float *w_gate, const float *w_up,
                           const float *w_down, int d, int d_ff, const float *x,
                           int B, const uint8_t *mask, const double *act_in,
                           double *y)
{
    double *h = (double *)malloc(sizeof(double) * (size_t)d_ff);
    for (int b = 0; b < B; ++b) {
        const float *xb = x + (size_t)b * d;
        const uint8_t *mb = mask ? mask + (size_t)b * d_ff : NULL;
#pragma omp parallel for schedule(static)
        for (int j = 0; j < d_ff; ++j) {
            if (mb && !mb[j]) {
                h[j] = 0.0;
                continue;
            }
            double a = act_in ? act_in[(size_t)b * d_ff + j]
                              : sigma_act(dot_fd(w_gate + (size_t)j * d, xb, d));
            double u = dot_fd(w_up + (size_t)j * d, xb, d);
            h[j] = a * u;
        }
        double *yb = y + (size_t)b * d;
        /* each thread owns a block of output columns and walks j upward */
#pragma omp parallel
        {
#ifdef _OPENMP
            int nt = omp_get_num_threads(), id = omp_get_thread_num();
#else
            int nt = 1, id = 0;
#endif
            int lo = (int)((int64_t)d * id / nt), hi = (int)((int64_t)d * (id + 1) / nt);
            for (int i = lo; i < hi; ++i) yb[i] = 0.0;
            for (int j = 0; j < d_ff; ++j) {
                if (mb && !mb[j]) continue;
                double hv = h[j];
                const float *wd = w_down + (size_t)j * d;
                for (int i = lo; i < hi; ++i) yb[i] += hv * (double)wd[i];
            }
        }
    }
    free(h);
}

/* ------------------------------------------------------------------------
 * Sparse decode of one layer (Algorithm "CLADA Inference", generation phase:
 * regenerate the mask by thresholding, then the sparse forward pass).
 *   keep_bj = (|a_bj| >= tau_b)      (cut iff strictly below; NaN is cut)
 *   y_b     = sum_{j kept for b} a_bj u_bj W_down[j,:]
 *   active_idx = ascending { j : kept for some b },  n_active[0] = its size,
 *   n_active[1+b] = kept count of token b.
 * Optional outputs: act [B][d_ff], mask [B][d_ff] (0/1), active_idx [d_ff],
 * n_active [1+B].
 * ---------------------------------------------------------------------- */
int clada_oracle_sparse_decode(const float *w_gate, const float *w_up,
                               const float *w_down, int d, int d_ff,
                               const float *x, int B, const double *tau,
                               double *y, double *act, uint8_t *mask,
                               int32_t *active_idx, int32_t *n_active)
{
    if (!w_gate || !w_up || !w_down || !x || !tau || !y || d <= 0 || d_ff <= 0 || B < 0)
        return 1;
    size_t n = (size_t)(B > 0 ? B : 1) * (size_t)d_ff;
    double *a = (double *)malloc(sizeof(double) * n);
    uint8_t *m = (uint8_t *)malloc(n);
    if (!a || !m) return 2;
    clada_oracle_gate_act(w_gate, d, d_ff, x, B, a);
    for (int b = 0; b < B; ++b)
        for (int j = 0; j < d_ff; ++j)
            m[(size_t)b * d_ff + j] = (fabs(a[(size_t)b * d_ff + j]) >= tau[b]) ? 1 : 0;
    ffn_given_mask(w_gate, w_up, w_down, d, d_ff, x, B, m, a, y);
    if (n_active || active_idx) {
        int32_t nu = 0;
        for (int j = 0; j < d_ff; ++j) {
            int any = 0;
            for (int b = 0; b < B; ++b) any |= m[(size_t)b * d_ff + j];
            if (any) {
                if (active_idx) active_idx[nu] = j;
                ++nu;
            }
        }
        if (n_active) {
            n_active[0] = nu;
            for (int b = 0; b < B; ++b) {
                int32_t c = 0;
                for (int j = 0; j < d_ff; ++j) c += m[(size_t)b * d_ff + j];
                n_active[1 + b] = c;
            }
        }
    }
    if (act) memcpy(act, a, sizeof(double) * (size_t)B * d_ff);
    if (mask) memcpy(mask, m, (size_t)B * d_ff);
    free(a);
    free(m);
    return 0;
}

/* The same forward pass on a kept set supplied by the caller (used to check a
 * device result whose mask differs from the oracle's only inside the allowed
 * band around the threshold). */
int clada_oracle_decode_given_mask(const float *w_gate, const float *w_up,
                                   const float *w_down, int d, int d_ff,
                                   const float *x, int B, const uint8_t *mask,
                                   double *y)
{
    if (!w_gate || !w_up || !w_down || !x || !mask || !y || d <= 0 || d_ff <= 0 || B < 0)
        return 1;
    ffn_given_mask(w_gate, w_up, w_down, d, d_ff, x, B, mask, NULL, y);
    return 0;
}

/* Dense twin: every neuron kept (the paper's "Dense" column). */
int clada_oracle_dense_decode(const float *w_gate, const float *w_up,
                              const float *w_down, int d, int d_ff,
                              const float *x, int B, double *y)
{
    if (!w_gate || !w_up || !w_down || !x || !y || d <= 0 || d_ff <= 0 || B < 0) return 1;
    ffn_given_mask(w_gate, w_up, w_down, d, d_ff, x, B, NULL, NULL, y);
    return 0;
}

/* ------------------------------------------------------------------------
 * Cumulative error of tail truncation (section 3.2.2, base-threshold equation).
 *
 *   CETT(x; eps) = || sum_{j in S_cut(x; eps)} n_j(x) ||_2 / || MLP(x) ||_2
 *
 * read with n_j(x) = h_j(x) W_down[j,:] (neuron j's contribution to the output,
 * h_j = SiLU(W_gate[j,:].x) (W_up[j,:].x)), MLP(x) = sum over all j of n_j(x),
 * and S_cut(x; eps) = { j : |a_j(x)| < eps }: the magnitude and the strict cut
 * rule are those of the decode step, so that the eps found here is directly the
 * tau_base the decode step compares with.  A token whose dense output is
 * exactly zero has nothing to lose and gets CETT = 0.  A NaN magnitude is never
 * below eps, so such a neuron is never in the cut set.
 * cett [T] per token; *mean = (1/T) sum_t cett[t] (t ascending), the estimate
 * of the expectation over the validation tokens.
 * ---------------------------------------------------------------------- */
int clada_oracle_cett(const float *w_gate, const float *w_up, const float *w_down,
                      int d, int d_ff, const float *x, int T, double eps,
                      double *cett, double *mean)
{
    if (!w_gate || !w_up || !w_down || !x || !cett || d <= 0 || d_ff <= 0 || T <= 0) return 1;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *xt = x + (size_t)t * d;
        double *cut = (double *)calloc((size_t)d, sizeof(double));
        double *full = (double *)calloc((size_t)d, sizeof(double));
        if (!cut || !full) { bad = 1; free(cut); free(full); continue; }
        for (int j = 0; j < d_ff; ++j) {
            double a = sigma_act(dot_fd(w_gate + (size_t)j * d, xt, d));
            double u = dot_fd(w_up + (size_t)j * d, xt, d);
            double h = a * u;
            const float *wd = w_down + (size_t)j * d;
            int is_cut = fabs(a) < eps;
            for (int i = 0; i < d; ++i) {
                double n = h * (double)wd[i];
                full[i] += n;
                if (is_cut) cut[i] += n;
            }
        }
        double nc = 0.0, nf = 0.0;
        for (int i = 0; i < d; ++i) { nc += cut[i] * cut[i]; nf += full[i] * full[i]; }
        cett[t] = nf > 0.0 ? sqrt(nc) / sqrt(nf) : 0.0;
        free(cut);
        free(full);
    }
    if (bad) return 2;
    if (mean) {
        double s = 0.0;
        for (int t = 0; t < T; ++t) s += cett[t];
        *mean = s / (double)T;
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Layer-wise base threshold (section 3.2.2):
 *     tau_base = max eps  subject to  mean_t CETT(x_t; eps) <= bound
 * over the validation tokens x [T][d] (bound = 0.2 in the paper).
 *
 * The cut sets change only when eps passes one of the T*d_ff magnitudes
 * |a_tj|, and every eps in (v, v'] between two neighbouring magnitudes cuts
 * what eps = v' cuts.  So if any eps is feasible, the largest feasible one is
 * either a magnitude or unbounded.  The function visits every distinct
 * magnitude v in ascending order, keeps per token the running cut sum
 * c_t = sum_{|a_tj| < v} n_j(x_t), and records the last v whose mean is within
 * the bound.  Nothing is assumed about monotonicity: the norm of a sum can
 * shrink when a term is added, so every candidate is checked.
 *
 * Outputs: *tau = that magnitude, *mean_at_tau = the mean CETT there.
 * Returns 0 on success, 3 if the all-cut mean (eps above every magnitude) is
 * still within the bound (then the maximum is unbounded; *tau = +inf), 4 if no
 * magnitude is feasible (cannot happen for bound >= 0, since the smallest
 * magnitude cuts nothing).
 * ---------------------------------------------------------------------- */
typedef struct { double v; int t, j; } cett_event;

static int cmp_event(const void *a, const void *b)
{
    const cett_event *x = (const cett_event *)a, *y = (const cett_event *)b;
    if (x->v != y->v) return (x->v > y->v) - (x->v < y->v);
    if (x->t != y->t) return (x->t > y->t) - (x->t < y->t);
    return (x->j > y->j) - (x->j < y->j);
}

int clada_oracle_cett_search(const float *w_gate, const float *w_up, const float *w_down,
                             int d, int d_ff, const float *x, int T, double bound,
                             double *tau, double *mean_at_tau)
{
    if (!w_gate || !w_up || !w_down || !x || !tau || d <= 0 || d_ff <= 0 || T <= 0) return 1;
    size_t N = (size_t)T * (size_t)d_ff;
    double *h = (double *)malloc(sizeof(double) * N);
    cett_event *ev = (cett_event *)malloc(sizeof(cett_event) * N);
    double *c = (double *)calloc((size_t)T * (size_t)d, sizeof(double));
    double *den = (double *)malloc(sizeof(double) * (size_t)T);
    double *cur = (double *)calloc((size_t)T, sizeof(double));
    if (!h || !ev || !c || !den || !cur) { free(h); free(ev); free(c); free(den); free(cur); return 2; }

#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *xt = x + (size_t)t * d;
        double *full = c + (size_t)t * d;                 /* borrowed as the dense sum, cleared below */
        for (int j = 0; j < d_ff; ++j) {
            double a = sigma_act(dot_fd(w_gate + (size_t)j * d, xt, d));
            double u = dot_fd(w_up + (size_t)j * d, xt, d);
            double hv = a * u;
            h[(size_t)t * d_ff + j] = hv;
            cett_event e = { fabs(a), t, j };
            ev[(size_t)t * d_ff + j] = e;
            const float *wd = w_down + (size_t)j * d;
            for (int i = 0; i < d; ++i) full[i] += hv * (double)wd[i];
        }
        double nf = 0.0;
        for (int i = 0; i < d; ++i) { nf += full[i] * full[i]; full[i] = 0.0; }
        den[t] = sqrt(nf);
    }
    /* NaN magnitudes are never cut: move them out of the visited range */
    size_t n_ev = 0;
    for (size_t k = 0; k < N; ++k)
        if (ev[k].v == ev[k].v) ev[n_ev++] = ev[k];
    qsort(ev, n_ev, sizeof(cett_event), cmp_event);

    int found = 0;
    double best = 0.0, best_mean = 0.0;
    size_t k = 0;
    while (k < n_ev) {
        double v = ev[k].v;
        double s = 0.0;
        for (int t = 0; t < T; ++t) s += cur[t];
        double m = s / (double)T;
        if (m <= bound) { found = 1; best = v; best_mean = m; }
        /* every magnitude equal to v joins the cut sets of all larger eps */
        while (k < n_ev && ev[k].v == v) {
            int t = ev[k].t, j = ev[k].j;
            double hv = h[(size_t)t * d_ff + j];
            const float *wd = w_down + (size_t)j * d;
            double *ct = c + (size_t)t * d;
            double nc = 0.0;
            for (int i = 0; i < d; ++i) { ct[i] += hv * (double)wd[i]; nc += ct[i] * ct[i]; }
            cur[t] = den[t] > 0.0 ? sqrt(nc) / den[t] : 0.0;
            ++k;
        }
    }
    double s = 0.0;
    for (int t = 0; t < T; ++t) s += cur[t];
    double all_cut = s / (double)T;
    int rc = 0;
    if (all_cut <= bound) { rc = 3; best = INFINITY; best_mean = all_cut; }
    else if (!found) rc = 4;
    *tau = best;
    if (mean_at_tau) *mean_at_tau = best_mean;
    free(h); free(ev); free(c); free(den); free(cur);
    return rc;
}

/* ------------------------------------------------------------------------
 * Prefix-static masks.
 *
 * (i) The generation-phase line "regenerate the masks by thresholding A" of the
 * algorithm "CLADA Inference" read literally: the prefill magnitudes A_j of the
 * neuron-activation equation (section 3.2.1) are compared with tau_final;
 * keep iff A_j >= tau (cut iff strictly below, as in the cut set of the
 * base-threshold equation; NaN is cut).
 * (ii) A hard top-k on a per-neuron prefix score, the way section 4 describes
 * the Griffin baseline: the k neurons with the largest score; equal scores go
 * to the lower index; NaN ranks below every number.
 * Outputs: mask [d_ff] 0/1 (may be NULL), idx ascending (may be NULL), *n.
 * ---------------------------------------------------------------------- */
int clada_oracle_static_mask_threshold(const double *A, int d_ff, double tau,
                                       uint8_t *mask, int32_t *idx, int32_t *n)
{
    if (!A || !n || d_ff <= 0) return 1;
    int32_t c = 0;
    for (int j = 0; j < d_ff; ++j) {
        int keep = A[j] >= tau;
        if (mask) mask[j] = (uint8_t)keep;
        if (keep) { if (idx) idx[c] = j; ++c; }
    }
    *n = c;
    return 0;
}

typedef struct { double s; int j; } score_item;

static int cmp_score_desc(const void *a, const void *b)
{
    const score_item *x = (const score_item *)a, *y = (const score_item *)b;
    int xn = x->s != x->s, yn = y->s != y->s;
    if (xn != yn) return xn - yn;                       /* numbers before NaN */
    if (!xn && x->s != y->s) return (x->s < y->s) - (x->s > y->s);   /* larger first */
    return (x->j > y->j) - (x->j < y->j);               /* then lower index first */
}

int clada_oracle_static_mask_topk(const double *score, int d_ff, int k,
                                  uint8_t *mask, int32_t *idx, int32_t *n)
{
    if (!score || !n || d_ff <= 0 || k < 0 || k > d_ff) return 1;
    score_item *it = (score_item *)malloc(sizeof(score_item) * (size_t)d_ff);
    uint8_t *m = (uint8_t *)calloc((size_t)d_ff, 1);
    if (!it || !m) { free(it); free(m); return 2; }
    for (int j = 0; j < d_ff; ++j) { it[j].s = score[j]; it[j].j = j; }
    qsort(it, (size_t)d_ff, sizeof(score_item), cmp_score_desc);
    for (int r = 0; r < k; ++r) m[it[r].j] = 1;
    int32_t c = 0;
    for (int j = 0; j < d_ff; ++j)
        if (m[j]) { if (idx) idx[c] = j; ++c; }
    if (mask) memcpy(mask, m, (size_t)d_ff);
    *n = c;
    free(it);
    free(m);
    return 0;
}

/* ------------------------------------------------------------------------
 * Non-gated ReLU FFN (the OPT models of the experimental set-up): the
 * neuron-activation equation of section 3.2.1 without the V_in factor and with
 * sigma = ReLU, biases as in those models:
 *   a_bj = max(0, W_in[j,:] . x_b + b_in[j])
 *   keep_bj = a_bj >= tau_b            (the decode step's cut rule; a >= 0)
 *   y_b = sum_{j kept} a_bj W_out[j,:] + b_out
 * W_in, W_out neuron-major [d_ff][d]; b_in [d_ff], b_out [d] may be NULL (zero).
 * Kept set: tau != NULL -> by threshold; else mask_in != NULL -> as given;
 * else every neuron (dense twin).  Optional outputs as in the gated decode.
 * ---------------------------------------------------------------------- */
int clada_oracle_relu_decode(const float *w_in, const float *b_in, const float *w_out,
                             const float *b_out, int d, int d_ff, const float *x, int B,
                             const double *tau, const uint8_t *mask_in, double *y,
                             double *act, uint8_t *mask, int32_t *active_idx,
                             int32_t *n_active)
{
    if (!w_in || !w_out || !x || !y || d <= 0 || d_ff <= 0 || B < 0) return 1;
    size_t n = (size_t)(B > 0 ? B : 1) * (size_t)d_ff;
    double *a = (double *)malloc(sizeof(double) * n);
    uint8_t *m = (uint8_t *)malloc(n);
    if (!a || !m) { free(a); free(m); return 2; }
    for (int b = 0; b < B; ++b) {
        const float *xb = x + (size_t)b * d;
#pragma omp parallel for schedule(static)
        for (int j = 0; j < d_ff; ++j) {
            double g = dot_fd(w_in + (size_t)j * d, xb, d) + (b_in ? (double)b_in[j] : 0.0);
            double v = g > 0.0 ? g : (g != g ? g : 0.0);          /* NaN stays NaN */
            a[(size_t)b * d_ff + j] = v;
            int keep = tau ? (v >= tau[b]) : (mask_in ? mask_in[(size_t)b * d_ff + j] != 0 : 1);
            m[(size_t)b * d_ff + j] = (uint8_t)keep;
        }
        double *yb = y + (size_t)b * d;
#pragma omp parallel for schedule(static)
        for (int i = 0; i < d; ++i) {
            double s = 0.0;
            for (int j = 0; j < d_ff; ++j)
                if (m[(size_t)b * d_ff + j]) s += a[(size_t)b * d_ff + j] * (double)w_out[(size_t)j * d + i];
            yb[i] = s + (b_out ? (double)b_out[i] : 0.0);
        }
    }
    if (n_active || active_idx) {
        int32_t nu = 0;
        for (int j = 0; j < d_ff; ++j) {
            int any = 0;
            for (int b = 0; b < B; ++b) any |= m[(size_t)b * d_ff + j];
            if (any) { if (active_idx) active_idx[nu] = j; ++nu; }
        }
        if (n_active) {
            n_active[0] = nu;
            for (int b = 0; b < B; ++b) {
                int32_t c = 0;
                for (int j = 0; j < d_ff; ++j) c += m[(size_t)b * d_ff + j];
                n_active[1 + b] = c;
            }
        }
    }
    if (act) memcpy(act, a, sizeof(double) * (size_t)B * d_ff);
    if (mask) memcpy(mask, m, (size_t)B * d_ff);
    free(a);
    free(m);
    return 0;
}

/* Prefill statistics of the non-gated ReLU FFN: the aggregates of
 * clada_oracle_prefix_stats with a_tj = max(0, W_in[j,:].x_t + b_in[j]), h_tj = a_tj,
 * Y[t,:] = sum_j h_tj W_out[j,:] + b_out. */
int clada_oracle_relu_prefix_stats(const float *w_in, const float *b_in, const float *w_out,
                                   const float *b_out, int d, int d_ff, const float *x, int T,
                                   double *y, double *sum_abs_act, double *sum_sq_act,
                                   double *max_abs_act, double *sum_sq_h, double *A, double *pool)
{
    if (!w_in || !w_out || !x || d <= 0 || d_ff <= 0 || T < 0) return 1;
    double *h = NULL;
    if (y) {
        h = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * (size_t)d_ff);
        if (!h) return 2;
    }
#pragma omp parallel for schedule(static)
    for (int j = 0; j < d_ff; ++j) {
        double s_abs = 0.0, s_sq = 0.0, mx = 0.0, wn2 = 0.0;
        for (int t = 0; t < T; ++t) {
            double g = dot_fd(w_in + (size_t)j * d, x + (size_t)t * d, d) + (b_in ? (double)b_in[j] : 0.0);
            double a = g > 0.0 ? g : (g != g ? g : 0.0);
            s_abs += a;
            s_sq += a * a;
            if (a != a) mx = a;
            else if (mx == mx && a > mx) mx = a;
            if (pool) pool[(size_t)t * d_ff + j] = a;
            if (h) h[(size_t)t * d_ff + j] = a;
        }
        for (int i = 0; i < d; ++i) wn2 += (double)w_out[(size_t)j * d + i] * (double)w_out[(size_t)j * d + i];
        if (sum_abs_act) sum_abs_act[j] = s_abs;
        if (sum_sq_act) sum_sq_act[j] = s_sq;
        if (max_abs_act) max_abs_act[j] = mx;
        if (sum_sq_h) sum_sq_h[j] = s_sq;
        if (A) A[j] = sqrt(s_sq) * sqrt(wn2);
    }
    if (y) {
#pragma omp parallel for schedule(static)
        for (int t = 0; t < T; ++t) {
            double *yt = y + (size_t)t * d;
            for (int i = 0; i < d; ++i) yt[i] = 0.0;
            for (int j = 0; j < d_ff; ++j) {
                double hv = h[(size_t)t * d_ff + j];
                for (int i = 0; i < d; ++i) yt[i] += hv * (double)w_out[(size_t)j * d + i];
            }
            if (b_out)
                for (int i = 0; i < d; ++i) yt[i] += (double)b_out[i];
        }
        free(h);
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * CETT of the non-gated ReLU FFN (the OPT models of the experimental set-up;
 * section 3.2.2 writes the quantity for a generic MLP):
 *   a_j = max(0, W_in[j,:].x + b_in[j]),  n_j(x) = a_j W_out[j,:],
 *   MLP(x) = sum_j n_j(x) + b_out,
 *   CETT(x; eps) = || sum_{j : a_j < eps} n_j(x) ||_2 / || MLP(x) ||_2
 * (strict cut as in the decode step, NaN never cut; a token whose output is
 * zero counts as 0).  The bias belongs to the layer's output, not to any
 * neuron, so it appears in the denominator only.
 * ---------------------------------------------------------------------- */
static double relu_act(const float *w_in, const float *b_in, int j, const float *xt, int d)
{
    double g = dot_fd(w_in + (size_t)j * d, xt, d) + (b_in ? (double)b_in[j] : 0.0);
    return g > 0.0 ? g : (g != g ? g : 0.0);
}

int clada_oracle_relu_cett(const float *w_in, const float *b_in, const float *w_out, const float *b_out,
                           int d, int d_ff, const float *x, int T, double eps,
                           double *cett, double *mean)
{
    if (!w_in || !w_out || !x || !cett || d <= 0 || d_ff <= 0 || T <= 0) return 1;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *xt = x + (size_t)t * d;
        double *cut = (double *)calloc((size_t)d, sizeof(double));
        double *full = (double *)calloc((size_t)d, sizeof(double));
        if (!cut || !full) { bad = 1; free(cut); free(full); continue; }
        for (int j = 0; j < d_ff; ++j) {
            double a = relu_act(w_in, b_in, j, xt, d);
            const float *wo = w_out + (size_t)j * d;
            int is_cut = a < eps;
            for (int i = 0; i < d; ++i) {
                double n = a * (double)wo[i];
                full[i] += n;
                if (is_cut) cut[i] += n;
            }
        }
        double nc = 0.0, nf = 0.0;
        for (int i = 0; i < d; ++i) {
            double f = full[i] + (b_out ? (double)b_out[i] : 0.0);
            nc += cut[i] * cut[i];
            nf += f * f;
        }
        cett[t] = nf > 0.0 ? sqrt(nc) / sqrt(nf) : 0.0;
        free(cut);
        free(full);
    }
    if (bad) return 2;
    if (mean) {
        double s = 0.0;
        for (int t = 0; t < T; ++t) s += cett[t];
        *mean = s / (double)T;
    }
    return 0;
}

/* The base-threshold search for the ReLU FFN: as clada_oracle_cett_search, every
 * distinct activation value a candidate, the last feasible one wins.  (About
 * half the activations are exactly zero; eps = 0 cuts nothing and is always
 * feasible.)  Return codes as there. */
int clada_oracle_relu_cett_search(const float *w_in, const float *b_in, const float *w_out,
                                  const float *b_out, int d, int d_ff, const float *x, int T,
                                  double bound, double *tau, double *mean_at_tau)
{
    if (!w_in || !w_out || !x || !tau || d <= 0 || d_ff <= 0 || T <= 0) return 1;
    size_t N = (size_t)T * (size_t)d_ff;
    cett_event *ev = (cett_event *)malloc(sizeof(cett_event) * N);
    double *c = (double *)calloc((size_t)T * (size_t)d, sizeof(double));
    double *den = (double *)malloc(sizeof(double) * (size_t)T);
    double *cur = (double *)calloc((size_t)T, sizeof(double));
    if (!ev || !c || !den || !cur) { free(ev); free(c); free(den); free(cur); return 2; }

#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *xt = x + (size_t)t * d;
        double *full = c + (size_t)t * d;                 /* borrowed as the dense sum, cleared below */
        for (int j = 0; j < d_ff; ++j) {
            double a = relu_act(w_in, b_in, j, xt, d);
            cett_event e = { a, t, j };
            ev[(size_t)t * d_ff + j] = e;
            const float *wo = w_out + (size_t)j * d;
            for (int i = 0; i < d; ++i) full[i] += a * (double)wo[i];
        }
        double nf = 0.0;
        for (int i = 0; i < d; ++i) {
            double f = full[i] + (b_out ? (double)b_out[i] : 0.0);
            nf += f * f;
            full[i] = 0.0;
        }
        den[t] = sqrt(nf);
    }
    size_t n_ev = 0;
    for (size_t k = 0; k < N; ++k)
        if (ev[k].v == ev[k].v) ev[n_ev++] = ev[k];       /* NaN is never cut */
    qsort(ev, n_ev, sizeof(cett_event), cmp_event);

    int found = 0;
    double best = 0.0, best_mean = 0.0;
    size_t k = 0;
    while (k < n_ev) {
        double v = ev[k].v;
        double s = 0.0;
        for (int t = 0; t < T; ++t) s += cur[t];
        double m = s / (double)T;
        if (m <= bound) { found = 1; best = v; best_mean = m; }
        while (k < n_ev && ev[k].v == v) {
            int t = ev[k].t, j = ev[k].j;
            const float *wo = w_out + (size_t)j * d;
            double *ct = c + (size_t)t * d;
            double nc = 0.0;
            for (int i = 0; i < d; ++i) { ct[i] += v * (double)wo[i]; nc += ct[i] * ct[i]; }
            cur[t] = den[t] > 0.0 ? sqrt(nc) / den[t] : 0.0;
            ++k;
        }
    }
    double s = 0.0;
    for (int t = 0; t < T; ++t) s += cur[t];
    double all_cut = s / (double)T;
    int rc = 0;
    if (all_cut <= bound) { rc = 3; best = INFINITY; best_mean = all_cut; }
    else if (!found) rc = 4;
    *tau = best;
    if (mean_at_tau) *mean_at_tau = best_mean;
    free(ev); free(c); free(den); free(cur);
    return rc;
}
