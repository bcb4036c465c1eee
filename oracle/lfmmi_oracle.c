/*
 * fp64 log-domain HMM forward-backward: the CPU oracle for the LF-MMI hot path.
 *
 * TEST INFRASTRUCTURE ONLY. Slow and plain on purpose; shares no code with the
 * HIP library and must never be reached from the product path.
 *
 * What it computes (Section 2.1 Eq. 2, Section 2.2 Eq. 3, Section 3.4 Alg. 1,
 * with the leaky-HMM of the cited LF-MMI work read as an epsilon-weighted
 * restart from the initial distribution after every frame and at t = 0):
 *
 *   arcs a = (src, dst, pdf, w = exp(logw)); pi = initial probs; f = final
 *   probs; eps = leak; x_t = logits row of frame t (t = 1..T_b, row t-1).
 *
 *   alpha'_0 = L(pi),            L(v)  = v + eps * (sum v) * pi
 *   alpha_t[j] = sum_{a: dst=j} w_a * exp(x_t[pdf_a]) * alpha'_{t-1}[src_a]
 *   alpha'_t = L(alpha_t)
 *   Z = sum_j f[j] * alpha'_T[j]                       (Alg. 1, per-sequence T)
 *
 *   beta'_T = Lt(f),             Lt(u) = u + eps * (pi . u) * 1
 *   beta_{t-1}[i] = sum_{a: src=i} w_a * exp(x_t[pdf_a]) * beta'_t[dst_a]
 *   beta'_{t-1} = Lt(beta_{t-1})
 *
 *   gamma_t[d] = (1/Z) sum_{a: pdf=d} alpha'_{t-1}[src] w_a exp(x_t[d]) beta'_t[dst]
 *              = d log Z / d x_t[d]                    (Eq. 3: pdf occupancy)
 *
 * Everything is carried as natural logs in double precision; sums are
 * log-sum-exp (maximum, then sum of exponentials of the differences). There is
 * no rescaling, blocking or reordering beyond that.
 *
 * Parity status: pinned by the closed forms, brute-force path enumeration, the
 * dense matrix-product twin, invariants and finite differences in
 * tests/test_oracle_pins.py. The leak convention itself (how the cited work
 * defines it) is "parity unpinned": the paper does not define it.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static const double NEG_INF = -INFINITY;

static double log_add(double a, double b)
{
    if (a == NEG_INF) return b;
    if (b == NEG_INF) return a;
    double hi = a > b ? a : b, lo = a > b ? b : a;
    return hi + log1p(exp(lo - hi));
}

/* log(sum_i exp(v[i])), n >= 0 */
static double lse(const double *v, long n)
{
    double mx = NEG_INF;
    for (long i = 0; i < n; ++i) if (v[i] > mx) mx = v[i];
    if (mx == NEG_INF) return NEG_INF;
    double s = 0.0;
    for (long i = 0; i < n; ++i) s += exp(v[i] - mx);
    return mx + log(s);
}

/* out[key[a]] = log sum over arcs a of exp(term[a]); keys in [0, n) */
static void lse_by_key(const double *term, const int *key, long num_arcs,
                       long n, double *mx, double *sum, double *out)
{
    for (long k = 0; k < n; ++k) { mx[k] = NEG_INF; sum[k] = 0.0; }
    for (long a = 0; a < num_arcs; ++a)
        if (term[a] > mx[key[a]]) mx[key[a]] = term[a];
    for (long a = 0; a < num_arcs; ++a)
        if (term[a] != NEG_INF) sum[key[a]] += exp(term[a] - mx[key[a]]);
    for (long k = 0; k < n; ++k)
        out[k] = (mx[k] == NEG_INF) ? NEG_INF : mx[k] + log(sum[k]);
}

static int one_sequence(int S, int P, long A, const int *src, const int *dst,
                        const int *pdf, const float *logw, const double *lpi,
                        const double *lf, double leps, int T, const float *x,
                        double *logz_out, double *logz_bwd_out, double *gamma)
{
    double *la = (double *)malloc(sizeof(double) * (size_t)(T + 1) * S); /* alpha' */
    double *lb = (double *)malloc(sizeof(double) * S);                   /* beta'_t */
    double *raw = (double *)malloc(sizeof(double) * S);
    double *mx = (double *)malloc(sizeof(double) * S);
    double *sm = (double *)malloc(sizeof(double) * S);
    double *term = (double *)malloc(sizeof(double) * (A > 0 ? A : 1));
    double *tmp = (double *)malloc(sizeof(double) * S);
    if (!la || !lb || !raw || !mx || !sm || !term || !tmp) {
        free(la); free(lb); free(raw); free(mx); free(sm); free(term); free(tmp);
        return 1;
    }

    /* alpha'_0 = L(pi) */
    double tot = lse(lpi, S);
    for (int i = 0; i < S; ++i)
        la[i] = log_add(lpi[i], leps + tot + lpi[i]);

    for (int t = 1; t <= T; ++t) {
        const double *prev = la + (size_t)(t - 1) * S;
        double *cur = la + (size_t)t * S;
        const float *xt = x + (size_t)(t - 1) * P;
        for (long a = 0; a < A; ++a)
            term[a] = prev[src[a]] + (double)logw[a] + (double)xt[pdf[a]];
        lse_by_key(term, dst, A, S, mx, sm, raw);
        tot = lse(raw, S);
        for (int i = 0; i < S; ++i)
            cur[i] = log_add(raw[i], leps + tot + lpi[i]);
    }
    for (int i = 0; i < S; ++i) tmp[i] = la[(size_t)T * S + i] + lf[i];
    double logz = lse(tmp, S);
    *logz_out = logz;

    /* beta'_T = Lt(f) */
    for (int i = 0; i < S; ++i) tmp[i] = lpi[i] + lf[i];
    double dot = lse(tmp, S);
    for (int i = 0; i < S; ++i) lb[i] = log_add(lf[i], leps + dot);

    for (int t = T; t >= 1; --t) {
        const double *prev = la + (size_t)(t - 1) * S;
        const float *xt = x + (size_t)(t - 1) * P;
        /* occupancy of frame t */
        if (gamma) {
            double *g = gamma + (size_t)(t - 1) * P;
            for (int d = 0; d < P; ++d) g[d] = 0.0;
            if (logz != NEG_INF)
                for (long a = 0; a < A; ++a) {
                    double e = prev[src[a]] + (double)logw[a] + (double)xt[pdf[a]]
                               + lb[dst[a]] - logz;
                    if (e != NEG_INF) g[pdf[a]] += exp(e);
                }
        }
        /* beta_{t-1}, then beta'_{t-1} = Lt(beta_{t-1}) */
        for (long a = 0; a < A; ++a)
            term[a] = (double)logw[a] + (double)xt[pdf[a]] + lb[dst[a]];
        lse_by_key(term, src, A, S, mx, sm, raw);
        for (int i = 0; i < S; ++i) tmp[i] = lpi[i] + raw[i];
        dot = lse(tmp, S);
        for (int i = 0; i < S; ++i) lb[i] = log_add(raw[i], leps + dot);
    }
    for (int i = 0; i < S; ++i) tmp[i] = lpi[i] + lb[i];
    if (logz_bwd_out) *logz_bwd_out = lse(tmp, S);

    free(la); free(lb); free(raw); free(mx); free(sm); free(term); free(tmp);
    return 0;
}

/*
 * One graph shared by B sequences.
 *   logits [B, T, P] float32 row-major; lengths[b] in [0, T]; frames at and
 *   after lengths[b] are never read and their gamma rows are written as 0.
 *   logz [B]; logz_bwd [B] or NULL (the same total, from the backward pass);
 *   gamma [B, T, P] or NULL.
 * Returns 0, 1 on allocation failure, 2 on an invalid argument.
 * num_threads <= 0 means the OpenMP default.
 */
int lfmmi_oracle_forward_backward(int num_states, int num_pdfs, long num_arcs,
                                  const int *src, const int *dst, const int *pdf,
                                  const float *logw, const float *init_prob,
                                  const float *final_prob, double leak, int B,
                                  int T, const float *logits, const int *lengths,
                                  double *logz, double *logz_bwd, double *gamma,
                                  int num_threads)
{
    int S = num_states, P = num_pdfs;
    if (S < 1 || P < 1 || num_arcs < 0 || B < 0 || T < 0 || leak < 0.0) return 2;
    for (long a = 0; a < num_arcs; ++a)
        if (src[a] < 0 || src[a] >= S || dst[a] < 0 || dst[a] >= S ||
            pdf[a] < 0 || pdf[a] >= P)
            return 2;
    for (int b = 0; b < B; ++b)
        if (lengths[b] < 0 || lengths[b] > T) return 2;

    double *lpi = (double *)malloc(sizeof(double) * S);
    double *lf = (double *)malloc(sizeof(double) * S);
    if (!lpi || !lf) { free(lpi); free(lf); return 1; }
    for (int i = 0; i < S; ++i) {
        lpi[i] = init_prob[i] > 0.f ? log((double)init_prob[i]) : NEG_INF;
        lf[i] = final_prob[i] > 0.f ? log((double)final_prob[i]) : NEG_INF;
    }
    double leps = leak > 0.0 ? log(leak) : NEG_INF;
    int failed = 0;

#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int Tb = lengths[b];
        double *g = gamma ? gamma + (size_t)b * T * P : NULL;
        if (g)
            memset(g + (size_t)Tb * P, 0, sizeof(double) * (size_t)(T - Tb) * P);
        int rc = one_sequence(S, P, num_arcs, src, dst, pdf, logw, lpi, lf, leps,
                              Tb, logits + (size_t)b * T * P, &logz[b],
                              logz_bwd ? &logz_bwd[b] : NULL, g);
        if (rc) {
#pragma omp atomic write
            failed = 1;
        }
    }
    free(lpi); free(lf);
    return failed;
}

/* Number of threads the parallel loop above would use. */
int lfmmi_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
