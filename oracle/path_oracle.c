/*
 * PaTH attention -- CPU oracle (TEST INFRASTRUCTURE, not part of the product).
 *
 * A plain, slow, fp64 implementation of what the GPU library computes, written
 * directly from the paper's definition.  Only the tests, the smoke check and
 * the benchmark's CPU-baseline leg may call it.  It shares no code, header,
 * table or helper with the HIP kernels.
 *
 * What it computes (paper Sec. 2.1 multiplicative-position-encoding formula,
 * Sec. 2.2 transition H_t = I - beta_t w_t w_t^T and the "PaTH:" output
 * formula with its normaliser Z_t):
 *
 *     s_ij = scale * k_j^T (H_{j+1} ... H_i) q_i          for j <= i
 *     o_i  = sum_{j<=i} softmax_j(s_ij) v_j ,   lse_i = log sum_j exp(s_ij)
 *
 * The product is evaluated the way the definition reads from the query's
 * side: start from u = q_i, take the logit against k_j, then move one token
 * to the left by u <- H_j u.  H_i therefore acts on the query first, which is
 * the order fixed jointly by the RNN recurrence S_t = S_{t-1} H_t + v_t k_t^T
 * (Sec. 2.2), the boxed full-matrix form (Sec. 3.1) and the in-place key-cache
 * update (Sec. 3.4, Eq. 1).  The empty product (j = i) is the identity.
 * `scale` is not in the paper (its logits are unscaled); it multiplies the
 * finished bilinear form.  w is used as given (no normalisation), beta is
 * used as given (no clipping).
 *
 * The paper gives no backward pass.  path_oracle_bwd is the reverse-mode
 * derivative of exactly the walk above, derived by hand (see the comment on
 * the function) and pinned by finite differences of path_oracle_fwd and by an
 * independent autograd model in the tests.
 *
 * PaTH-FoX (the paper's "Extension: PaTH-FoX" paragraph in Sec. 2.2): with forget gates
 * f_s in (0,1) the attention weight gets the extra factor prod_{s=j+1..i} f_s, i.e. the
 * logit gets + sum_{s=j+1..i} log f_s (outside `scale`: the paper adds it to the finished
 * logit).  Every function takes `logf` ([B,H,L], the LOG of the gates, NULL = no gates); the
 * walk adds the running sum as it moves left.  Backward: with zbar_ij = p_ij (dO_i.v_j -
 * delta_i) the gradient of the total logit, dlogf_s = sum_{j < s <= i} zbar_ij.
 *
 * Layout: q,k,v,w,o,dO and gradients [B,H,L,d] contiguous; beta, lse, dbeta, logf, dlogf
 * [B,H,L].  Everything is double.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int path_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double dot(const double *a, const double *b, int d)
{
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += a[c] * b[c];
    return s;
}

/* One query row of one head.  s (length i+1) receives the scaled logits;
 * if `states` is non-NULL, states[j*d .. j*d+d) receives the walk vector u
 * as it stood when the logit against k_j was taken (u^{(i)} = q_i). */
static void walk_row(const double *q_i, const double *K, const double *W,
                     const double *beta, const double *logf, int i, int d, double scale,
                     double *s, double *u, double *states)
{
    double bias = 0.0;      /* sum_{s=j+1..i} log f_s: empty for j = i */
    memcpy(u, q_i, sizeof(double) * (size_t)d);
    for (int j = i; j >= 0; --j) {
        const double *kj = K + (size_t)j * d;
        const double *wj = W + (size_t)j * d;
        if (states) memcpy(states + (size_t)j * d, u, sizeof(double) * (size_t)d);
        s[j] = scale * dot(u, kj, d) + bias;
        if (logf) bias += logf[j];
        /* u <- H_j u = u - beta_j (w_j . u) w_j   (Sec. 2.2) */
        double a = beta[j] * dot(wj, u, d);
        for (int c = 0; c < d; ++c) u[c] -= a * wj[c];
    }
}

/* Softmax statistics of one row: returns lse, fills p with exp(s - lse). */
static double softmax_row(const double *s, int n, double *p)
{
    double m = s[0];
    for (int j = 1; j < n; ++j) if (s[j] > m) m = s[j];
    double z = 0.0;
    for (int j = 0; j < n; ++j) z += exp(s[j] - m);
    double lse = m + log(z);
    for (int j = 0; j < n; ++j) p[j] = exp(s[j] - lse);
    return lse;
}

/* Forward for a list of query rows of every (b,h).
 * rows[n_rows] are token indices in [0,L); o_rows is [B,H,n_rows,d],
 * lse_rows is [B,H,n_rows].  Rows are independent, so a sample of rows is
 * exact for those rows. */
void path_oracle_fwd_rows(const double *q, const double *k, const double *v,
                          const double *w, const double *beta, const double *logf,
                          const int *rows, int n_rows,
                          double *o_rows, double *lse_rows,
                          int B, int H, int L, int d, double scale)
{
    const long BH = (long)B * H;
    const long total = BH * n_rows;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)L);
        double *p = (double *)malloc(sizeof(double) * (size_t)L);
        double *u = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 4)
        for (long it = 0; it < total; ++it) {
            long bh = it / n_rows;
            int r = (int)(it % n_rows);
            int i = rows[r];
            const double *Q = q + bh * L * d, *K = k + bh * L * d;
            const double *V = v + bh * L * d, *W = w + bh * L * d;
            const double *Bt = beta + bh * L;
            const double *Lf = logf ? logf + bh * L : NULL;
            walk_row(Q + (size_t)i * d, K, W, Bt, Lf, i, d, scale, s, u, NULL);
            double lse = softmax_row(s, i + 1, p);
            double *oi = o_rows + (bh * n_rows + r) * d;
            for (int c = 0; c < d; ++c) oi[c] = 0.0;
            for (int j = 0; j <= i; ++j) {
                const double *vj = V + (size_t)j * d;
                for (int c = 0; c < d; ++c) oi[c] += p[j] * vj[c];
            }
            lse_rows[bh * n_rows + r] = lse;
        }
        free(s); free(p); free(u);
    }
}

/* Full forward: every row. */
void path_oracle_fwd(const double *q, const double *k, const double *v,
                     const double *w, const double *beta, const double *logf,
                     double *o, double *lse,
                     int B, int H, int L, int d, double scale)
{
    int *rows = (int *)malloc(sizeof(int) * (size_t)L);
    for (int i = 0; i < L; ++i) rows[i] = i;
    path_oracle_fwd_rows(q, k, v, w, beta, logf, rows, L, o, lse, B, H, L, d, scale);
    free(rows);
}

/* Dense scaled logits of one head ([L,L], upper triangle set to 0) -- for
 * small-L checks against explicit matrix products and printed closed forms. */
void path_oracle_logits(const double *q, const double *k, const double *w,
                        const double *beta, double *S, int L, int d, double scale)
{
    double *s = (double *)malloc(sizeof(double) * (size_t)L);
    double *u = (double *)malloc(sizeof(double) * (size_t)d);
    for (int i = 0; i < L; ++i) {
        walk_row(q + (size_t)i * d, k, w, beta, NULL, i, d, scale, s, u, NULL);
        for (int j = 0; j < L; ++j) S[(size_t)i * L + j] = (j <= i) ? s[j] : 0.0;
    }
    free(s); free(u);
}

/* Euclidean norm of the walk vector of query row i of one head at every
 * position: norms[j] = || u^{(j)} ||, j = i..0 (entries j > i left at 0). */
void path_oracle_walk_norms(const double *q, const double *k, const double *w,
                            const double *beta, int i, double *norms,
                            int L, int d)
{
    double *s = (double *)malloc(sizeof(double) * (size_t)L);
    double *u = (double *)malloc(sizeof(double) * (size_t)d);
    double *st = (double *)malloc(sizeof(double) * (size_t)L * d);
    walk_row(q + (size_t)i * d, k, w, beta, NULL, i, d, 1.0, s, u, st);
    for (int j = 0; j < L; ++j)
        norms[j] = (j <= i) ? sqrt(dot(st + (size_t)j * d, st + (size_t)j * d, d)) : 0.0;
    free(s); free(u); free(st);
}

/*
 * Backward of loss = sum_i dO_i . o_i  with respect to q, k, v, w, beta.
 *
 * Not in the paper; reverse-mode derivative of the walk.  With
 *   p_ij = exp(s_ij - lse_i),  delta_i = dO_i . o_i,
 *   g_ij = d loss / d(u^{(j)} . k_j) = scale * p_ij (dO_i . v_j - delta_i),
 * and walk states u^{(i)} = q_i, u^{(t-1)} = H_t u^{(t)}:
 *   dv_j += p_ij dO_i ;   dk_j += g_ij u^{(j)}
 * and the adjoint of the walk vector runs back up from j = 0 to j = i:
 *   ubar^{(0)} = g_i0 k_0
 *   for t = 1..i:   (u^{(t-1)} = u^{(t)} - beta_t (w_t.u^{(t)}) w_t)
 *       a = w_t . ubar^{(t-1)},  b = w_t . u^{(t)}
 *       dbeta_t -= a b
 *       dw_t    -= beta_t (b ubar^{(t-1)} + a u^{(t)})
 *       ubar^{(t)} = ubar^{(t-1)} - beta_t a w_t + g_it k_t
 *   dq_i = ubar^{(i)}
 * H_0 never enters a logit that is used, so dw_0 = dbeta_0 = 0.
 * With gates (logf != NULL) the logits carry the running sum of log f and, with
 * zbar_ij = g_ij / scale, dlogf_s = sum_i sum_{j<s<=i} zbar_ij (dlogf_0 = 0).
 */
void path_oracle_bwd(const double *q, const double *k, const double *v,
                     const double *w, const double *beta, const double *logf, const double *dO,
                     double *dq, double *dk, double *dv, double *dw, double *dbeta, double *dlogf,
                     int B, int H, int L, int d, double scale)
{
    const long BH = (long)B * H;
    const size_t Ld = (size_t)L * d;
    memset(dq, 0, sizeof(double) * BH * Ld);
    memset(dk, 0, sizeof(double) * BH * Ld);
    memset(dv, 0, sizeof(double) * BH * Ld);
    memset(dw, 0, sizeof(double) * BH * Ld);
    memset(dbeta, 0, sizeof(double) * BH * (size_t)L);
    if (dlogf) memset(dlogf, 0, sizeof(double) * BH * (size_t)L);

    for (long bh = 0; bh < BH; ++bh) {
        const double *Q = q + bh * Ld, *K = k + bh * Ld, *V = v + bh * Ld;
        const double *W = w + bh * Ld, *Bt = beta + bh * L, *DO = dO + bh * Ld;
        double *DQ = dq + bh * Ld, *DK = dk + bh * Ld, *DV = dv + bh * Ld;
        double *DW = dw + bh * Ld, *DB = dbeta + bh * L;
        const double *Lf = logf ? logf + bh * L : NULL;
        double *DLF = (logf && dlogf) ? dlogf + bh * L : NULL;
#pragma omp parallel
        {
            double *s = (double *)malloc(sizeof(double) * (size_t)L);
            double *p = (double *)malloc(sizeof(double) * (size_t)L);
            double *g = (double *)malloc(sizeof(double) * (size_t)L);
            double *u = (double *)malloc(sizeof(double) * (size_t)d);
            double *ub = (double *)malloc(sizeof(double) * (size_t)d);
            double *oi = (double *)malloc(sizeof(double) * (size_t)d);
            double *st = (double *)malloc(sizeof(double) * Ld);
            double *tk = (double *)calloc(Ld, sizeof(double));
            double *tv = (double *)calloc(Ld, sizeof(double));
            double *tw = (double *)calloc(Ld, sizeof(double));
            double *tb = (double *)calloc((size_t)L, sizeof(double));
            double *tf = (double *)calloc((size_t)L, sizeof(double));
#pragma omp for schedule(dynamic, 4)
            for (int ii = 0; ii < L; ++ii) {
                int i = L - 1 - ii; /* longest rows first */
                walk_row(Q + (size_t)i * d, K, W, Bt, Lf, i, d, scale, s, u, st);
                softmax_row(s, i + 1, p);
                const double *doi = DO + (size_t)i * d;
                for (int c = 0; c < d; ++c) oi[c] = 0.0;
                for (int j = 0; j <= i; ++j)
                    for (int c = 0; c < d; ++c) oi[c] += p[j] * V[(size_t)j * d + c];
                double delta = dot(doi, oi, d);
                for (int j = 0; j <= i; ++j) {
                    g[j] = scale * p[j] * (dot(doi, V + (size_t)j * d, d) - delta);
                    for (int c = 0; c < d; ++c) {
                        tv[(size_t)j * d + c] += p[j] * doi[c];
                        tk[(size_t)j * d + c] += g[j] * st[(size_t)j * d + c];
                    }
                }
                for (int c = 0; c < d; ++c) ub[c] = g[0] * K[c];
                for (int t = 1; t <= i; ++t) {
                    const double *wt = W + (size_t)t * d;
                    const double *ut = st + (size_t)t * d;
                    const double *kt = K + (size_t)t * d;
                    double a = dot(wt, ub, d), b = dot(wt, ut, d);
                    tb[t] -= a * b;
                    for (int c = 0; c < d; ++c) {
                        tw[(size_t)t * d + c] -= Bt[t] * (b * ub[c] + a * ut[c]);
                        ub[c] += -Bt[t] * a * wt[c] + g[t] * kt[c];
                    }
                }
                memcpy(DQ + (size_t)i * d, ub, sizeof(double) * (size_t)d);
                if (DLF) {      /* gate s sits on the path of every pair (i, j) with j < s <= i */
                    double csum = 0.0;
                    for (int sgate = 1; sgate <= i; ++sgate) {
                        csum += g[sgate - 1] / scale;
                        tf[sgate] += csum;
                    }
                }
            }
#pragma omp critical
            {
                for (size_t x = 0; x < Ld; ++x) { DK[x] += tk[x]; DV[x] += tv[x]; DW[x] += tw[x]; }
                for (int t = 0; t < L; ++t) DB[t] += tb[t];
                if (DLF) for (int t = 0; t < L; ++t) DLF[t] += tf[t];
            }
            free(s); free(p); free(g); free(u); free(ub); free(oi);
            free(st); free(tk); free(tv); free(tw); free(tb); free(tf);
        }
    }
}
