/*
 * Host-side sanitizer run of the CPU oracle (TEST INFRASTRUCTURE, CPU only; never built for or run on a GPU).
 *
 * Built together with path_oracle.c under -fsanitize=address,undefined (see tests/test_oracle_sanitizers.py),
 * this driver calls every entry point of the oracle on small seeded inputs whose buffers are allocated with
 * their exact sizes, so that an out-of-bounds read or write, a use of freed memory, a leak or undefined
 * arithmetic in the oracle ends the run with a report and a non-zero status.  It checks no values: the
 * oracle's arithmetic is pinned elsewhere.  L includes 1 (empty walk), sizes that are no multiple of
 * anything, and row lists with repeated and boundary rows.
 */
#include <stdio.h>
#include <stdlib.h>

void path_oracle_fwd_rows(const double *q, const double *k, const double *v, const double *w, const double *beta,
                          const double *logf, const int *rows, int n_rows, double *o_rows, double *lse_rows,
                          int B, int H, int L, int d, double scale);
void path_oracle_fwd(const double *q, const double *k, const double *v, const double *w, const double *beta,
                     const double *logf, double *o, double *lse, int B, int H, int L, int d, double scale);
void path_oracle_logits(const double *q, const double *k, const double *w, const double *beta, double *S, int L, int d,
                        double scale);
void path_oracle_walk_norms(const double *q, const double *k, const double *w, const double *beta, int i, double *norms, int L, int d);
void path_oracle_bwd(const double *q, const double *k, const double *v, const double *w, const double *beta,
                     const double *logf, const double *dO, double *dq, double *dk, double *dv, double *dw, double *dbeta,
                     double *dlogf, int B, int H, int L, int d, double scale);
int path_oracle_num_threads(void);

static unsigned long long state = 88172645463325252ULL;
static double rnd(void)                  /* xorshift64, uniform in (-1, 1) */
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 4503599627370496.0 - 1.0;
}
static double *filled(size_t n, double lo, double hi)
{
    double *p = (double *)malloc(sizeof(double) * (n ? n : 1));
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    for (size_t i = 0; i < n; ++i) p[i] = lo + (hi - lo) * 0.5 * (rnd() + 1.0);
    return p;
}

static void one_case(int B, int H, int L, int d, int with_gates)
{
    const size_t n = (size_t)B * H * L * d, m = (size_t)B * H * L;
    double *q = filled(n, -1, 1), *k = filled(n, -1, 1), *v = filled(n, -1, 1), *w = filled(n, -0.5, 0.5), *dO = filled(n, -1, 1);
    double *beta = filled(m, 0, 2), *logf = with_gates ? filled(m, -1, 0) : NULL;
    double *o = filled(n, 0, 0), *lse = filled(m, 0, 0);
    path_oracle_fwd(q, k, v, w, beta, logf, o, lse, B, H, L, d, 0.37);
    int rows[5] = {0, L - 1, L / 2, L - 1, 0};
    double *orow = filled((size_t)B * H * 5 * d, 0, 0), *lrow = filled((size_t)B * H * 5, 0, 0);
    path_oracle_fwd_rows(q, k, v, w, beta, logf, rows, 5, orow, lrow, B, H, L, d, 0.37);
    double *S = filled((size_t)L * L, 0, 0), *nrm = filled((size_t)L, 0, 0);
    path_oracle_logits(q, k, w, beta, S, L, d, 1.0);               /* (first head only: one [L,d] problem) */
    path_oracle_walk_norms(q, k, w, beta, L - 1, nrm, L, d);
    path_oracle_walk_norms(q, k, w, beta, 0, nrm, L, d);
    double *dq = filled(n, 0, 0), *dk = filled(n, 0, 0), *dv = filled(n, 0, 0), *dw = filled(n, 0, 0);
    double *db = filled(m, 0, 0), *dl = with_gates ? filled(m, 0, 0) : NULL;
    path_oracle_bwd(q, k, v, w, beta, logf, dO, dq, dk, dv, dw, db, dl, B, H, L, d, 0.37);
    double acc = o[n - 1] + lse[m - 1] + orow[(size_t)B * H * 5 * d - 1] + S[(size_t)L * L - 1] + dq[0] + dk[n - 1] + dv[0] + dw[n - 1] + db[m - 1];
    if (acc != acc) { fprintf(stderr, "NaN in the oracle's output (B=%d H=%d L=%d d=%d)\n", B, H, L, d); exit(3); }
    free(q); free(k); free(v); free(w); free(dO); free(beta); free(logf); free(o); free(lse); free(orow); free(lrow);
    free(S); free(nrm); free(dq); free(dk); free(dv); free(dw); free(db); free(dl);
}

int main(void)
{
    one_case(1, 1, 1, 3, 0);
    one_case(1, 2, 2, 5, 1);
    one_case(2, 3, 37, 7, 0);
    one_case(1, 2, 65, 16, 1);
    printf("oracle sanitizer run: ok (%d threads)\n", path_oracle_num_threads());
    return 0;
}
