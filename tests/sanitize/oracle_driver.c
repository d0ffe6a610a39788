/* Driver for the address / undefined-behaviour sanitizer run of the fp64 oracle (tests/test_oracle_sanitize.py):
 * calls every exported function of oracle/flare_oracle.c on small shapes that touch its edge cases -- one token,
 * one latent, token subsets (first, last, repeated index), several batch items and heads -- with every array
 * allocated at its exact size, so that an access one element past any of them is reported.  Prints "ok". */
#include <stdio.h>
#include <stdlib.h>

int flare_oracle_threads(void);
int flare_oracle_forward(int B, int H, int N, int M, int d, const double *q, const double *k, const double *v,
                         double scale, const long long *tok, int n_tok, double *y, double *z, double *lse);
int flare_oracle_backward(int B, int H, int N, int M, int d, const double *q, const double *k, const double *v,
                          const double *dy, double scale, const long long *tok, int n_tok, double *dq, double *dk,
                          double *dv);
int flare_oracle_explicit_w(int N, int M, int d, const double *q, const double *k, double scale, double *we,
                            double *wd, double *w);

static double *filled(size_t n, unsigned seed)
{
    double *p = (double *)malloc(n * sizeof(double));
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    for (size_t i = 0; i < n; ++i) {
        seed = seed * 1664525u + 1013904223u;
        p[i] = ((double)(seed >> 8) / (double)(1u << 24) - 0.5) * 3.0;
    }
    return p;
}

static int run(int B, int H, int N, int M, int d, const long long *tok, int n_tok)
{
    const size_t nq = (size_t)H * M * d, nk = (size_t)B * H * N * d;
    const size_t n_out = (size_t)B * H * (tok ? n_tok : N) * d;
    double *q = filled(nq, 1), *k = filled(nk, 2), *v = filled(nk, 3), *dy = filled(nk, 4);
    double *y = filled(n_out, 5), *z = filled((size_t)B * H * M * d, 6), *lse = filled((size_t)B * H * M, 7);
    double *dq = filled(nq, 8), *dk = filled(n_out, 9), *dv = filled(n_out, 10);
    int rc = flare_oracle_forward(B, H, N, M, d, q, k, v, 0.37, tok, n_tok, y, z, lse);
    if (rc == 0) rc = flare_oracle_backward(B, H, N, M, d, q, k, v, dy, 0.37, tok, n_tok, dq, dk, dv);
    if (rc == 0) rc = flare_oracle_backward(B, H, N, M, d, q, k, v, dy, 0.37, tok, n_tok, dq, NULL, NULL);
    free(q); free(k); free(v); free(dy); free(y); free(z); free(lse); free(dq); free(dk); free(dv);
    return rc;
}

int main(void)
{
    const long long some[4] = {0, 6, 6, 2}, last[1] = {6};
    int rc = 0;
    if (flare_oracle_threads() < 1) return 3;
    rc |= run(1, 1, 1, 1, 4, NULL, 0);          /* one token, one latent */
    rc |= run(2, 3, 7, 5, 8, NULL, 0);
    rc |= run(2, 3, 7, 5, 8, some, 4);          /* token subset with a repeated and the last index */
    rc |= run(1, 2, 7, 1, 16, last, 1);
    rc |= run(3, 1, 33, 40, 32, NULL, 0);
    {
        const int N = 6, M = 3, d = 4;
        double *q = filled((size_t)M * d, 11), *k = filled((size_t)N * d, 12);
        double *we = filled((size_t)M * N, 13), *wd = filled((size_t)N * M, 14), *w = filled((size_t)N * N, 15);
        rc |= flare_oracle_explicit_w(N, M, d, q, k, 1.0, we, wd, w);
        free(q); free(k); free(we); free(wd); free(w);
    }
    if (rc != 0) { fprintf(stderr, "an oracle call failed: %d\n", rc); return 1; }
    printf("ok\n");
    return 0;
}
