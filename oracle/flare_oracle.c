/*
 * flare_oracle.c -- plain fp64 CPU oracle for FLARE's encode-decode token mixer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct definition
 * that the HIP library is compared against.  It shares no code, header, table or
 * helper with the GPU path, and nothing on the product path may call it: only the
 * tests, the smoke check and the benchmark's cpu_baseline leg load it.
 *
 * What it computes (paper: Section 3.1 "FLARE", Eq. flare_encode / Eq. flare_decode;
 * per-latent and per-token forms in Appendix F; explicit weights in the paragraph
 * "Low-rank communication", Eq. attn_W, and the unfused listing of Appendix C):
 *
 *   per batch item b and head h, with  S[m][n] = scale * sum_j q[h][m][j] * k[b][h][n][j]
 *     encode:  Z[m][:] = sum_n softmax_n(S[m][.])[n] * v[n][:]      (softmax over the N tokens)
 *     decode:  Y[n][:] = sum_m softmax_m(S[.][n])[m] * Z[m][:]      (softmax over the M latents)
 *   `scale` is a multiplier on q.k (the paper's listing passes scale=1.0 to both calls).
 *
 * The fused method is an exact re-association of  Y = (W_dec . W_enc) . V, so the
 * oracle is that definition written out: two-pass softmax (max, then sum), plain
 * loops, fp64 everywhere, no blocking or reordering.  Scores are recomputed where
 * they are needed instead of being stored, which changes no arithmetic.
 *
 * Backward: the paper gives no derivation (it differentiates through the two
 * attention calls automatically).  The formulas below follow from the softmax
 * Jacobian applied to the two equations above; they are pinned in the tests by
 * central finite differences and by an autograd run of the paper's listing.
 *
 * Parity pins (tests/test_oracle_*.py): explicit W.V on tiny N, W row-stochastic /
 * non-negative / rank <= M, spectral identity of Appendix C.1 (Algorithm 1),
 * permutation equivariance, constant V, linearity in V, closed forms (Q=0, M=1,
 * N=1, duplicated tokens, one-hot cluster example with hand-computed rationals in
 * tests/golden/), shift invariance, finite differences and gradient identities.
 * No function here is "parity unpinned".
 *
 * All pointers are HOST pointers to fp64, contiguous, innermost dim d.
 * Return value: 0 on success, -1 on a bad argument.
 */
#include <math.h>
#include <stdlib.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int flare_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* S[m][n] for one head: scale * <q_m, k_n>   (Eq. flare_encode with SDPA's score) */
static double score(const double *q_m, const double *k_n, int d, double scale)
{
    double s = 0.0;
    for (int j = 0; j < d; ++j) s += q_m[j] * k_n[j];
    return scale * s;
}

/* Encode for one (b,h): Z[M][d], and the row statistics rmax[m] = max_n S[m][n],
 * rsum[m] = sum_n exp(S[m][n] - rmax[m]).   Appendix F, per-latent form of z_m. */
static void encode_head(int N, int M, int d, const double *q, const double *k, const double *v,
                        double scale, double *z, double *rmax, double *rsum)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        const double *q_m = q + (size_t)m * d;
        double mx = -INFINITY;
        for (int n = 0; n < N; ++n) {
            double s = score(q_m, k + (size_t)n * d, d, scale);
            if (s > mx) mx = s;
        }
        double sum = 0.0;
        double *z_m = z + (size_t)m * d;
        for (int j = 0; j < d; ++j) z_m[j] = 0.0;
        for (int n = 0; n < N; ++n) {
            double e = exp(score(q_m, k + (size_t)n * d, d, scale) - mx);
            sum += e;
            const double *v_n = v + (size_t)n * d;
            for (int j = 0; j < d; ++j) z_m[j] += e * v_n[j];
        }
        for (int j = 0; j < d; ++j) z_m[j] /= sum;
        rmax[m] = mx;
        rsum[m] = sum;
    }
}

/* Column statistics of one token n: cmax = max_m S[m][n], csum = sum_m exp(S[m][n]-cmax). */
static void token_stats(int M, int d, const double *q, const double *k_n, double scale,
                        double *cmax, double *csum)
{
    double mx = -INFINITY;
    for (int m = 0; m < M; ++m) {
        double s = score(q + (size_t)m * d, k_n, d, scale);
        if (s > mx) mx = s;
    }
    double sum = 0.0;
    for (int m = 0; m < M; ++m) sum += exp(score(q + (size_t)m * d, k_n, d, scale) - mx);
    *cmax = mx;
    *csum = sum;
}

/* Decode of one token: y_n[:] = sum_m R[n][m] Z[m][:].   Appendix F, per-token form of y_n. */
static void decode_token(int M, int d, const double *q, const double *k_n, const double *z,
                         double scale, double *y_n)
{
    double cmax, csum;
    token_stats(M, d, q, k_n, scale, &cmax, &csum);
    for (int j = 0; j < d; ++j) y_n[j] = 0.0;
    for (int m = 0; m < M; ++m) {
        double r = exp(score(q + (size_t)m * d, k_n, d, scale) - cmax) / csum;
        const double *z_m = z + (size_t)m * d;
        for (int j = 0; j < d; ++j) y_n[j] += r * z_m[j];
    }
}

/*
 * Forward of the multi-head mixer (listing in Section 3.1: Q:[H M D], K,V:[B H N D] -> Y:[B H N D]).
 *   q[H][M][d], k,v[B][H][N][d]
 *   z[B][H][M][d], lse_enc[B][H][M] = log sum_n exp(S[m][n])   (either may be NULL)
 *   tok == NULL : y is [B][H][N][d], every token decoded
 *   tok != NULL : y is [B][H][n_tok][d], row i holds token tok[i] (0 <= tok[i] < N)
 */
int flare_oracle_forward(int B, int H, int N, int M, int d,
                         const double *q, const double *k, const double *v, double scale,
                         const long long *tok, int n_tok,
                         double *y, double *z, double *lse_enc)
{
    if (B < 1 || H < 1 || N < 1 || M < 1 || d < 1 || !q || !k || !v || !y) return -1;
    if (tok) {
        if (n_tok < 1) return -1;
        for (int i = 0; i < n_tok; ++i) if (tok[i] < 0 || tok[i] >= N) return -1;
    }
    const int n_out = tok ? n_tok : N;
    double *zbuf = (double *)malloc(sizeof(double) * (size_t)M * d);
    double *rmax = (double *)malloc(sizeof(double) * (size_t)M);
    double *rsum = (double *)malloc(sizeof(double) * (size_t)M);
    if (!zbuf || !rmax || !rsum) { free(zbuf); free(rmax); free(rsum); return -1; }

    for (int b = 0; b < B; ++b) for (int h = 0; h < H; ++h) {
        const size_t bh = (size_t)b * H + h;
        const double *q_h = q + (size_t)h * M * d;
        const double *k_bh = k + bh * N * d;
        const double *v_bh = v + bh * N * d;
        double *y_bh = y + bh * n_out * d;

        encode_head(N, M, d, q_h, k_bh, v_bh, scale, zbuf, rmax, rsum);
        if (z) for (size_t i = 0; i < (size_t)M * d; ++i) z[bh * M * d + i] = zbuf[i];
        if (lse_enc) for (int m = 0; m < M; ++m) lse_enc[bh * M + m] = rmax[m] + log(rsum[m]);

#pragma omp parallel for schedule(static)
        for (int i = 0; i < n_out; ++i) {
            const size_t n = tok ? (size_t)tok[i] : (size_t)i;
            decode_token(M, d, q_h, k_bh + n * d, zbuf, scale, y_bh + (size_t)i * d);
        }
    }
    free(zbuf); free(rmax); free(rsum);
    return 0;
}

/*
 * Backward of the mixer.  With P = W_enc (M x N, rows sum to 1), R = W_dec (N x M, rows
 * sum to 1), Z = P V, Y = R Z and upstream dY:
 *     dZ[m]      = sum_n R[n][m] dY[n]
 *     delta[n]   = <dY[n], Y[n]>                 eps[m] = <dZ[m], Z[m]>
 *     dV[n]      = sum_m P[m][n] dZ[m]
 *     dS[m][n]   = P[m][n] (<dZ[m], V[n]> - eps[m])  +  R[n][m] (<dY[n], Z[m]> - delta[n])
 *     dK[n]      = scale * sum_m dS[m][n] q[m]
 *     dQ[m]      = scale * sum_n dS[m][n] k[n],   summed over the batch (Q is shared over it)
 *
 *   dy[B][H][N][d] (always full);  dq[H][M][d] (overwritten)
 *   tok == NULL : dk, dv are [B][H][N][d];  else [B][H][n_tok][d] for the listed tokens.
 *   dk and dv may be NULL (then only dq is produced).
 */
int flare_oracle_backward(int B, int H, int N, int M, int d,
                          const double *q, const double *k, const double *v, const double *dy,
                          double scale, const long long *tok, int n_tok,
                          double *dq, double *dk, double *dv)
{
    if (B < 1 || H < 1 || N < 1 || M < 1 || d < 1 || !q || !k || !v || !dy || !dq) return -1;
    if ((dk == NULL) != (dv == NULL)) return -1;
    if (tok) {
        if (n_tok < 1) return -1;
        for (int i = 0; i < n_tok; ++i) if (tok[i] < 0 || tok[i] >= N) return -1;
    }
    const int n_out = tok ? n_tok : N;
    const size_t Md = (size_t)M * d;
    double *z = (double *)malloc(sizeof(double) * Md);
    double *dz = (double *)malloc(sizeof(double) * Md);
    double *rmax = (double *)malloc(sizeof(double) * (size_t)M);
    double *rsum = (double *)malloc(sizeof(double) * (size_t)M);
    double *eps = (double *)malloc(sizeof(double) * (size_t)M);
    double *cmax = (double *)malloc(sizeof(double) * (size_t)N);
    double *csum = (double *)malloc(sizeof(double) * (size_t)N);
    double *delta = (double *)malloc(sizeof(double) * (size_t)N);
    if (!z || !dz || !rmax || !rsum || !eps || !cmax || !csum || !delta) {
        free(z); free(dz); free(rmax); free(rsum); free(eps); free(cmax); free(csum); free(delta);
        return -1;
    }
    for (size_t i = 0; i < (size_t)H * Md; ++i) dq[i] = 0.0;

    for (int b = 0; b < B; ++b) for (int h = 0; h < H; ++h) {
        const size_t bh = (size_t)b * H + h;
        const double *q_h = q + (size_t)h * Md;
        const double *k_bh = k + bh * N * d;
        const double *v_bh = v + bh * N * d;
        const double *dy_bh = dy + bh * N * d;

        /* forward quantities */
        encode_head(N, M, d, q_h, k_bh, v_bh, scale, z, rmax, rsum);
#pragma omp parallel for schedule(static)
        for (int n = 0; n < N; ++n) {
            const double *k_n = k_bh + (size_t)n * d;
            token_stats(M, d, q_h, k_n, scale, &cmax[n], &csum[n]);
            double dl = 0.0;                       /* delta[n] = <dY[n], Y[n]> */
            for (int m = 0; m < M; ++m) {
                double r = exp(score(q_h + (size_t)m * d, k_n, d, scale) - cmax[n]) / csum[n];
                double t = 0.0;
                for (int j = 0; j < d; ++j) t += dy_bh[(size_t)n * d + j] * z[(size_t)m * d + j];
                dl += r * t;
            }
            delta[n] = dl;
        }
        /* dZ = R^T dY, eps */
#pragma omp parallel for schedule(static)
        for (int m = 0; m < M; ++m) {
            double *dz_m = dz + (size_t)m * d;
            for (int j = 0; j < d; ++j) dz_m[j] = 0.0;
            for (int n = 0; n < N; ++n) {
                double r = exp(score(q_h + (size_t)m * d, k_bh + (size_t)n * d, d, scale) - cmax[n]) / csum[n];
                for (int j = 0; j < d; ++j) dz_m[j] += r * dy_bh[(size_t)n * d + j];
            }
            double e = 0.0;
            for (int j = 0; j < d; ++j) e += dz_m[j] * z[(size_t)m * d + j];
            eps[m] = e;
        }
        /* dK, dV for the requested tokens */
        if (dk) {
#pragma omp parallel for schedule(static)
            for (int i = 0; i < n_out; ++i) {
                const size_t n = tok ? (size_t)tok[i] : (size_t)i;
                const double *k_n = k_bh + n * d, *v_n = v_bh + n * d, *dy_n = dy_bh + n * d;
                double *dk_n = dk + (bh * n_out + (size_t)i) * d;
                double *dv_n = dv + (bh * n_out + (size_t)i) * d;
                for (int j = 0; j < d; ++j) { dk_n[j] = 0.0; dv_n[j] = 0.0; }
                for (int m = 0; m < M; ++m) {
                    const double *q_m = q_h + (size_t)m * d, *z_m = z + (size_t)m * d, *dz_m = dz + (size_t)m * d;
                    double s = score(q_m, k_n, d, scale);
                    double p = exp(s - rmax[m]) / rsum[m];
                    double r = exp(s - cmax[n]) / csum[n];
                    double a = 0.0, c = 0.0;
                    for (int j = 0; j < d; ++j) { a += dz_m[j] * v_n[j]; c += dy_n[j] * z_m[j]; }
                    double ds = p * (a - eps[m]) + r * (c - delta[n]);
                    for (int j = 0; j < d; ++j) { dk_n[j] += scale * ds * q_m[j]; dv_n[j] += p * dz_m[j]; }
                }
            }
        }
        /* dQ, accumulated over the batch in b order */
#pragma omp parallel for schedule(static)
        for (int m = 0; m < M; ++m) {
            const double *q_m = q_h + (size_t)m * d, *z_m = z + (size_t)m * d, *dz_m = dz + (size_t)m * d;
            double acc[256];
            double *g = (d <= 256) ? acc : (double *)malloc(sizeof(double) * (size_t)d);
            for (int j = 0; j < d; ++j) g[j] = 0.0;
            for (int n = 0; n < N; ++n) {
                const double *k_n = k_bh + (size_t)n * d, *v_n = v_bh + (size_t)n * d, *dy_n = dy_bh + (size_t)n * d;
                double s = score(q_m, k_n, d, scale);
                double p = exp(s - rmax[m]) / rsum[m];
                double r = exp(s - cmax[n]) / csum[n];
                double a = 0.0, c = 0.0;
                for (int j = 0; j < d; ++j) { a += dz_m[j] * v_n[j]; c += dy_n[j] * z_m[j]; }
                double ds = p * (a - eps[m]) + r * (c - delta[n]);
                for (int j = 0; j < d; ++j) g[j] += scale * ds * k_n[j];
            }
            for (int j = 0; j < d; ++j) dq[(size_t)h * Md + (size_t)m * d + j] += g[j];
            if (g != acc) free(g);
        }
    }
    free(z); free(dz); free(rmax); free(rsum); free(eps); free(cmax); free(csum); free(delta);
    return 0;
}

/*
 * Explicit weights of one head (paragraph "Low-rank communication", Eq. attn_W; unfused
 * listing of Appendix C):  w_enc[M][N] = softmax over n of S,  w_dec[N][M] = softmax over m
 * of S^T,  w[N][N] = w_dec . w_enc.  Tiny N only: O(N^2 M) time, O(N^2) memory.
 * Any of the three outputs may be NULL.
 */
int flare_oracle_explicit_w(int N, int M, int d, const double *q, const double *k, double scale,
                            double *w_enc, double *w_dec, double *w)
{
    if (N < 1 || M < 1 || d < 1 || !q || !k) return -1;
    double *s = (double *)malloc(sizeof(double) * (size_t)M * N);
    double *we = (double *)malloc(sizeof(double) * (size_t)M * N);
    double *wd = (double *)malloc(sizeof(double) * (size_t)N * M);
    if (!s || !we || !wd) { free(s); free(we); free(wd); return -1; }
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n)
            s[(size_t)m * N + n] = score(q + (size_t)m * d, k + (size_t)n * d, d, scale);
    for (int m = 0; m < M; ++m) {                     /* softmax along each row of S */
        double mx = -INFINITY, sum = 0.0;
        for (int n = 0; n < N; ++n) if (s[(size_t)m * N + n] > mx) mx = s[(size_t)m * N + n];
        for (int n = 0; n < N; ++n) sum += exp(s[(size_t)m * N + n] - mx);
        for (int n = 0; n < N; ++n) we[(size_t)m * N + n] = exp(s[(size_t)m * N + n] - mx) / sum;
    }
    for (int n = 0; n < N; ++n) {                     /* softmax along each row of S^T */
        double mx = -INFINITY, sum = 0.0;
        for (int m = 0; m < M; ++m) if (s[(size_t)m * N + n] > mx) mx = s[(size_t)m * N + n];
        for (int m = 0; m < M; ++m) sum += exp(s[(size_t)m * N + n] - mx);
        for (int m = 0; m < M; ++m) wd[(size_t)n * M + m] = exp(s[(size_t)m * N + n] - mx) / sum;
    }
    if (w_enc) for (size_t i = 0; i < (size_t)M * N; ++i) w_enc[i] = we[i];
    if (w_dec) for (size_t i = 0; i < (size_t)N * M; ++i) w_dec[i] = wd[i];
    if (w) {
        for (int a = 0; a < N; ++a)
            for (int c = 0; c < N; ++c) {
                double t = 0.0;
                for (int m = 0; m < M; ++m) t += wd[(size_t)a * M + m] * we[(size_t)m * N + c];
                w[(size_t)a * N + c] = t;
            }
    }
    free(s); free(we); free(wd);
    return 0;
}
