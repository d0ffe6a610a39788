// Spectral analysis of the mixing matrix W = W_dec W_enc of one (b,h) (Appendix C.1, Algorithm 1):
// the nonzero eigenvalues of the N x N matrix W are those of the M x M matrix
//     G = J J^T,   J = L_M^(1/2) A L_N^(1/2),   A = exp(scale * Q K^T),
// and its eigenvectors are L_N^(1/2) J^T U Sigma^(-1) = W_dec (L_M^(1/2) U Sigma^(-1)): the decode
// applied to an M x M "latent sequence".  With lse_enc = log row sums of A and lse_dec = log column
// sums (what the forward leaves behind),  J[m][n] = exp(S[m][n] - (lse_enc[m] + lse_dec[n]) / 2).
//
// Steps here:  G as a streaming reduction over the tokens (matrix-core kernel in flare_mfma_fwd.hip,
// or the fp32 kernel below), a fixed-order sum of the per-chunk partials, a symmetric eigensolver in fp64
// (one workgroup per (b,h): Householder tridiagonalisation, bisection for the eigenvalues, a twisted factorisation
// for each of the d eigenvectors that were asked for, and the reflectors applied to those), and a last kernel that
// forms the decode-ready block L_M^(1/2) U Sigma^(-1) of those eigenvectors.
#include <stdlib.h>

#include "flare_internal.h"

namespace flare {
namespace {

typedef uint16_t bf16_t;
struct f16_t { uint16_t bits; };
__device__ __forceinline__ float elem(const f16_t *p, size_t i) { return (float)reinterpret_cast<const _Float16 *>(p)[i]; }
__device__ __forceinline__ float elem(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float elem(const bf16_t *p, size_t i) { return __uint_as_float((uint32_t)p[i] << 16); }

inline int check_launch() { return hipGetLastError() == hipSuccess ? FLARE_OK : FLARE_ELAUNCH; }

// ---- G partials on the vector ALUs (any M, any d, f32 or bf16 storage) -----------------------------
// Workgroup = (token chunk, b*h, block of 16 rows of G).  Per token the workgroup forms the column
// J[.][n] in LDS (thread t takes the latents t, t + 256, ...), then thread (r, c) adds
// J[row0 + r][n] * J[c + 16 i][n] to its accumulators, i < ceil(M / 16) <= kGramCols.
constexpr int kGramCols = 32;   // M <= 512 on this path
template <typename T>
__global__ __launch_bounds__(256) void gram_valu_kernel(
    const T *__restrict__ q, const T *__restrict__ k, const float *__restrict__ lse_enc,
    const float *__restrict__ lse_dec, float *__restrict__ g_part, TokStride ts, int H, int N, int M, int d,
    int chunk_len, int chunks, float scale)
{
    extern __shared__ float jcol[];   // M floats
    const int tid = threadIdx.x, r = tid >> 4, c = tid & 15;
    const int bh = blockIdx.y, h = bh % H, chunk = blockIdx.x, row0 = 16 * blockIdx.z;
    const int n0 = chunk * chunk_len, n1 = min(N, n0 + chunk_len);
    const T *kb = k + (size_t)(bh / H) * (size_t)ts.sb + (size_t)(bh % H) * (size_t)ts.sh;
    float acc[kGramCols];
#pragma unroll
    for (int i = 0; i < kGramCols; ++i) acc[i] = 0.f;
    const int ncol = (M + 15) / 16;
    for (int n = n0; n < n1; ++n) {
        const T *kr = kb + (size_t)n * (size_t)ts.sn;
        const float hd = 0.5f * lse_dec[(size_t)bh * N + n];
        for (int m = tid; m < M; m += 256) {
            const T *qr = q + (size_t)h * ts.sq + (size_t)m * d;
            float s = 0.f;
            for (int j = 0; j < d; ++j) s = fmaf(elem(qr, j), elem(kr, j), s);
            jcol[m] = __expf(scale * s - 0.5f * lse_enc[(size_t)bh * M + m] - hd);
        }
        __syncthreads();
        const float mine = (row0 + r < M) ? jcol[row0 + r] : 0.f;
#pragma unroll
        for (int i = 0; i < kGramCols; ++i)
            if (i < ncol && c + 16 * i < M) acc[i] = fmaf(mine, jcol[c + 16 * i], acc[i]);
        __syncthreads();
    }
    if (row0 + r < M) {
        float *out = g_part + (((size_t)bh * chunks + chunk) * M + row0 + r) * M;
#pragma unroll
        for (int i = 0; i < kGramCols; ++i)
            if (i < ncol && c + 16 * i < M) out[c + 16 * i] = acc[i];
    }
}

// ---- fixed-order sum of the partials: G in fp32 (optional output) and in fp64 for the solver ----------
__global__ __launch_bounds__(256) void gram_reduce_kernel(const float *__restrict__ g_part, float *__restrict__ gram,
                                                          double *__restrict__ a, int chunks, size_t mm, size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const size_t bh = i / mm, e = i % mm;
    double s = 0.0;
    for (int c = 0; c < chunks; ++c) s += (double)g_part[(bh * chunks + c) * mm + e];
    a[i] = s;
    if (gram) gram[i] = (float)s;
}

// ---- symmetric eigensolver, fp64, one workgroup per matrix ------------------------------------------------
// G = Q T Q^T by Householder reflections (T tridiagonal); all eigenvalues of T by bisection, one thread each;
// the dvec eigenvectors the caller asked for (ranks first .. first + dvec - 1) by a twisted factorisation of
// T - lambda I, one thread each; those vectors multiplied by Q, reflector by reflector, one wave each.  Everything
// after the reduction is parallel over eigenvalues or vectors: a QL iteration, whose scalar recurrence is one serial
// chain of ~M^2 rotations, took three times as long as the reduction (and a Jacobi method on the rows of G, the
// first solver here, 25 times).  All sums run in a fixed order (bit-reproducible).
//   1. for k = 0 .. M-3:  x = G[k][k+1..] (= the column below the diagonal, G is kept symmetric in full),
//      sigma = |x|, alpha = -sign(x_0) sigma, v = x - alpha e_0, beta = 1 / (sigma (sigma + |x_0|)), so that
//      H = I - beta v v^T maps x to alpha e_0;  p = beta G22 v,  w = p - (beta p.v / 2) v,
//      G22 -= v w^T + w v^T  (= H G22 H);  v stays in row k for step 4, d[k] = G[k][k], e[k] = alpha.
//      Thread (j, g) owns column j and the rows g (mod RG), so every pass reads and writes whole rows side by side.
//   2. - 4. are described where they stand.  Q itself is never formed: forming it costs as much as step 1.
// Non-finite input gives non-finite eigenvalues: status != 0, and the caller returns NaN eigenvalues and a zero block.
constexpr int kEigThreads = 1024;

__device__ __forceinline__ double block_sum(double x, double *red)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    __syncthreads();                 // red may still be read from the previous call
    if (lane == 0) red[wave] = x;
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kEigThreads / 64; ++w) s += red[w];
    return s;
}

// sum over rows i = first, first + RG, ... < M of mat[i][j] * vec[i], eight rows requested at a time; one fixed order
template <int RG>
__device__ __forceinline__ double column_dot(const double *__restrict__ mat, const double *vec, int first, int M, int j)
{
    double acc = 0.0;
    int i = first;
    for (; i + 7 * RG < M; i += 8 * RG) {
        double x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = mat[(size_t)(i + u * RG) * M + j];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc = fma(x[u], vec[i + u * RG], acc);
    }
    for (; i < M; i += RG) acc = fma(mat[(size_t)i * M + j], vec[i], acc);
    return acc;
}

// CP: columns the workgroup can hold (256 or 512); the 1024 threads are RG = 1024 / CP groups of CP threads,
// thread (g, j) owns column j and, in the passes over a matrix, the rows i = g (mod RG).
template <int CP>
__global__ __launch_bounds__(kEigThreads) void eigen_kernel(double *__restrict__ a_all, double *__restrict__ q_all,
                                                            double *__restrict__ lam_all, int *__restrict__ status_all,
                                                            double *__restrict__ vec_all, int M, int first, int dvec)
{
    constexpr int RG = kEigThreads / CP;
    __shared__ double d[CP], e[CP], v[CP], w[CP], beta[CP], part[RG][CP], red[kEigThreads / 64];
    __shared__ double x_first;
    const int tid = threadIdx.x, j = tid % CP, g = tid / CP;
    const bool col = j < M;
    double *a = a_all + (size_t)blockIdx.x * M * M;
    double *qm = q_all + (size_t)blockIdx.x * 2 * M * dvec;   // pivots of the twisted factorisations (step 3)

    // ---- 1. tridiagonalisation ----
    for (int k = 0; k + 2 < M; ++k) {
        const double xj = (g == 0 && col && j > k) ? a[(size_t)k * M + j] : 0.0;
        if (g == 0 && j == k + 1) x_first = xj;     // read by all after the barriers of the sum (row k is overwritten below)
        const double sig2 = block_sum(xj * xj, red);
        const double x0 = x_first;
        if (tid == 0) d[k] = a[(size_t)k * M + k];
        if (!(sig2 > 0.0)) {         // nothing to eliminate in this row
            if (tid == 0) { e[k] = 0.0; beta[k] = 0.0; }
            continue;
        }
        const double sigma = sqrt(sig2);
        const double alpha = x0 >= 0.0 ? -sigma : sigma;
        const double bt = 1.0 / (sigma * (sigma + fabs(x0)));
        if (g == 0) {
            const double vj = (col && j > k) ? (j == k + 1 ? xj - alpha : xj) : 0.0;
            v[j] = vj;
            if (col && j > k) a[(size_t)k * M + j] = vj;
        }
        if (tid == 0) { e[k] = alpha; beta[k] = bt; }
        __syncthreads();
        {   // p = beta G22 v: each row group sums its rows, group 0 adds the groups in order
            double pj = 0.0;
            if (col && j > k) pj = column_dot<RG>(a, v, k + 1 + g, M, j);
            part[g][j] = pj;
        }
        __syncthreads();
        double pj = 0.0, vj = 0.0;
        if (g == 0) {
#pragma unroll
            for (int r = 0; r < RG; ++r) pj += part[r][j];
            pj *= bt;
            vj = v[j];
        }
        const double kk = 0.5 * bt * block_sum(g == 0 ? pj * vj : 0.0, red);
        if (g == 0) w[j] = pj - kk * vj;
        __syncthreads();
        if (col && j > k) {
            const double wj = w[j], vv = v[j];
            int i = k + 1 + g;
            for (; i + 7 * RG < M; i += 8 * RG) {      // eight rows requested before the first is used
                double x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = a[(size_t)(i + u * RG) * M + j];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    a[(size_t)(i + u * RG) * M + j] = x[u] - v[i + u * RG] * wj - w[i + u * RG] * vv;
            }
            for (; i < M; i += RG) {
                const size_t at = (size_t)i * M + j;
                a[at] = a[at] - v[i] * wj - w[i] * vv;
            }
        }
        __syncthreads();
    }
    if (tid == 0) {
        if (M >= 2) {
            d[M - 2] = a[(size_t)(M - 2) * M + M - 2];
            e[M - 2] = a[(size_t)(M - 1) * M + M - 2];
        }
        d[M - 1] = a[(size_t)(M - 1) * M + M - 1];
        e[M - 1] = 0.0;
    }
    __syncthreads();
    // ---- 2. all eigenvalues of T by bisection, one thread per eigenvalue ----
    // Sturm count: the number of negative pivots q_i of T - x I (q_0 = d_0 - x, q_i = d_i - x - e_{i-1}^2 / q_{i-1})
    // is the number of eigenvalues below x; thread t halves the Gershgorin interval until it holds only the
    // eigenvalue of rank t (descending).  A pivot below pivmin in size is replaced by -pivmin (a change of T far
    // below its rounding).  The eigenvalues come out ordered and to the absolute accuracy of T's entries.
    double *e2 = w, *lam_s = v;                     // LDS: squares of the off-diagonal, the ordered eigenvalues
    if (tid < M) e2[tid] = e[tid] * e[tid];
    __syncthreads();
    double gl = INFINITY, gu = -INFINITY, emax2 = 0.0;
    for (int i = 0; i < M; ++i) {
        const double rad = fabs(e[i]) + (i > 0 ? fabs(e[i - 1]) : 0.0);
        gl = fmin(gl, d[i] - rad);
        gu = fmax(gu, d[i] + rad);
        emax2 = fmax(emax2, e2[i]);
    }
    const double tnorm = fmax(fabs(gl), fabs(gu));
    const double pivmin = fmax(4.9e-32 * emax2, 1e-290);
    if (tid < M) {
        const int idx = M - 1 - tid;                // rank from below
        double lo = gl - 1e-15 * tnorm - pivmin, hi = gu + 1e-15 * tnorm + pivmin;
        for (int it = 0; it < 60; ++it) {
            const double x = 0.5 * (lo + hi);
            double q = d[0] - x;
            int cnt = q < 0.0 ? 1 : 0;
#pragma unroll 4
            for (int i = 1; i < M; ++i) {
                if (fabs(q) < pivmin) q = -pivmin;
                double r = __builtin_amdgcn_rcp(q);
                r = r * fma(-q, r, 2.0);            // one Newton step: 1 / q to fp64
                q = fma(-e2[i - 1], r, d[i] - x);
                cnt += q < 0.0 ? 1 : 0;
            }
            if (cnt > idx) hi = x; else lo = x;
        }
        const double lam = 0.5 * (lo + hi);
        lam_s[tid] = lam;
        lam_all[(size_t)blockIdx.x * M + tid] = lam;
    }
    __syncthreads();
    if (tid == 0) {
        bool bad = false;
        for (int i = 0; i < M; ++i) bad |= !(fabs(lam_s[i]) <= 1e300);
        status_all[blockIdx.x] = bad ? 1 : 0;
    }

    // ---- 3. the requested eigenvectors of T, one thread per vector: twisted factorisation ----
    // For the eigenvalue lambda: the pivots q+ of T - lambda I from the top (as above) and q- from the bottom;
    // gamma_k = q+_k + q-_k - (d_k - lambda) is what is left of row k when everything above is eliminated from the
    // top and everything below from the bottom, and z with z_k = 1, z_{i-1} = -e_{i-1} z_i / q+_{i-1} above k,
    // z_{i+1} = -e_i z_i / q-_{i+1} below k solves every row of (T - lambda I) z = 0 but row k, whose residual
    // is gamma_k: with k at the smallest |gamma| the residual is of the size of lambda's error.
    double *qp_all = qm, *qn_all = qm + (size_t)M * dvec;     // [i][c]: neighbouring threads, neighbouring addresses
    double *z_all = vec_all + (size_t)blockIdx.x * dvec * M;   // [c][i]
    auto guard = [&](double q) { return fabs(q) < pivmin ? -pivmin : q; };
    // the vector of eigenvalue lam from the stored pivots of thread c, twisted at k; returns its norm
    auto build_vector = [&](int c, int k) {
        double *z = z_all + (size_t)c * M;
        z[k] = 1.0;
        double n2 = 1.0, zi = 1.0;
        for (int i = k - 1; i >= 0; --i) {
            zi = -e[i] * zi / guard(qp_all[(size_t)i * dvec + c]);
            if (fabs(zi) > 1e150) {              // rescale what is there (rare: a run of tiny pivots)
                for (int j = i + 1; j <= k; ++j) z[j] *= 1e-150;
                zi *= 1e-150;
                n2 *= 1e-300;
            }
            z[i] = zi;
            n2 = fma(zi, zi, n2);
        }
        zi = z[k];
        for (int i = k + 1; i < M; ++i) {
            zi = -e[i - 1] * zi / guard(qn_all[(size_t)i * dvec + c]);
            if (fabs(zi) > 1e150) {
                for (int j = 0; j < i; ++j) z[j] *= 1e-150;
                zi *= 1e-150;
                n2 *= 1e-300;
            }
            z[i] = zi;
            n2 = fma(zi, zi, n2);
        }
        const double inv = 1.0 / sqrt(n2);
        for (int i = 0; i < M; ++i) z[i] *= inv;
    };
    auto gamma_at = [&](int c, int i, double lam) {
        return qp_all[(size_t)i * dvec + c] + qn_all[(size_t)i * dvec + c] - (d[i] - lam);
    };
    if (tid < dvec && first + tid < M) {
        const int c = tid;
        const double lam = lam_s[first + c];
        double q = d[0] - lam;
        for (int i = 1; i < M; ++i) {
            q = guard(q);
            qp_all[(size_t)(i - 1) * dvec + c] = q;
            q = (d[i] - lam) - e2[i - 1] / q;
        }
        qp_all[(size_t)(M - 1) * dvec + c] = q;
        q = d[M - 1] - lam;
        for (int i = M - 2; i >= 0; --i) {
            q = guard(q);
            qn_all[(size_t)(i + 1) * dvec + c] = q;
            q = (d[i] - lam) - e2[i] / q;
        }
        qn_all[(size_t)0 * dvec + c] = q;
        int k = 0;
        double best = INFINITY;
        for (int i = 0; i < M; ++i) {
            const double gmm = fabs(gamma_at(c, i, lam));
            if (gmm < best) { best = gmm; k = i; }
        }
        build_vector(c, k);
    }
    __syncthreads();
    // Eigenvalues that agree to 1e-12 |T| (T splits, or nearly: only then can eigenvalues of a tridiagonal matrix
    // coincide): the recipe above may give them the same vector.  One thread goes over such runs in order: a later
    // vector of a run is twisted at the smallest |gamma| among the rows where the earlier ones are small, and made
    // orthogonal to them.
    if (tid == 0) {
        for (int c = 1; c < dvec && first + c < M; ++c) {
            int c0 = c;
            while (c0 > 0 && fabs(lam_s[first + c0 - 1] - lam_s[first + c]) <= 1e-12 * tnorm) --c0;
            if (c0 == c) continue;
            const double lam = lam_s[first + c];
            int k = -1;
            double best = INFINITY;
            for (int i = 0; i < M; ++i) {
                double seen = 0.0;
                for (int p = c0; p < c; ++p) seen = fmax(seen, fabs(z_all[(size_t)p * M + i]));
                const double gmm = fabs(gamma_at(c, i, lam));
                if (seen < 1e-3 && gmm < best) { best = gmm; k = i; }
            }
            if (k >= 0) build_vector(c, k);
            double *z = z_all + (size_t)c * M;
            for (int p = c0; p < c; ++p) {
                const double *zp = z_all + (size_t)p * M;
                double dot = 0.0;
                for (int i = 0; i < M; ++i) dot = fma(zp[i], z[i], dot);
                for (int i = 0; i < M; ++i) z[i] = fma(-dot, zp[i], z[i]);
            }
            double n2 = 0.0;
            for (int i = 0; i < M; ++i) n2 = fma(z[i], z[i], n2);
            if (n2 > 1e-16) {
                const double inv = 1.0 / sqrt(n2);
                for (int i = 0; i < M; ++i) z[i] *= inv;
            }
        }
    }
    __syncthreads();

    // ---- 4. the eigenvectors of G: x = H_0 ... H_{M-3} z, one wave per vector ----
    // The vector in registers (lane l holds the elements l, l + 64, ...), the reflector's row requested one step ahead.
    constexpr int NE = CP / 64;
    const int lane = tid & 63, wave = tid >> 6;
    for (int c = wave; c < dvec; c += kEigThreads / 64) {
        double *out = vec_all + ((size_t)blockIdx.x * dvec + c) * M;
        const int rk = first + c;
        if (rk >= M) {
            for (int i = 0; i < NE; ++i)
                if (lane + 64 * i < M) out[lane + 64 * i] = 0.0;
            continue;
        }
        const double *z = out;                        // step 3 left the eigenvector of T there
        double y[NE], v[NE], vn[NE];
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            const int m = lane + 64 * i;
            y[i] = m < M ? z[m] : 0.0;
            vn[i] = 0.0;
        }
        auto load_reflector = [&](int k, double (&t)[NE]) {
#pragma unroll
            for (int i = 0; i < NE; ++i) {
                const int m = lane + 64 * i;
                t[i] = (m > k && m < M) ? a[(size_t)k * M + m] : 0.0;
            }
        };
        if (M >= 3) load_reflector(M - 3, vn);
        for (int k = M - 3; k >= 0; --k) {
#pragma unroll
            for (int i = 0; i < NE; ++i) v[i] = vn[i];
            if (k > 0) load_reflector(k - 1, vn);
            const double bt = beta[k];
            if (bt == 0.0) continue;
            double dot = 0.0;
#pragma unroll
            for (int i = 0; i < NE; ++i) dot = fma(v[i], y[i], dot);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
            const double t = bt * dot;
#pragma unroll
            for (int i = 0; i < NE; ++i) y[i] = fma(-t, v[i], y[i]);
        }
#pragma unroll
        for (int i = 0; i < NE; ++i)
            if (lane + 64 * i < M) out[lane + 64 * i] = y[i];
    }
}

// ---- eigenvalues in descending order, and the decode-ready block of d eigenvectors -------------------
// Row j of the matrix buffer is the unit eigenvector q_j, lam_in[j] its eigenvalue (clamped at zero: G is
// positive semi-definite).  rank of eigenvalue j = how many are larger (ties broken by index): a stable order
// without a sort.
// zvec[b*h][m][c] = exp(-lse_enc[m] / 2) * q_j[m] / sqrt(lambda_j),  j = the (first + c)-th largest;
// zero where that index is beyond M or the eigenvalue is below 1e-12 of the largest.
// A solver that did not converge (status != 0) gives NaN eigenvalues and a zero block.
__global__ __launch_bounds__(256) void spectral_post_kernel(const double *__restrict__ b_all,
                                                            const double *__restrict__ lam_in,
                                                            const int *__restrict__ status,
                                                            const float *__restrict__ lse_enc,
                                                            float *__restrict__ evals, float *__restrict__ zvec, int M,
                                                            int d, int first)
{
    extern __shared__ double lam[];   // lam[M], then int row_of[M]
    int *row_of = reinterpret_cast<int *>(lam + M);
    const int bh = blockIdx.x, tid = threadIdx.x;
    const double *bm = b_all + (size_t)bh * d * M;       // row c: the unit eigenvector of rank first + c
    const bool bad = status[bh] != 0;
    for (int j = tid; j < M; j += 256) lam[j] = fmax(lam_in[(size_t)bh * M + j], 0.0);
    __syncthreads();
    for (int j = tid; j < M; j += 256) {
        int rank = 0;
        for (int i = 0; i < M; ++i) rank += (lam[i] > lam[j] || (lam[i] == lam[j] && i < j)) ? 1 : 0;
        row_of[rank] = j;
        evals[(size_t)bh * M + rank] = bad ? __builtin_nanf("") : (float)lam[j];
    }
    __syncthreads();
    const double top = lam[row_of[0]];
    for (int w = tid; w < M * d; w += 256) {
        const int m = w / d, c = w % d, rk = first + c;
        float out = 0.f;
        if (rk < M && !bad) {
            const int j = row_of[rk];
            if (lam[j] > 1e-12 * top && lam[j] > 1e-300)
                out = (float)(exp(-0.5 * (double)lse_enc[(size_t)bh * M + m]) * bm[(size_t)c * M + m] / sqrt(lam[j]));
        }
        zvec[((size_t)bh * M + m) * d + c] = out;
    }
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

Split spectral_split(const flare_shape &s)
{
    return plan_split(s.N, s.B * s.H, 256, mfma_gram_supported(s) ? 512 : 1024);
}

// doubles per (b,h) for the pivots of the twisted factorisations: two arrays of M per requested vector
static size_t pivot_elems(const flare_shape &s) { return 2 * (size_t)s.M * s.d; }

size_t spectral_bytes(const flare_shape &s)
{
    const size_t BH = (size_t)s.B * s.H, mm = (size_t)s.M * s.M;
    const Split sp = spectral_split(s);
    // partial G's; one fp64 matrix per (b,h) (G, then its reflectors); the pivots of the requested vectors;
    // eigenvalues; solver status; the d requested eigenvectors
    return align256(BH * sp.chunks * mm * 4) + align256(BH * mm * 8) + align256(BH * pivot_elems(s) * 8) +
           align256(BH * s.M * 8) + align256(BH * 4) + align256(BH * s.d * s.M * 8);
}

int spectral_run(const flare_shape &s, const void *q, const void *k, const float *lse_enc, const float *lse_dec,
                 float scale, int first, float *evals, float *zvec, float *gram, void *ws, hipStream_t stream)
{
    const size_t BH = (size_t)s.B * s.H, mm = (size_t)s.M * s.M;
    const Split sp = spectral_split(s);
    char *base = static_cast<char *>(ws);
    float *g_part = reinterpret_cast<float *>(base);
    double *a = reinterpret_cast<double *>(base + align256(BH * sp.chunks * mm * 4));
    double *qbuf = reinterpret_cast<double *>(reinterpret_cast<char *>(a) + align256(BH * mm * 8));
    double *lam = reinterpret_cast<double *>(reinterpret_cast<char *>(qbuf) + align256(BH * pivot_elems(s) * 8));
    int *status = reinterpret_cast<int *>(reinterpret_cast<char *>(lam) + align256(BH * s.M * 8));
    double *vec = reinterpret_cast<double *>(reinterpret_cast<char *>(status) + align256(BH * 4));
    if (mfma_gram_supported(s)) {
        const int rc = mfma_gram_partial(s, sp, q, k, lse_enc, lse_dec, g_part, scale, stream);
        if (rc != FLARE_OK) return rc;
    } else {
        const dim3 grid(sp.chunks, (unsigned)BH, (s.M + 15) / 16);
        const TokStride ts = tok_stride(s);
        LaunchTimer t(KID_SPECTRAL_GRAM, stream);
        if (s.dtype == FLARE_F32)
            gram_valu_kernel<float><<<grid, 256, s.M * 4, stream>>>((const float *)q, (const float *)k, lse_enc, lse_dec,
                                                                   g_part, ts, s.H, s.N, s.M, s.d, sp.chunk_len,
                                                                   sp.chunks, scale);
        else if (s.dtype == FLARE_F16)
            gram_valu_kernel<f16_t><<<grid, 256, s.M * 4, stream>>>((const f16_t *)q, (const f16_t *)k, lse_enc,
                                                                   lse_dec, g_part, ts, s.H, s.N, s.M, s.d,
                                                                   sp.chunk_len, sp.chunks, scale);
        else
            gram_valu_kernel<bf16_t><<<grid, 256, s.M * 4, stream>>>((const bf16_t *)q, (const bf16_t *)k, lse_enc,
                                                                    lse_dec, g_part, ts, s.H, s.N, s.M, s.d,
                                                                    sp.chunk_len, sp.chunks, scale);
        if (check_launch() != FLARE_OK) return FLARE_ELAUNCH;
    }
    {
        LaunchTimer t(KID_SPECTRAL_REDUCE, stream);
        const size_t total = BH * mm;
        gram_reduce_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(g_part, gram, a, sp.chunks, mm, total);
    }
    if (check_launch() != FLARE_OK) return FLARE_ELAUNCH;
    {
        LaunchTimer t(KID_SPECTRAL_EIGEN, stream);
        if (s.M <= 256) eigen_kernel<256><<<(unsigned)BH, kEigThreads, 0, stream>>>(a, qbuf, lam, status, vec, s.M, first, s.d);
        else eigen_kernel<512><<<(unsigned)BH, kEigThreads, 0, stream>>>(a, qbuf, lam, status, vec, s.M, first, s.d);
    }
    if (check_launch() != FLARE_OK) return FLARE_ELAUNCH;
    {
        LaunchTimer t(KID_SPECTRAL_POST, stream);
        spectral_post_kernel<<<(unsigned)BH, 256, s.M * 12, stream>>>(vec, lam, status, lse_enc, evals, zvec, s.M, s.d,
                                                                      first);
    }
    return check_launch();
}

}  // namespace flare
