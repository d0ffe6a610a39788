// Spectral analysis of the mixing matrix W = W_dec W_enc of one (b,h) (Appendix C.1, Algorithm 1):
// the nonzero eigenvalues of the N x N matrix W are those of the M x M matrix
//     G = J J^T,   J = L_M^(1/2) A L_N^(1/2),   A = exp(scale * Q K^T),
// and its eigenvectors are L_N^(1/2) J^T U Sigma^(-1) = W_dec (L_M^(1/2) U Sigma^(-1)): the decode
// applied to an M x M "latent sequence".  With lse_enc = log row sums of A and lse_dec = log column
// sums (what the forward leaves behind),  J[m][n] = exp(S[m][n] - (lse_enc[m] + lse_dec[n]) / 2).
//
// Steps here:  G as a streaming reduction over the tokens (matrix-core kernel in flare_mfma_fwd.hip,
// or the fp32 kernel below), a fixed-order sum of the per-chunk partials, a symmetric eigensolver in fp64
// (one workgroup per (b,h): Householder tridiagonalisation, the implicit QL iteration with its rotations
// accumulated from the identity, and the reflectors applied to the d eigenvectors that were asked for), and a last
// kernel that orders the eigenvalues and forms the decode-ready block L_M^(1/2) U Sigma^(-1) of those eigenvectors.
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
// G = Q T Q^T by Householder reflections (T tridiagonal), then the implicit-shift QL iteration on T with its
// plane rotations applied to the rows of a second matrix that starts as the identity; at the end row j of that
// matrix is the j-th eigenvector of T and lam[j] its eigenvalue (unordered), and the dvec eigenvectors of G that
// the caller asked for (ranks first .. first + dvec - 1) are those rows multiplied by Q, reflector by reflector.
// Thread j owns column j throughout, so every pass over a matrix reads and writes whole rows side by side; all
// sums run in a fixed order (bit-reproducible).
//   1. for k = 0 .. M-3:  x = G[k][k+1..] (= the column below the diagonal, G is kept symmetric in full),
//      sigma = |x|, alpha = -sign(x_0) sigma, v = x - alpha e_0, beta = 1 / (sigma (sigma + |x_0|)), so that
//      H = I - beta v v^T maps x to alpha e_0;  p = beta G22 v,  w = p - (beta p.v / 2) v,
//      G22 -= v w^T + w v^T  (= H G22 H);  v stays in row k for step 2, d[k] = G[k][k], e[k] = alpha.
//   2. the second buffer := I.  (Q itself is never formed: forming it costs as much as step 1, and only dvec of
//      its M columns' worth of work is wanted.)
//   3. QL with Wilkinson shifts on (d, e): thread 0 runs the scalar recurrence of one iteration and leaves the
//      rotations (c_i, s_i) in LDS (1 / r from the hardware reciprocal square root and one third-order step: no
//      division, no square root in the chain; a loop body without branches: a lone wave issues about one
//      instruction per 10 clocks, so the step costs its ~40 instructions, not its dependent chain of ~120
//      clocks); meanwhile one thread per column applies the rotations of the
//      previous iteration to its column of the second buffer, rows m .. l, with the rows and rotations it will need requested
//      eight steps ahead.  The two sides swap LDS buffers at one barrier per iteration.  An off-diagonal element
//      counts as zero at 2^-52 (|d_m| + |d_m+1|) + 1e-10 |T|: the result is the exact eigensystem of a matrix
//      within 1e-10 |G| of G, while G itself (sums of 10^6 products in fp32, bf16 weights on the matrix-core
//      path) is no more accurate than 4e-7 |G|; the eigenvalues are delivered in fp32.  (A floor of 1e-22 |T|
//      costs a fifth more sweeps and changes no printed digit of the test results.)
// 60 iterations without convergence for one eigenvalue: the solver stops and reports it (status != 0; the caller
// then returns NaN eigenvalues).  The previous solver here, a one-sided Jacobi method on the rows of G, needed
// ~2500 rounds of row-pair rotations through global memory (102 ms for eight 256 x 256 matrices).
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

// 1 / sqrt(h) to full fp64 accuracy from the hardware estimate y (relative error e0 <= 2^-20, far more than it
// needs) and one third-order step: with e = 1 - h y^2,  1/sqrt(h) = y (1 - e)^(-1/2) = y (1 + e/2 + 3 e^2/8 + O(e^3)).
// (h > 0, normal.)
__device__ __forceinline__ double rsqrt_full(double h)
{
    const double y = __builtin_amdgcn_rsq(h);
    const double e = fma(-h * y, y, 1.0);
    return fma(y * e, fma(0.375, e, 0.5), y);
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
    __shared__ double cc[2][CP], ss[2][CP];
    __shared__ int ctl[2][4];        // per buffer: top row, bottom row, kind (0 rotate, 2 finished), failed
    __shared__ double x_first;
    const int tid = threadIdx.x, j = tid % CP, g = tid / CP;
    const bool col = j < M;
    double *a = a_all + (size_t)blockIdx.x * M * M;
    double *qm = q_all + (size_t)blockIdx.x * M * M;

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
    // ---- 2. the second buffer := identity: QL rotates its rows into the eigenvectors of T ----
    // (The product of the reflectors is not formed: only the requested eigenvectors are transformed back, at the end.)
    if (col)
        for (int i = g; i < M; i += RG) qm[(size_t)i * M + j] = (i == j) ? 1.0 : 0.0;
    __syncthreads();

    // ---- 3. implicit QL; rotations act on rows i, i+1 of the second buffer ----
    // Thread 0 (wave 0) produces the rotations of iteration n+1 into one LDS buffer while threads 64 .. 64 + M - 1
    // apply those of iteration n from the other: both between the same two barriers, no waiting on flags.
    double anorm = 0.0;
    for (int i = 0; i < M; ++i) anorm = fmax(anorm, fabs(d[i]) + fabs(e[i]));
    const double floor_abs = 1e-10 * anorm;
    int l = 0, iter = 0;             // producer state (the first wave, uniform over its lanes)
    // One step of the producer: the next QL iteration (or the end), written into buffer `bf`.  Called by the whole
    // first wave: its lanes look for the next negligible off-diagonal element 64 at a time; lane 0 alone runs
    // the recurrence.
    auto produce = [&](int bf) {
        const int lane = tid;        // tid < 64 here
        for (;;) {
            if (l >= M) {
                if (lane == 0) { ctl[bf][2] = 2; ctl[bf][3] = 0; }
                return;
            }
            int m = l;
            for (;;) {
                const int idx = m + lane;
                bool small = idx >= M - 1;
                if (!small) small = fabs(e[idx]) <= 2.220446049250313e-16 * (fabs(d[idx]) + fabs(d[idx + 1])) + floor_abs;
                const unsigned long long mask = __ballot(small);
                if (mask != 0ull) { m += __ffsll((long long)mask) - 1; break; }
                m += 64;
            }
            if (m == l) { ++l; iter = 0; continue; }             // eigenvalue l has converged
            if (iter == 60) {
                if (lane == 0) { ctl[bf][2] = 2; ctl[bf][3] = 1; }
                return;
            }
            ++iter;
            if (lane == 0) {
                double gg = (d[l + 1] - d[l]) / (2.0 * e[l]);
                double r = sqrt(gg * gg + 1.0);
                gg = d[m] - d[l] + e[l] / (gg + (gg >= 0.0 ? r : -r));
                double s = 1.0, c = 1.0, p = 0.0;
                int i = m - 1;
                double ei = e[i], di = d[i], di1 = d[i + 1];
                double g1 = 0.0;
                bool ok = true;
                // The loop body has no branch of its own (a taken branch costs a single wave more than the whole
                // dependent chain of the step): a rotation that is undefined (h underflows) is computed like any
                // other, ends the loop, and what it stored is put right afterwards.
                do {
                    // the next step's elements are requested now and only looked at when this step is done
                    const int ip = i > 0 ? i - 1 : 0;
                    const double en = e[ip], dn = d[ip];
                    const double f = s * ei, b = c * ei;
                    const double h = fma(f, f, gg * gg);
                    // s = f / r0, c = g / r0 with r0 = sqrt(h); everything that does not need 1 / r0 is formed
                    // while it is computed, so that two operations separate it from the next step's g
                    g1 = di1 - p;
                    const double wr = fma(di - g1, f, 2.0 * gg * b);     // = r0 ((d_i - g1) s + 2 c b)
                    const double ri = rsqrt_full(h);
                    e[i + 1] = h * ri;
                    s = f * ri;
                    c = gg * ri;
                    r = wr * ri;
                    p = s * r;
                    d[i + 1] = g1 + p;
                    gg = fma(c, r, -b);
                    cc[bf][i] = c;
                    ss[bf][i] = s;
                    di1 = di;
                    di = dn;
                    ei = en;
                    ok = h > 1e-290;
                    --i;
                } while (ok && i >= l);
                const bool under = !ok;
                if (under) {                         // step i + 1 was undefined: deflate there and start over
                    ++i;
                    e[i + 1] = 0.0;
                    d[i + 1] = g1;
                    e[m] = 0.0;
                } else {
                    d[l] -= p;
                    e[l] = gg;
                    e[m] = 0.0;
                }
                ctl[bf][0] = m;                      // rotations exist for rows m-1 down to the bottom row
                ctl[bf][1] = under ? i + 1 : l;
                ctl[bf][2] = 0;
                ctl[bf][3] = 0;
            }
            return;
        }
    };
    if (tid < 64) produce(0);
    __syncthreads();
    bool failed = false;
    for (int n = 0;; ++n) {
        const int bf = n & 1;
        const int top = ctl[bf][0], bot = ctl[bf][1], kind = ctl[bf][2];
        if (kind == 2) { failed = ctl[bf][3] != 0; break; }
        if (tid < 64) {
            produce(bf ^ 1);
        } else if (tid < 64 + M && top > bot) {
            const int jc = tid - 64;
            // rows top-1 .. bot, each rotated against the row above it; row top's value is carried down.  Eight
            // rows and their rotations are in flight at any time; the loop body has no branches (a request past
            // the bottom row is clamped to it and its result ignored), so that nothing waits for a request it
            // does not need yet.
            double hi = qm[(size_t)top * M + jc];
            double buf[8], cb[8], sb[8];
            int i = top - 1;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = max(i - u, bot);
                buf[u] = qm[(size_t)r * M + jc];
                cb[u] = cc[bf][r];
                sb[u] = ss[bf][r];
            }
            while (i - 7 >= bot) {
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int r = i - u, rn = max(r - 8, bot);
                    const double lo = buf[u], c = cb[u], s = sb[u];
                    buf[u] = qm[(size_t)rn * M + jc];
                    cb[u] = cc[bf][rn];
                    sb[u] = ss[bf][rn];
                    qm[(size_t)(r + 1) * M + jc] = fma(s, lo, c * hi);
                    hi = fma(c, lo, -s * hi);
                }
                i -= 8;
            }
#pragma unroll
            for (int u = 0; u < 7; ++u) {      // the last rows, fewer than eight
                const int r = i - u;
                if (r >= bot) {
                    qm[(size_t)(r + 1) * M + jc] = fma(sb[u], buf[u], cb[u] * hi);
                    hi = fma(cb[u], buf[u], -sb[u] * hi);
                }
            }
            qm[(size_t)bot * M + jc] = hi;
        }
        __syncthreads();
    }
    if (tid < M) lam_all[(size_t)blockIdx.x * M + tid] = d[tid];
    if (tid == 0) status_all[blockIdx.x] = failed ? 1 : 0;

    // ---- 4. the requested eigenvectors of G: x = H_0 ... H_{M-3} z for the rows z of ranks first .. first + dvec - 1 ----
    // rank of eigenvalue j = how many are larger (ties broken by index; negative rounding noise counts as zero): the
    // order the caller's post-processing uses.  One wave per vector, the vector in registers (lane l holds the
    // elements l, l + 64, ...), the reflector's row requested one step ahead.
    int *row_of = reinterpret_cast<int *>(&part[0][0]);
    if (tid < M) {
        const double lj = fmax(d[tid], 0.0);
        int rank = 0;
        for (int i = 0; i < M; ++i) {
            const double li = fmax(d[i], 0.0);
            rank += (li > lj || (li == lj && i < tid)) ? 1 : 0;
        }
        row_of[rank] = tid;
    }
    __syncthreads();
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
        const double *z = qm + (size_t)row_of[rk] * M;
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

size_t spectral_bytes(const flare_shape &s)
{
    const size_t BH = (size_t)s.B * s.H, mm = (size_t)s.M * s.M;
    const Split sp = spectral_split(s);
    // partial G's; two fp64 matrices per (b,h) (G, then its reflectors; the rotated identity); eigenvalues; solver
    // status; the d requested eigenvectors
    return align256(BH * sp.chunks * mm * 4) + 2 * align256(BH * mm * 8) + align256(BH * s.M * 8) + align256(BH * 4) +
           align256(BH * s.d * s.M * 8);
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
    double *lam = reinterpret_cast<double *>(reinterpret_cast<char *>(qbuf) + align256(BH * mm * 8));
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
