// Spectral analysis of the mixing matrix W = W_dec W_enc of one (b,h) (Appendix C.1, Algorithm 1):
// the nonzero eigenvalues of the N x N matrix W are those of the M x M matrix
//     G = J J^T,   J = L_M^(1/2) A L_N^(1/2),   A = exp(scale * Q K^T),
// and its eigenvectors are L_N^(1/2) J^T U Sigma^(-1) = W_dec (L_M^(1/2) U Sigma^(-1)): the decode
// applied to an M x M "latent sequence".  With lse_enc = log row sums of A and lse_dec = log column
// sums (what the forward leaves behind),  J[m][n] = exp(S[m][n] - (lse_enc[m] + lse_dec[n]) / 2).
//
// Steps here:  G as a streaming reduction over the tokens (matrix-core kernel in flare_mfma_fwd.hip,
// or the fp32 kernel below), a fixed-order sum of the per-chunk partials, a one-sided cyclic Jacobi
// eigensolver in fp64 (one workgroup per (b,h); the rotations of a round act on disjoint pairs of
// rows), and a last kernel that orders the eigenvalues and forms the decode-ready block
// L_M^(1/2) U Sigma^(-1) of d consecutive eigenvectors.
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

// ---- one-sided cyclic Jacobi eigensolver, fp64, one workgroup of 1024 threads per matrix ------------------
// G is symmetric positive semi-definite, G = Q^T Lambda Q.  Rotating ROWS of B = G against each other
// until they are mutually orthogonal applies an orthogonal Q from the left with (QG)(QG)^T = Q G^2 Q^T
// diagonal, i.e. B ends as Lambda Q: row i is lambda_i times the i-th eigenvector, its length is
// lambda_i.  Only whole rows are read and written (coalesced), nothing else is accumulated, and the
// pairs of a round of the round-robin tournament (M' - 1 rounds per sweep, M' = M rounded up to
// even) are disjoint: a wave per few pairs, one barrier per round.  At most 40 sweeps.
constexpr int kJacobiThreads = 1024;
// RR = row elements per lane (M <= 64 * RR); a wave works on PB = 16 / RR pairs at a time so that
// the loads of all of them are in flight together.
template <int RR>
__global__ __launch_bounds__(kJacobiThreads) void jacobi_kernel(double *__restrict__ b_all, int M)
{
    constexpr int PB = 16 / RR;
    __shared__ unsigned long long worst;       // bits of the largest |cos| of the sweep (non-negative doubles order as integers)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double *bm = b_all + (size_t)blockIdx.x * M * M;
    const int Mp = M + (M & 1), pairs = Mp / 2;
    // Orthogonality is judged in absolute terms, inner product against the matrix's squared Frobenius
    // norm F2: below 1e-22 F2 a pair is left alone, and the solver stops after a sweep in which no inner
    // product exceeded 1e-18 F2.  (The eigenvalues are wanted to absolute accuracy; rows of tiny
    // eigenvalues carry rounding noise of the large ones, which no rotation can make orthogonal in
    // relative terms.)
    __shared__ double fro[kJacobiThreads / 64];
    {
        double f = 0.0;
        for (int i = tid; i < M * M; i += kJacobiThreads) f = fma(bm[i], bm[i], f);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) f += __shfl_xor(f, o);
        if (lane == 0) fro[wave] = f;
        __syncthreads();
    }
    double tiny = 0.0;
    for (int w = 0; w < kJacobiThreads / 64; ++w) tiny += fro[w];
    const double f2 = tiny;
    tiny *= 1e-22;
    for (int sweep = 0; sweep < 40; ++sweep) {
        if (tid == 0) worst = 0ull;
        __syncthreads();
        for (int round = 0; round < Mp - 1; ++round) {
            for (int i0 = wave * PB; i0 < pairs; i0 += (kJacobiThreads / 64) * PB) {
                double x[PB][RR], y[PB][RR];
                int pp[PB], qq[PB];
#pragma unroll
                for (int b = 0; b < PB; ++b) {
                    const int i = i0 + b;
                    int p = (i == 0) ? Mp - 1 : (round + i) % (Mp - 1);
                    int q = (i == 0) ? round : (round - i + Mp - 1) % (Mp - 1);
                    if (p > q) { const int t = p; p = q; q = t; }
                    const bool live = i < pairs && q < M;      // q == M: the padding index of an odd M
                    pp[b] = live ? p : -1;
                    qq[b] = q;
#pragma unroll
                    for (int t = 0; t < RR; ++t) {
                        const int j = lane + 64 * t;
                        x[b][t] = (live && j < M) ? bm[(size_t)p * M + j] : 0.0;
                        y[b][t] = (live && j < M) ? bm[(size_t)q * M + j] : 0.0;
                    }
                }
#pragma unroll
                for (int b = 0; b < PB; ++b) {
                    if (pp[b] < 0) continue;
                    double al = 0.0, be = 0.0, ga = 0.0;
#pragma unroll
                    for (int t = 0; t < RR; ++t) {
                        al = fma(x[b][t], x[b][t], al);
                        be = fma(y[b][t], y[b][t], be);
                        ga = fma(x[b][t], y[b][t], ga);
                    }
#pragma unroll
                    for (int o = 32; o > 0; o >>= 1) {
                        al += __shfl_xor(al, o);
                        be += __shfl_xor(be, o);
                        ga += __shfl_xor(ga, o);
                    }
                    const double den = sqrt(al * be);
                    if (!(fabs(ga) > tiny) || !(fabs(ga) > 1e-15 * den)) continue;   // orthogonal already
                    if (lane == 0) atomicMax(&worst, (unsigned long long)__double_as_longlong(fabs(ga)));
                    const double zeta = (be - al) / (2.0 * ga);
                    const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                    const double c = 1.0 / sqrt(1.0 + t * t), sn = c * t;
#pragma unroll
                    for (int r = 0; r < RR; ++r) {
                        const int j = lane + 64 * r;
                        if (j < M) {
                            bm[(size_t)pp[b] * M + j] = c * x[b][r] - sn * y[b][r];
                            bm[(size_t)qq[b] * M + j] = sn * x[b][r] + c * y[b][r];
                        }
                    }
                }
            }
            __syncthreads();
        }
        const double w = __longlong_as_double((long long)worst);
        __syncthreads();
        if (!(w > 1e-18 * f2)) break;
    }
}

// ---- eigenvalues in descending order, and the decode-ready block of d eigenvectors -------------------
// Row j of B is lambda_j q_j.  rank of eigenvalue j = how many are larger (ties broken by index): a
// stable order without a sort.
// zvec[b*h][m][c] = exp(-lse_enc[m] / 2) * q_j[m] / sqrt(lambda_j),  j = the (first + c)-th largest;
// zero where that index is beyond M or the eigenvalue is below 1e-12 of the largest.
__global__ __launch_bounds__(256) void spectral_post_kernel(const double *__restrict__ b_all,
                                                            const float *__restrict__ lse_enc,
                                                            float *__restrict__ evals, float *__restrict__ zvec, int M,
                                                            int d, int first)
{
    extern __shared__ double lam[];   // lam[M], then int row_of[M]
    int *row_of = reinterpret_cast<int *>(lam + M);
    const int bh = blockIdx.x, tid = threadIdx.x;
    const double *bm = b_all + (size_t)bh * M * M;
    for (int j = tid; j < M; j += 256) {
        double s = 0.0;
        for (int i = 0; i < M; ++i) s = fma(bm[(size_t)j * M + i], bm[(size_t)j * M + i], s);
        lam[j] = sqrt(s);
    }
    __syncthreads();
    for (int j = tid; j < M; j += 256) {
        int rank = 0;
        for (int i = 0; i < M; ++i) rank += (lam[i] > lam[j] || (lam[i] == lam[j] && i < j)) ? 1 : 0;
        row_of[rank] = j;
        evals[(size_t)bh * M + rank] = (float)lam[j];
    }
    __syncthreads();
    const double top = lam[row_of[0]];
    for (int w = tid; w < M * d; w += 256) {
        const int m = w / d, c = w % d, rk = first + c;
        float out = 0.f;
        if (rk < M) {
            const int j = row_of[rk];
            if (lam[j] > 1e-12 * top && lam[j] > 1e-300)
                out = (float)(exp(-0.5 * (double)lse_enc[(size_t)bh * M + m]) * bm[(size_t)j * M + m] /
                              (lam[j] * sqrt(lam[j])));
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
    return align256(BH * sp.chunks * mm * 4) + align256(BH * mm * 8);
}

int spectral_run(const flare_shape &s, const void *q, const void *k, const float *lse_enc, const float *lse_dec,
                 float scale, int first, float *evals, float *zvec, float *gram, void *ws, hipStream_t stream)
{
    const size_t BH = (size_t)s.B * s.H, mm = (size_t)s.M * s.M;
    const Split sp = spectral_split(s);
    char *base = static_cast<char *>(ws);
    float *g_part = reinterpret_cast<float *>(base);
    double *a = reinterpret_cast<double *>(base + align256(BH * sp.chunks * mm * 4));
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
        if (s.M <= 64) jacobi_kernel<1><<<(unsigned)BH, kJacobiThreads, 0, stream>>>(a, s.M);
        else if (s.M <= 128) jacobi_kernel<2><<<(unsigned)BH, kJacobiThreads, 0, stream>>>(a, s.M);
        else if (s.M <= 256) jacobi_kernel<4><<<(unsigned)BH, kJacobiThreads, 0, stream>>>(a, s.M);
        else jacobi_kernel<8><<<(unsigned)BH, kJacobiThreads, 0, stream>>>(a, s.M);
    }
    if (check_launch() != FLARE_OK) return FLARE_ELAUNCH;
    {
        LaunchTimer t(KID_SPECTRAL_POST, stream);
        spectral_post_kernel<<<(unsigned)BH, 256, s.M * 12, stream>>>(a, lse_enc, evals, zvec, s.M, s.d, first);
    }
    return check_launch();
}

}  // namespace flare
