// Internal declarations shared by the translation units of libflare.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "flare.h"
#include "flare_profile.h"

namespace flare {

// ---- kernel ids for the per-kernel timing hooks ------------------------------------------
enum KernelId {
    KID_ENCODE_PARTIAL = 0,
    KID_ENCODE_MERGE,
    KID_DECODE,
    KID_BWD_TOKEN_STATS,
    KID_BWD_PREP,
    KID_BWD_DZ_PARTIAL,
    KID_BWD_DZ_MERGE,
    KID_BWD_DQ_PARTIAL,
    KID_BWD_DQ_REDUCE,
    KID_BWD_DKDV,
    KID_BWD_DKDV_2EXP,
    KID_DECODE_MERGE,
    KID_SPECTRAL_GRAM,
    KID_SPECTRAL_REDUCE,
    KID_SPECTRAL_EIGEN,
    KID_SPECTRAL_POST,
    KID_DECODE_PROJECT,
    KID_COUNT
};

// Brackets one launch with events when timing is on (see flare_profile_enable).
struct LaunchTimer {
    LaunchTimer(int kid, hipStream_t stream);
    ~LaunchTimer();
    int slot;
    hipStream_t stream;
};

// ---- how the token axis is split over workgroups -------------------------------------------
struct Split {
    int chunks;     // number of token chunks per (b,h)
    int chunk_len;  // tokens per chunk (the last chunk may be shorter, never empty)
};
Split plan_split(int N, int BH, int min_len, int target_blocks);

// ---- where a row of a token tensor (k, v, y, dy, dk, dv) lives --------------------------------
// Element (b, h, n, j) is at b*sb + h*sh + n*sn + j (in elements), for either layout of flare.h.
// sq: elements between the latent queries of consecutive heads (M*d, or 0 when all heads share one
// latent sequence): head h's queries start at q_lat + h*sq.
struct TokStride {
    long long sb, sh, sn, sq;
};
inline TokStride tok_stride(const flare_shape &s)
{
    const long long H = s.H, N = s.N, d = s.d;
    const long long sq = s.shared_latents ? 0 : (long long)s.M * d;
    if (s.layout == FLARE_BNHD) return TokStride{N * H * d, d, H * d, sq};
    return TokStride{H * N * d, N * d, d, sq};
}
__device__ __forceinline__ size_t tok_base(const TokStride &t, int bh, int H)
{
    return (size_t)(bh / H) * (size_t)t.sb + (size_t)(bh % H) * (size_t)t.sh;
}
// Offset of token n's row inside its (b,h) slice.  A full-rate 24-bit multiply: the entry points
// admit only shapes with N < 2^24 and N * sn < 2^32 (see check_shape).
__device__ __forceinline__ size_t tok_off(const TokStride &t, int n)
{
    return (size_t)__umul24((unsigned)n, (unsigned)t.sn);
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// ---- fp32 vector-ALU path (any M, d in {4,8,16,32}, f32 or bf16 storage) -------------------
struct ValuPlan {
    Split enc;          // split used by the encode partials
    Split bwd;          // split used by the dZ and dQ partials
    size_t fwd_bytes;   // workspace for encode
    size_t bwd_bytes;   // workspace for backward
};
ValuPlan valu_plan(const flare_shape &s);

// Carves the encode workspace for sp.chunks partial slots per (b,h); returns its size in bytes.
// Any of the output pointers may be NULL (then ws is not touched).
size_t valu_fwd_layout(const flare_shape &s, const Split &sp, void *ws, float **m_part, float **l_part,
                       float **o_part);
// Fixed-order merge of `parts` partial slots per (b,h) into z and lse_enc (shared by both paths).
int launch_encode_merge(const flare_shape &s, const float *m_part, const float *l_part, const float *o_part,
                        float *z, float *lse_enc, int parts, hipStream_t stream);

int valu_encode(const flare_shape &s, const void *q, const void *k, const void *v, float *z,
                float *lse_enc, float scale, void *ws, hipStream_t stream);
int valu_decode(const flare_shape &s, const void *q, const void *k, const float *z, void *y,
                float *lse_dec, float scale, hipStream_t stream);
// The whole backward; uses the matrix-core kernels where the shape allows.  y and lse_dec may be
// NULL (then the token statistics are recomputed).
int valu_backward(const flare_shape &s, const void *q, const void *k, const void *v, const void *y,
                  const float *lse_dec, const void *dy, const float *z, const float *lse_enc, float *dq,
                  void *dk, void *dv, float scale, void *ws, hipStream_t stream);

// ---- bf16 matrix-core path (d in {16,32}; M = 32 or a multiple of 64 up to 256) --------------
struct MfmaPlan {
    Split enc;   // token chunks of the encode (one workgroup each)
    int parts;   // partial slots per (b,h) = chunks * token groups per workgroup
};
bool mfma_supported(const flare_shape &s);
MfmaPlan mfma_plan(const flare_shape &s);
size_t mfma_fwd_bytes(const flare_shape &s);
int mfma_encode(const flare_shape &s, const void *q, const void *k, const void *v, float *z,
                float *lse_enc, float scale, void *ws, hipStream_t stream);
// Shapes with M > 256 run the token-major kernels once per chunk of 256 latents.  The decode and the
// token statistics then need mfma_tok_part_bytes(s) of scratch (`ws`; unused and may be NULL
// otherwise), the dK/dV step mfma_dkdv_acc_bytes(s) for its fp32 sums.
size_t mfma_tok_part_bytes(const flare_shape &s);
size_t mfma_dkdv_acc_bytes(const flare_shape &s);
int mfma_decode(const flare_shape &s, const void *q, const void *k, const float *z, void *y,
                float *lse_dec, float scale, void *ws, hipStream_t stream);
// decode fused with the output projection (flare_mfma_proj.hip); y and lse_dec may be NULL
bool mfma_project_supported(const flare_shape &s);
int mfma_decode_project(const flare_shape &s, const void *q, const void *k, const float *z, const void *w_out,
                        const float *bias, void *out, void *y, float *lse_dec, float scale, hipStream_t stream);
int mfma_token_stats(const flare_shape &s, const void *q, const void *k, const float *z, const void *dy,
                     float *lse_dec2, float *delta, float scale, void *ws, hipStream_t stream);
bool mfma_dkdv_supported(const flare_shape &s);
// In the backward launchers below the per-token decode statistic is read as
// ld_mul * lse_dec2[n]: pass the workspace array with ld_mul = 1, or the forward's natural-log
// lse_dec with ld_mul = log2(e).
int mfma_dkdv(const flare_shape &s, const void *q, const void *k, const void *v, const void *dy, const float *z,
              const float *lse_enc, const float *dz, const float *eps, const float *lse_dec2, const float *delta,
              float ld_mul, const int *plan, void *dk, void *dv, float *acc32, float *dq_part, int m0, float scale,
              hipStream_t stream);
int mfma_dkdv_blocks(const flare_shape &s);
bool mfma_dq_fused(const flare_shape &s);
int mfma_dq_parts(const flare_shape &s);
int mfma_dq_partial(const flare_shape &s, const void *q, const void *k, const void *v, const void *dy,
                    const float *z, const float *lse_enc, const float *dz, const float *eps,
                    const float *lse_dec2, const float *delta, float ld_mul, const int *plan, float *dq_part,
                    float scale, hipStream_t stream);
// y and delta_out may be NULL; when given, delta_out[b][h][n] = <dY_n, Y_n> is written as a by-product.
int mfma_dz_partial(const flare_shape &s, const void *q, const void *k, const void *dy, const float *lse_dec2,
                    float ld_mul, const void *y, float *delta_out, float *ld_range, float *dz_part, float scale,
                    hipStream_t stream);
// The dQ and dK/dV kernels exist in two variants, one and two exponentials per score.  Both are
// launched; each leaves at once the (b,h) slices that plan[b*h] (1 = one exponential) gives to the
// other.  ld_range[b*h][part] = (min, max) of lse_dec2 as mfma_dz_partial recorded it.
// One exponential: P~ = 2^S2 as it comes, without a normaliser (S2 <= lse_enc2[m] and S2 <= lse_dec2[n], so with
// both log-sum-exps of a (b,h) within +-kPlanSpan nothing overflows and every weight that matters is a normal
// number), P = P~ e_m with e_m = 2^-lse_enc2[m] and R = P~ w_n with w_n = 2^-lse_dec2[n]:
//   dS = P (a - eps) + R (c - delta) = P~ (e_m (a - eps_m) + w_n (c - delta_n)),   dV += (e_m dZ_m) P~.
// e_m is folded into dZ where its partials are merged, BEFORE dZ is rounded to bf16 and eps = <dZ, Z> is formed
// (bwd_one_exp_ok decides there, and the kernels that follow take dZ and eps as they find them), so that a and
// eps still see the same rounded values and the score products need no correction k-step; w_n is a per-token
// scalar.  Anything else (log-sum-exps beyond +-kPlanSpan, non-finite statistics) takes the two-exponential
// kernels with dZ as it is.
// Called by a whole workgroup of 256 threads (of the kernel that merges the dZ partials: everything it reads is
// complete by then), all of whose threads take part in the reads (one memory latency, not one per 64 values);
// one barrier inside; every thread returns the same answer.  red: 16 floats of LDS.
constexpr float kPlanSpan = 60.f;
__device__ __forceinline__ bool bwd_one_exp_ok(const float *__restrict__ ld_range, const float *__restrict__ lse_enc,
                                               int bh, int parts, int M, int force_two, float *red)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // extremes of lse_enc2, as (max, -min), and of lse_dec2 likewise: one maximum each
    float le_hi = -INFINITY, le_lo = -INFINITY, ld_hi = -INFINITY, ld_lo = -INFINITY;
    bool nan = false;
    for (int m = tid; m < M; m += 256) {
        const float v = lse_enc[(size_t)bh * M + m] * 1.4426950408889634f;
        nan |= v != v;
        le_hi = fmaxf(le_hi, v);
        le_lo = fmaxf(le_lo, -v);
    }
    for (int p = tid; p < parts; p += 256) {
        const float a = ld_range[2 * ((size_t)bh * parts + p)], b = ld_range[2 * ((size_t)bh * parts + p) + 1];
        nan |= a != a || b != b;
        ld_lo = fmaxf(ld_lo, -a);
        ld_hi = fmaxf(ld_hi, b);
    }
    if (nan) le_hi = INFINITY;                       // a NaN anywhere makes the test fail
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        le_hi = fmaxf(le_hi, __shfl_xor(le_hi, off));
        le_lo = fmaxf(le_lo, __shfl_xor(le_lo, off));
        ld_hi = fmaxf(ld_hi, __shfl_xor(ld_hi, off));
        ld_lo = fmaxf(ld_lo, __shfl_xor(ld_lo, off));
    }
    if (lane == 0) { red[4 * wave] = le_hi; red[4 * wave + 1] = le_lo; red[4 * wave + 2] = ld_hi; red[4 * wave + 3] = ld_lo; }
    __syncthreads();
    float worst = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) worst = fmaxf(worst, red[i]);
    return worst <= kPlanSpan && !force_two;
}

// ---- spectral analysis (Appendix C.1, Algorithm 1) ---------------------------------------------
bool mfma_gram_supported(const flare_shape &s);
int mfma_gram_partial(const flare_shape &s, const Split &sp, const void *q, const void *k, const float *lse_enc,
                      const float *lse_dec, float *g_part, float scale, hipStream_t stream);
size_t spectral_bytes(const flare_shape &s);
int spectral_run(const flare_shape &s, const void *q, const void *k, const float *lse_enc, const float *lse_dec,
                 float scale, int first, float *evals, float *zvec, float *gram, void *ws, hipStream_t stream);

}  // namespace flare
