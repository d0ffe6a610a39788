/*
 * flare.h -- C ABI of libflare.so: FLARE's encode-decode token mixer on one MI355X (gfx950).
 *
 * The operator (paper Section 3.1, Eq. flare_encode and Eq. flare_decode; multi-head listing
 * of the same section with shapes Q:[H M D], K,V:[B H N D] -> Y:[B H N D]):
 *
 *     S[m][n]  = scale * <q_lat[h][m][:], k[b][h][n][:]>          one score matrix per (b,h)
 *     Z[m][:]  = sum_n softmax_n(S[m][.])[n] * v[b][h][n][:]       encode: softmax over N tokens
 *     Y[n][:]  = sum_m softmax_m(S[.][n])[m] * Z[m][:]             decode: softmax over M latents
 *
 * `scale` is a MULTIPLIER on q.k and is the same in both halves (the paper's listing passes
 * scale=1.0 to both attention calls; its Eq. sdpa writes a division by s, which coincides at
 * s=1).  The latent queries are shared by all batch items.  The M x N weights are never
 * written to memory.  There is no mask, dropout or bias.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller, contiguous with innermost
 *     dimension d, and 16-byte aligned.  The library allocates and frees nothing on the hot
 *     path, never synchronises the device, and only enqueues work on `stream` (a hipStream_t
 *     passed as void*; NULL is the default stream).  Results are ready when the stream reaches
 *     the point after the call.
 *   - Outputs are overwritten, never accumulated into.
 *   - `workspace` is caller-provided device scratch of at least the size that
 *     flare_workspace_bytes reports for the same shape; its contents are undefined on return.
 *     Two calls that share a workspace must be ordered on the same stream.
 *   - Return value: FLARE_OK (0) or a negative flare_status.  Nothing is launched when an
 *     argument check fails.  A launch failure reported by the HIP runtime gives FLARE_ELAUNCH.
 *   - Supported shapes: B,H,N,M >= 1 with B*H <= 65535, N < 2^24 and N times the token stride in
 *     elements (d, or H*d for FLARE_BNHD) below 2^32; d in {4, 8, 16, 32}; dtype f32, bf16 or f16;
 *     either flare_layout for the token tensors (every "[B][H][N][d]" below reads [B][N][H][d]
 *     when shape->layout is FLARE_BNHD; the per-token statistic lse_dec is [B][H][N] always).
 *     Shapes with dtype bf16 or f16, M <= 2048 and N >= 16 run on the matrix-core kernels (d < 16 with the
 *     contraction padded to 16; M in tiles of 32 on the geometry of the next of 32, 64, 128, 256
 *     or a multiple of 256, the latents beyond M being padding that is masked; M > 256 in chunks
 *     of 256 latents); everything else runs on the fp32 vector kernels.  On the matrix
 *     cores the scores come from exact products of the stored 16-bit values, the softmax weights
 *     and dS are rounded to bf16 whatever the storage type (with f16 storage v and dy are rounded
 *     to bf16 as they are read), sums are fp32, and outputs are rounded once from fp32.  With f16
 *     storage scale*log2(e)*q_lat and the scaled scores must stay below 65504 in magnitude.
 *   - Results are bit-identical from run to run for the same inputs and shape (no float atomics;
 *     every cross-block reduction is done in a fixed order).
 *   - Non-finite inputs give undefined results.
 */
#ifndef FLARE_H
#define FLARE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FLARE_F32 = 0,   /* q_lat, k, v, y, dy, dk, dv are IEEE fp32 */
    FLARE_BF16 = 1,  /* ... are bfloat16; all accumulation and the saved statistics stay fp32 */
    FLARE_F16 = 2    /* ... are IEEE fp16 (the paper's autocast type, Appendix G); likewise */
} flare_dtype;

typedef enum {
    FLARE_OK = 0,
    FLARE_EINVAL = -1,        /* null pointer, non-positive dimension, null shape */
    FLARE_EUNSUPPORTED = -2,  /* d, dtype, layout or B*H outside the supported set */
    FLARE_EALIGN = -3,        /* a data pointer is not 16-byte aligned */
    FLARE_EWORKSPACE = -4,    /* workspace is NULL or smaller than flare_workspace_bytes reports */
    FLARE_ELAUNCH = -5,       /* the HIP runtime rejected a launch or an event call */
    FLARE_ESTATIC = -6        /* flare_forward_static: the shape needs more scratch than FLARE_STATIC_SCRATCH_BYTES */
} flare_status;

typedef enum {
    FLARE_BHND = 0,  /* token tensors are [B][H][N][d]: one contiguous [N][d] slab per head */
    FLARE_BNHD = 1   /* token tensors are [B][N][H][d] = [B][N][C] with C = H*d, the layout the block's
                        linear projections produce (listing in Section 3.1 before its head split) */
} flare_layout;

typedef struct {
    int B;              /* batch items */
    int H;              /* heads; head h uses its own slice of M latent queries */
    int N;              /* tokens per batch item */
    int M;              /* latent queries per head */
    int d;              /* head dimension D = C / H */
    flare_dtype dtype;  /* element type of q_lat, k, v, y, dy, dk, dv */
    flare_layout layout; /* memory order of the token tensors k, v, y, dy, dk, dv (0 = [B][H][N][d]);
                            q_lat, z, lse_enc, lse_dec and dq_lat do not depend on it */
    int shared_latents;  /* 0: every head has its own M latent queries, q_lat and dq_lat are [H][M][d]
                            (Section 3.1).  1: all heads use one latent sequence (the shared-latent
                            variant of the ablation in Appendix G): q_lat and dq_lat are [M][d], and
                            dq_lat is summed over the heads as well as over the batch */
    int y_f32;           /* 0: y has the element type dtype.  1 (16-bit dtypes with M <= 2048, else
                            FLARE_EUNSUPPORTED): flare_decode / flare_forward write y as fp32 (same layout),
                            and the y handed to flare_backward is that fp32 tensor.  The backward then takes
                            delta_n = <dY_n, Y_n> from an unrounded Y, so that no shape of 16 tokens or more
                            needs the recomputation described at flare_backward (at d < 16 that pass is a
                            sixth of the step), at the price of a y of twice the bytes */
    int variant;         /* 0: the library picks its kernels.  Otherwise a set of flare_variant bits that forces
                            a kernel variant the library would not pick for this shape or these inputs (tests and
                            A/B measurements of flare_backward; results stay within the same tolerances).  Bits
                            that do not apply to a shape are ignored; unknown bits give FLARE_EINVAL */
} flare_shape;

typedef enum {
    FLARE_VARIANT_TWO_EXP = 1,      /* backward: both softmax weights of a score from an exponential of their own
                                       in every (b,h), as for inputs whose normalisers span too wide a range */
    FLARE_VARIANT_SEPARATE_DQ = 2   /* backward, d <= 16: dQ from the latent-major kernel of its own (as at d = 32)
                                       instead of out of the dK/dV kernel */
} flare_variant;

/* Library version: major*10000 + minor*100 + patch. */
int flare_version(void);

/* Static, NUL-terminated description of a flare_status value. */
const char *flare_strerror(int status);

/* Scratch bytes that flare_forward / flare_encode / flare_decode (fwd_bytes) and flare_backward
 * (bwd_bytes) need for this shape.  Either output pointer may be NULL.  Host-only; touches no
 * device. */
int flare_workspace_bytes(const flare_shape *shape, size_t *fwd_bytes, size_t *bwd_bytes);

/*
 * Encode (Eq. flare_encode; Appendix F, per-latent form of z_m): split-N partial softmax
 * reductions followed by a fixed-order merge.
 *   q_lat [H][M][d] dtype, k, v [B][H][N][d] dtype                         (in)
 *   z       [B][H][M][d] fp32: the latent sequence Z                        (out)
 *   lse_enc [B][H][M]    fp32: log sum_n exp(S[m][n]), natural log          (out)
 */
int flare_encode(const flare_shape *shape, const void *q_lat, const void *k, const void *v,
                 float *z, float *lse_enc, float scale,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Decode (Eq. flare_decode; Appendix F, per-token form of y_n): per-token softmax over the M
 * latents applied to Z.  Only matrix-core shapes with M > 256 use the workspace (per-chunk partial
 * results, merged in chunk order); for all others it may be NULL.
 *   q_lat [H][M][d] dtype, k [B][H][N][d] dtype, z [B][H][M][d] fp32        (in)
 *   y [B][H][N][d] dtype                                                    (out)
 *   lse_dec [B][H][N] fp32: log sum_m exp(S[m][n]), natural log; may be NULL (out, optional)
 */
int flare_decode(const flare_shape *shape, const void *q_lat, const void *k, const float *z,
                 void *y, float *lse_dec, float scale,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Forward of the mixer = flare_encode then flare_decode on the same stream (listing in
 * Section 3.1).  z and lse_enc are outputs the caller keeps for flare_backward; lse_dec (may be
 * NULL) is a third one that saves the backward one pass over the scores.
 */
int flare_forward(const flare_shape *shape, const void *q_lat, const void *k, const void *v,
                  void *y, float *z, float *lse_enc, float *lse_dec, float scale,
                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * Decode fused with the linear layer that follows the mixer in a FLARE block (Section 3.1: "the outputs from all
 * heads are concatenated along the feature dimension and passed through a final linear projection"; Appendix B.2,
 * "FLARE": a single linear layer):
 *     out[b][n][:] = concat_h(Y_h[b][n][:]) . w_out + bias,        C = H * d,
 * so that y need not be written and read back between the two (it is still written when y is not NULL, e.g. for
 * flare_backward).  One workgroup per 32-token tile with one wave per head; the sum over the heads is the
 * contraction of one matrix product, in a fixed order (bit-reproducible).
 *   q_lat, k, z as for flare_decode, with shape->layout = FLARE_BNHD (k is [B][N][H][d] = [B][N][C])      (in)
 *   w_out [C][C] of the storage dtype, row = input channel h*d + j, column = output channel               (in)
 *   bias  [C] fp32, or NULL                                                                               (in, optional)
 *   out   [B][N][C] of the storage dtype (rounded once from fp32)                                         (out)
 *   y     [B][N][H][d] dtype, lse_dec [B][H][N] fp32: as flare_decode writes them, or NULL              (out, optional)
 * Supported (else FLARE_EUNSUPPORTED, nothing launched): dtype bf16 or f16, layout FLARE_BNHD, d = 16,
 * H in {2, 4, 8}, M <= 256, N >= 16, y_f32 = 0.  The rows of Y enter the projection rounded to the storage
 * dtype, exactly the values a separate flare_decode would have stored.  Needs no workspace.
 * flare_forward_project = flare_encode followed by flare_decode_project on the same stream.
 */
int flare_decode_project(const flare_shape *shape, const void *q_lat, const void *k, const float *z,
                         const void *w_out, const float *bias, void *out, void *y, float *lse_dec, float scale,
                         void *stream);
int flare_forward_project(const flare_shape *shape, const void *q_lat, const void *k, const void *v,
                          const void *w_out, const float *bias, void *out, void *y, float *z, float *lse_enc,
                          float *lse_dec, float scale, void *workspace, size_t workspace_bytes, void *stream);

/*
 * flare_forward for callers that cannot allocate and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and kernels as
 * flare_forward, but the scratch (the encode's per-wave partial sums; with M > 256 also the decode's
 * per-chunk rows) lives in an array of FLARE_STATIC_SCRATCH_BYTES that the library's code object holds in
 * device memory, once per GPU the library runs on, until the process ends.  The call allocates and frees
 * nothing and calls no allocating routine; on its first call on a device it looks the array's address up
 * (hipGetSymbolAddress) and keeps it, so make that first call outside a capture.  A shape whose
 * flare_workspace_bytes forward size exceeds FLARE_STATIC_SCRATCH_BYTES is refused with FLARE_ESTATIC and
 * nothing is launched (the five reference workloads need 0.5 ... 18 MiB).  Nothing in the array has to start
 * at zero (every partial slot is written before it is read), so no clearing is enqueued.  All calls on one GPU
 * share the one array: calls that overlap there (different streams, or different threads without ordering)
 * race; order them on one stream.
 */
#define FLARE_STATIC_SCRATCH_BYTES (32u << 20)
int flare_forward_static(const flare_shape *shape, const void *q_lat, const void *k, const void *v,
                         void *y, float *z, float *lse_enc, float *lse_dec, float scale, void *stream);

/*
 * Backward of the mixer.  The paper differentiates its two attention calls automatically
 * (Appendix G, "Time and memory complexity": one forward and backward pass is what it
 * times); the gradients follow from the softmax Jacobian.  With P = softmax_n(S) (M x N),
 * R = softmax_m(S^T) (N x M), Z = P V, Y = R Z:
 *     dZ = R^T dY,  delta_n = <dY_n, Y_n>,  eps_m = <dZ_m, Z_m>,  dV = P^T dZ,
 *     dS[m][n] = P[m][n](<dZ_m, V_n> - eps_m) + R[n][m](<dY_n, Z_m> - delta_n),
 *     dK_n = scale * sum_m dS[m][n] q_m,   dQ_m = scale * sum_n dS[m][n] k_n  summed over B.
 *   q_lat, k, v as in the forward; dy [B][H][N][d] dtype                    (in)
 *   z, lse_enc: what flare_forward wrote for the same inputs                (in)
 *   y, lse_dec: what flare_forward wrote, or NULL.  When both are given, delta_n is taken from
 *     the stored y and the decode normaliser from lse_dec; when either is NULL both are
 *     recomputed from z (one more pass over the scores, Y in fp32).  With bf16 storage (or f16
 *     storage on the matrix-core kernels) and d < 16, or at most 32 tokens, or fewer tokens than latents, they are recomputed in
 *     either case: delta from a y of bf16 accuracy and so few terms would not meet the accuracy of
 *     the rest -- unless shape->y_f32 is set and y is the forward's fp32 output.  (16-bit shapes of
 *     fewer than 16 tokens run on the fp32 kernels throughout, forward and backward: with so few tokens
 *     the gradients' differences cancel too far for bf16 operands.)
 *                                                                           (in, optional)
 *   dq_lat [H][M][d] fp32 (summed over the batch), dk, dv [B][H][N][d] dtype (out)
 */
int flare_backward(const flare_shape *shape, const void *q_lat, const void *k, const void *v,
                   const void *y, const float *lse_dec, const void *dy, const float *z,
                   const float *lse_enc, float *dq_lat, void *dk, void *dv, float scale,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * Eigenpairs of the mixing matrix W = W_decode W_encode (N x N, rank <= M) of every (b,h) without
 * forming it (Appendix C.1 "Eigenanalysis procedure", Algorithm 1): with A = exp(S),
 * L_M = 1 / row sums, L_N = 1 / column sums and J = L_M^(1/2) A L_N^(1/2), the nonzero eigenvalues
 * of W are those of the M x M matrix J J^T = U Sigma^2 U^T and its eigenvectors are
 * L_N^(1/2) J^T U Sigma^(-1) = W_decode (L_M^(1/2) U Sigma^(-1)).  The library forms J J^T in one
 * pass over the tokens, diagonalises it on the device in fp64 (Householder reduction to
 * tridiagonal form, bisection for all eigenvalues, a twisted factorisation and the reflectors
 * for the requested eigenvectors only; one workgroup per (b,h)) and returns
 *   eigenvalues [B][H][M] fp32, in descending order                                   (out)
 *   z_vec [B][H][M][d] fp32 = L_M^(1/2) U Sigma^(-1) restricted to the eigenvectors number
 *         first .. first + d - 1 (zero beyond M or where the eigenvalue is not positive): passed
 *         as `z` to flare_decode it yields those d eigenvectors of W, one per column of y   (out)
 *   gram [B][H][M][M] fp32 = J J^T; may be NULL                                       (out, optional)
 *   q_lat, k as in the forward; lse_enc, lse_dec: what flare_forward wrote             (in)
 * Supported for M <= 512.  flare_spectral_workspace_bytes gives the scratch size (partial sums of
 * J J^T plus one fp64 M x M matrix and 3 d vectors per (b,h)).  Eigenvectors are defined up to
 * sign; those of a repeated eigenvalue span its eigenspace.  z_vec is fp32 and carries the
 * factor exp(-lse_enc[m] / 2): scores whose log-sum-exp exceeds ~170 underflow it.  A (b,h)
 * with non-finite input gets NaN eigenvalues and a zero z_vec; the call still returns
 * FLARE_OK, as the forward does for non-finite inputs.
 */
int flare_spectral_workspace_bytes(const flare_shape *shape, size_t *bytes);
int flare_spectral(const flare_shape *shape, const void *q_lat, const void *k, const float *lse_enc,
                   const float *lse_dec, float scale, int first, float *eigenvalues, float *z_vec,
                   float *gram, void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FLARE_H */
