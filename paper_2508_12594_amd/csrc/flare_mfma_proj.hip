// Decode fused with the output projection that follows the mixer (Section 3.1: the head outputs are
// concatenated along the feature dimension and passed through a final linear projection; Appendix B.2,
// "FLARE": a single linear layer):
//     out[b][n][:] = concat_h(Y_h[b][n][:]) . W_out + bias,     Y_h = softmax_m(K_h Q_h^T) Z_h  (Eq. flare_decode).
// Token tensors in the [B][N][H][d] order the block's projections produce, d = 16, so one token's keys of all
// heads are one contiguous row of C = 16 H elements and so is its output row.
//
// A workgroup has one wave per head and walks over 32-token tiles; wave h decodes head h of the tile exactly as
// decode_mfma_kernel does (Q_h and Zaug_h^T in registers, one sweep over the latent tiles, the stabiliser from
// the first latent tile, an exact second attempt when a denominator overflows).  The normalised rows of Y_h are
// rounded to the storage type -- the same values a separate decode would store -- and written into a tile
// Y[32 tokens][C] in LDS; after one barrier wave w multiplies the whole tile with its 16 columns of W_out,
//     out^T[c'][n] = sum_c W_out[c][c'] Y[n][c],   c' = 16 w .. 16 w + 15,   with v_mfma_f32_16x16x32,
// (W_out^T as the A operand, resident in registers; Y rows straight from the LDS tile as the B operand), adds the
// bias and stores its 32-byte piece of each output row.  The sum over the heads is the contraction of that
// product: a fixed order, no atomics, bit-reproducible.  The LDS tile is double-buffered: one barrier per tile.
// Optionally the kernel also stores y (and lse_dec) for a backward pass.
#include "flare_mfma_common.h"

namespace flare {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kProjPad = 8;   // 16-bit elements of padding per LDS row of the Y tile (rows of 2 C + 16 bytes)

template <bool F>
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c)
{
    if constexpr (F)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// MT: 32-latent tiles per head (padded geometry); HW: waves = heads; F: fp16 storage.
// (Launch bounds: two waves per SIMD need at most 256 registers; with two waves per workgroup a minimum of four
// workgroups per CU made the compiler keep to 128 registers and spill at four and more latent tiles.)
template <int MT, int HW, bool F>
__global__ __launch_bounds__(64 * HW, HW == 8 ? 1 : 2) void decode_project_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const float *__restrict__ z,
    const bf16_t *__restrict__ w_out, const float *__restrict__ bias, bf16_t *__restrict__ out,
    bf16_t *__restrict__ y, float *__restrict__ lse_dec, long long sq, int N, int Mtot, float c2)
{
    constexpr int DR = 16, C = 16 * HW, KP = C / 32;          // KP: k-steps of the projection (HW >= 2)
    constexpr int ROW = C + kProjPad;                          // uint16 per LDS row
    __shared__ __attribute__((aligned(16))) uint16_t ytile[2][32 * ROW];
    const int lane = threadIdx.x & 63, l32 = lane & 31, hh = lane >> 5;
    const int h = threadIdx.x >> 6;                            // this wave's head
    const int b = blockIdx.y;
    const int c16 = lane & 15, g16 = lane >> 4;

    // ---- resident operands: q' (hi, lo) and Zaug^T of this head, W_out^T columns 16 h .. 16 h + 15 ----
    bf16x8 qh[MT][1], ql[MT][1];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int m = 32 * t + l32;
        load_q_operand<DR, true, F, false>(q + (size_t)h * sq + (size_t)min(m, Mtot - 1) * DR, hh, c2, false, qh[t], ql[t]);
    }
    bf16x8 zt[2 * MT];
    {
        const float *zb = z + ((size_t)(b * HW + h) * Mtot) * DR;
#pragma unroll
        for (int s = 0; s < 2 * MT; ++s) {
            u32x4 w;
#pragma unroll
            for (int i = 0; i < 8; i += 2) {
                const int la = 32 * (s / 2) + perm_index(s % 2, hh, i), lb = 32 * (s / 2) + perm_index(s % 2, hh, i + 1);
                float a, bb;
                if (l32 < 16) {          // rows 0-15: columns of Z; a padding latent's row is zero
                    a = la < Mtot ? zb[(size_t)la * DR + l32] : 0.f;
                    bb = lb < Mtot ? zb[(size_t)lb * DR + l32] : 0.f;
                } else {                 // row 16: ones for the real latents (the denominator); the rest zero
                    a = (l32 == 16 && la < Mtot) ? 1.f : 0.f;
                    bb = (l32 == 16 && lb < Mtot) ? 1.f : 0.f;
                }
                w[i / 2] = rne_bf16(a) | (rne_bf16(bb) << 16);
            }
            zt[s] = as_bf16x8(w);
        }
    }
    bf16x8 wa[KP];                       // A operand: row c' = 16 h + lane % 16, slots c = 32 ks + 8 (lane / 16) + i
#pragma unroll
    for (int ks = 0; ks < KP; ++ks) {
        u32x4 w;
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
            const int c0 = 32 * ks + 8 * g16 + i;
            const uint32_t lo = w_out[(size_t)c0 * C + 16 * h + c16], hi = w_out[(size_t)(c0 + 1) * C + 16 * h + c16];
            w[i / 2] = lo | (hi << 16);
        }
        wa[ks] = as_bf16x8(w);
    }
    float bs[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) bs[r] = bias ? bias[16 * h + 4 * g16 + r] : 0.f;

    const size_t row_stride = (size_t)C;                       // elements between tokens in k, y, out
    const bf16_t *kb = k + (size_t)b * N * row_stride + (size_t)h * DR;
    const int tiles = (N + 31) / 32;
    bf16x8 kt, ktn;
    int tile = blockIdx.x;
    // The decode of one head, as in decode_mfma_kernel, operation for operation (y is bit-identical): the stabiliser
    // of a token tile is the maximum of the hi product of its first latent tile; the scores of that latent tile are
    // the same product minus the stabiliser plus the lo product; the last latent tile requests the first hi
    // product of the wave's next token tile.
    auto qk_hi = [&](int t, bf16x8 kk) { return mfma_s<F>(qh[t][0], kk, splat16(0.f)); };
    auto tile_max = [&](const f32x16 &hi) {
        const float m = max16(hi, -INFINITY);
        return fmaxf(m, __shfl_xor(m, 32));
    };
    auto first_scores = [&](f32x16 hi, float m, bf16x8 kk) {
#pragma unroll
        for (int i = 0; i < 16; ++i) hi[i] -= m;
        return mfma_s<F>(ql[0][0], kk, hi);
    };
    float mx = 0.f;
    f32x16 s_cur0 = splat16(0.f);
    if (tile < tiles) {
        kt = as_bf16x8(*reinterpret_cast<const u32x4 *>(kb + (size_t)min(tile * 32 + l32, N - 1) * row_stride + 8 * hh));
        const f32x16 hi = qk_hi(0, kt);
        mx = tile_max(hi);
        s_cur0 = first_scores(hi, mx, kt);
    }
    for (int it = 0; tile < tiles; tile += gridDim.x, ++it) {
        const int n = tile * 32 + l32;
        {   // keys of the workgroup's next tile (the last one is simply loaded again)
            const int tn = (tile + (int)gridDim.x < tiles) ? tile + (int)gridDim.x : tile;
            ktn = as_bf16x8(*reinterpret_cast<const u32x4 *>(kb + (size_t)min(tn * 32 + l32, N - 1) * row_stride + 8 * hh));
        }
        bf16x8 kt2;
        {
            u32x4 w = __builtin_bit_cast(u32x4, kt);
            asm volatile("" : "+v"(w));                        // keeps the hi products apart from the lo ones
            kt2 = as_bf16x8(w);
        }
        f32x16 acc;
        auto sweep = [&](f32x16 s_cur, const f32x16 cinit, auto ahead_tag) {
            constexpr bool AHEAD = decltype(ahead_tag)::value;
            f32x16 s_next = s_cur;
            acc = splat16(0.f);
            sched_fence();
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                // dependent pairs alternate (hi, value, lo, value), as in decode_mfma_kernel
                if (t + 1 < MT) s_next = mfma_s<F>(qh[t + 1][0], kt2, cinit);
                else if constexpr (AHEAD) s_next = qk_hi(0, ktn);
                bf16x8 p0, p1;
                exp_pack(s_cur, p0, p1);
                acc = mfma(zt[2 * t], p0, acc);
                if (t + 1 < MT) s_next = mfma_s<F>(ql[t + 1][0], kt, s_next);
                acc = mfma(zt[2 * t + 1], p1, acc);
                if (t + 1 < MT) {
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_MFMA(1);
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_VALU(4);
                    FLARE_GROUP_MFMA(1);
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_MFMA(1);
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_VALU(4);
                    FLARE_GROUP_MFMA(1);
                } else if (AHEAD) {
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_MFMA(1);
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_VALU(4);
                    FLARE_GROUP_MFMA(1);
                    FLARE_GROUP_TRANS(8);
                    FLARE_GROUP_VALU(4);
                    FLARE_GROUP_MFMA(1);
                } else {
                    FLARE_GROUP_TRANS(8);
                    FLARE_GROUP_VALU(4);
                    FLARE_GROUP_MFMA(1);
                    FLARE_GROUP_TRANS(8);
                    FLARE_GROUP_VALU(4);
                    FLARE_GROUP_MFMA(1);
                }
                sched_fence();
                s_cur = s_next;
            }
            return s_cur;
        };
        f32x16 s_ahead = sweep(s_cur0, splat16(-mx), PlainTag<true>{});
        // a denominator at or beyond 2^64 (or not finite): once more with the exact maximum over all latent tiles
        if (__any((__float_as_uint(acc[8]) & 0x7f800000u) >= ((127u + 64u) << 23))) {
            float m = -INFINITY;
            f32x16 hi0 = qk_hi(0, kt), s_cur = hi0, s_next = hi0;
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                if (t + 1 < MT) s_next = qk_hi(t + 1, kt);
                sched_fence();
                m = max16(s_cur, m);
                s_cur = s_next;
            }
            mx = fmaxf(m, __shfl_xor(m, 32));
            (void)sweep(first_scores(hi0, mx, kt), splat16(-mx), PlainTag<false>{});
            s_ahead = qk_hi(0, ktn);
        }
        const float mx_next = tile_max(s_ahead);
        s_cur0 = first_scores(s_ahead, mx_next, ktn);
        const float den = __shfl(acc[8], l32);
        const float inv = 1.f / den;
        // this lane: token l32, columns 4 hh .. 4 hh + 3 (registers 0-3) and 8 + 4 hh .. (registers 4-7) of Y_h
        u32x2 w0, w1;
        w0[0] = pack_elems<F>(acc[0] * inv, acc[1] * inv);
        w0[1] = pack_elems<F>(acc[2] * inv, acc[3] * inv);
        w1[0] = pack_elems<F>(acc[4] * inv, acc[5] * inv);
        w1[1] = pack_elems<F>(acc[6] * inv, acc[7] * inv);
        uint16_t *yt = ytile[it & 1] + l32 * ROW + 16 * h;
        *reinterpret_cast<u32x2 *>(yt + 4 * hh) = w0;
        *reinterpret_cast<u32x2 *>(yt + 8 + 4 * hh) = w1;
        if (n < N) {
            if (y != nullptr) {
                bf16_t *yr = y + ((size_t)b * N + n) * row_stride + (size_t)h * DR;
                *reinterpret_cast<u32x2 *>(yr + 4 * hh) = w0;
                *reinterpret_cast<u32x2 *>(yr + 8 + 4 * hh) = w1;
            }
            if (lse_dec != nullptr && hh == 0) lse_dec[((size_t)(b * HW + h)) * N + n] = (mx + log2f(den)) * kLn2;
        }
        __syncthreads();     // every head's columns of this tile are in LDS
        // ---- projection: this wave's 16 output columns for the 32 tokens of the tile ----
        f32x4 pacc[2];
        pacc[0] = f32x4{0.f, 0.f, 0.f, 0.f};
        pacc[1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int th = 0; th < 2; ++th)
#pragma unroll
            for (int ks = 0; ks < KP; ++ks) {
                const u32x4 bop = *reinterpret_cast<const u32x4 *>(ytile[it & 1] + (16 * th + c16) * ROW + 32 * ks + 8 * g16);
                pacc[th] = mfma16<F>(wa[ks], as_bf16x8(bop), pacc[th]);
            }
#pragma unroll
        for (int th = 0; th < 2; ++th) {     // rows c' = 16 h + 4 (lane / 16) + r, column token 16 th + lane % 16
            const int nt = tile * 32 + 16 * th + c16;
            if (nt < N) {
                u32x2 w;
                w[0] = pack_elems<F>(pacc[th][0] + bs[0], pacc[th][1] + bs[1]);
                w[1] = pack_elems<F>(pacc[th][2] + bs[2], pacc[th][3] + bs[3]);
                *reinterpret_cast<u32x2 *>(out + ((size_t)b * N + nt) * row_stride + 16 * h + 4 * g16) = w;
            }
        }
        kt = ktn;
        mx = mx_next;
    }
}

}  // namespace

bool mfma_project_supported(const flare_shape &s)
{
    return mfma_supported(s) && s.layout == FLARE_BNHD && s.d == 16 && s.M <= kLatChunk && !s.y_f32 &&
           (s.H == 2 || s.H == 4 || s.H == 8);
}

int mfma_decode_project(const flare_shape &s, const void *q, const void *k, const float *z, const void *w_out,
                        const float *bias, void *out, void *y, float *lse_dec, float scale, hipStream_t stream)
{
    if (!mfma_project_supported(s)) return FLARE_EUNSUPPORTED;
    const int tiles = (s.N + 31) / 32;
    int blocks = (256 + s.B - 1) / s.B;                       // one workgroup per compute unit
    if (blocks > tiles) blocks = tiles;
    const dim3 grid(blocks, s.B);
    const float c2 = scale * kLog2e;
    const long long sq = s.shared_latents ? 0 : (long long)s.M * s.d;
    const int MT = lat_eff(s.M) / 32;
    const bool f16 = s.dtype == FLARE_F16;
    LaunchTimer t(KID_DECODE_PROJECT, stream);
#define FLARE_PROJ_ARGS                                                                                          \
    (const bf16_t *)q, (const bf16_t *)k, z, (const bf16_t *)w_out, bias, (bf16_t *)out, (bf16_t *)y, lse_dec, sq, \
        s.N, s.M, c2
#define FLARE_PROJ(MTT, HWW)                                                                        \
    do {                                                                                            \
        if (f16) decode_project_kernel<MTT, HWW, true><<<grid, 64 * HWW, 0, stream>>>(FLARE_PROJ_ARGS);   \
        else decode_project_kernel<MTT, HWW, false><<<grid, 64 * HWW, 0, stream>>>(FLARE_PROJ_ARGS);      \
    } while (0)
#define FLARE_PROJ_H(MTT)                       \
    switch (s.H) {                              \
        case 2: FLARE_PROJ(MTT, 2); break;      \
        case 4: FLARE_PROJ(MTT, 4); break;      \
        default: FLARE_PROJ(MTT, 8); break;     \
    }
    switch (MT) {
        case 1: FLARE_PROJ_H(1) break;
        case 2: FLARE_PROJ_H(2) break;
        case 4: FLARE_PROJ_H(4) break;
        case 6: FLARE_PROJ_H(6) break;
        case 8: FLARE_PROJ_H(8) break;
        default: return FLARE_EUNSUPPORTED;
    }
#undef FLARE_PROJ_H
#undef FLARE_PROJ
#undef FLARE_PROJ_ARGS
    return check_launch();
}

}  // namespace flare
