// Matrix-core kernels of the forward (encode, decode), of the first backward pass (dZ partials, token
// statistics: the same two kernels in their MODE 1) and of the spectral analysis (companion matrix).
// Operand layouts, helpers and the tile geometry are in flare_mfma_common.h.
#include "flare_mfma_common.h"

namespace flare {
namespace {

// ============================================================================================
// Decode.  One wave owns 32 tokens at a time and all M latents.  One pass over the latent tiles:
//   the stabiliser b of a token is its largest score (hi terms only) among the FIRST 32 latents: a
//   real score, so b <= max_m S2 and the largest weight is at least 1; the other weights may exceed
//   1 by whatever the later latents' scores exceed b, which fp32 sums and bf16 weights (same
//   exponent range) absorb up to 2^64;
//   per latent tile: full scores minus b (-b is the C operand the score products of all latent
//   tiles start from: one 16-register splat per token tile), 2^x, pack, and
//   Y^T += Zaug^T . E with Zaug = [Z | 1].
//   Only when a token's denominator comes out above 2^64 (or not finite) the tile is done again
//   with the exact maximum over all latents (one more sweep of hi products first).
// Q (as A operand) and Z^T (as A operand, latents in the permuted order) live in registers
// for the whole kernel; K streams from HBM straight into the B-operand layout; no LDS.
// The MFMAs of latent tile t+1 are issued before the vector work on tile t.
// PRE = false (shapes whose operands would not fit otherwise): raw q, no lo term, and
// 2^(|c2| s - b) formed with one v_fma_f32 per score.
// ============================================================================================
// MODE 0 writes y and, when lse_dec2 is not NULL, log sum_m exp(S[m][n]) (natural log) there.
// MODE 1 (first step of the backward when nothing was saved) writes per token
//   lse_dec2[n] = log2 sum_m 2^S2[m][n]   and   delta[n] = <dY_n, Y_n>   (Y_n kept in fp32).
template <int DR, int MT, bool PRE, int MINB, int MODE, bool F>
__global__ __launch_bounds__(256, MINB) void decode_mfma_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const float *__restrict__ z,
    bf16_t *__restrict__ y, const bf16_t *__restrict__ dy, float *__restrict__ lse_dec2,
    float *__restrict__ delta, TokStride ts, TokStride ts_y, int H, int N, int Mtot, int m0, float c2, int flags)
{
    // flags: bit 0 (d <= 8): Z enters the value product as a hi + lo pair (see the Zaug operand below);
    // bit 1 (MODE 0): y is an fp32 tensor of the same layout (flare_shape.y_f32)
    const bool z_lo = (flags & 1) != 0, y32 = (flags & 2) != 0;
    // The kernel works on the latents m0 .. m0 + M of the head's Mtot (M = 32*MT of them); with more than
    // one chunk its outputs are one chunk's partial result (y normalised within the chunk, lse_dec of the
    // chunk) that decode_merge_kernel combines.  ts_y: where the rows of y go.
    // Latents at or beyond Mtot are padding and cost no mask code in the loops: a padding latent gets the
    // queries of the last real one (the clamped load), so its score never exceeds the real maximum and
    // its weight is at most 1, and its row of Zaug -- the Z values and the 1 that feeds the denominator --
    // is zero, so that weight multiplies zeros only.
    constexpr int D = padded_dim(DR);
    constexpr int KS = D / 16;   // k-steps of the score product
    constexpr int HV = D / 16;   // 16-wide column groups of Z, each with its own ones row
    constexpr bool PACK = PRE && pack_dim(DR);   // q' hi | lo in one operand, keys repeated in both lane halves
    const int lane = threadIdx.x & 63, l32 = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // known to be wave-uniform: scalar unit
    const GridPos gp = grid_pos(ts, H, DR * 2);
    const int bh = gp.y, h = bh % H;
    const bool flip = c2 < 0.f;
    const float ac2 = PRE ? c2 : fabsf(c2);

    bf16x8 qh[MT][KS], ql[MT][KS];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int m = m0 + 32 * t + l32;
        load_q_operand<DR, PRE, F, PACK>(q + (size_t)h * ts.sq + (size_t)min(m, Mtot - 1) * DR, hh, c2, flip, qh[t],
                                         ql[t]);
    }
    const int mleft = Mtot - m0;   // real latents from m0 on (may exceed the 32*MT this kernel covers)

    // Zaug^T operand: row l32 (< 16: column 16*hv + l32 of Z; 16: ones; else zero).  In registers, or --
    // for the shapes whose registers would not allow two waves per SIMD otherwise (ZLDS = !PRE) --
    // built once per workgroup in LDS (the four waves share one (b,h)) and read per latent tile.
    constexpr bool ZLDS = !PRE;
    __shared__ __attribute__((aligned(16))) u32x4 zlds[ZLDS ? HV * 2 * MT * 64 : 1];
    bf16x8 zt[ZLDS ? 1 : HV][ZLDS ? 1 : 2 * MT];
    {
        const float *zb = z + ((size_t)bh * Mtot + m0) * DR;
#pragma unroll
        for (int hv = 0; hv < HV; ++hv)
#pragma unroll
            for (int s = 0; s < 2 * MT; ++s) {
                if (ZLDS && (s & 3) != wave) continue;   // each wave builds a quarter of the images
                u32x4 w;
#pragma unroll
                for (int i = 0; i < 8; i += 2) {
                    float a, b;
                    if (l32 < 16 && 16 * hv + l32 < DR) {
                        const int la = 32 * (s / 2) + perm_index(s % 2, hh, i);
                        const int lb = 32 * (s / 2) + perm_index(s % 2, hh, i + 1);
                        a = la < mleft ? zb[(size_t)la * DR + 16 * hv + l32] : 0.f;
                        b = lb < mleft ? zb[(size_t)lb * DR + 16 * hv + l32] : 0.f;
                    } else if (DR <= 8 && z_lo && l32 >= 8 && l32 < 8 + DR) {
                        // rows 8 .. 8 + d - 1 (free at d <= 8): what the rounding of Z to bf16 left over, so
                        // that the rows of Y behind delta carry Z as a hi + lo pair like the c chain does
                        const int la = 32 * (s / 2) + perm_index(s % 2, hh, i);
                        const int lb = 32 * (s / 2) + perm_index(s % 2, hh, i + 1);
                        a = la < mleft ? zb[(size_t)la * DR + l32 - 8] : 0.f;
                        b = lb < mleft ? zb[(size_t)lb * DR + l32 - 8] : 0.f;
                        a -= __uint_as_float(rne_bf16(a) << 16);
                        b -= __uint_as_float(rne_bf16(b) << 16);
                    } else {   // row 16: ones (for the real latents), the rest: zero
                        a = (l32 == 16 && 32 * (s / 2) + perm_index(s % 2, hh, i) < mleft) ? 1.f : 0.f;
                        b = (l32 == 16 && 32 * (s / 2) + perm_index(s % 2, hh, i + 1) < mleft) ? 1.f : 0.f;
                    }
                    w[i / 2] = rne_bf16(a) | (rne_bf16(b) << 16);
                }
                if constexpr (ZLDS) zlds[(hv * 2 * MT + s) * 64 + lane] = w;
                else zt[hv][s] = as_bf16x8(w);
            }
    }
    if constexpr (ZLDS) __syncthreads();
    auto z_op = [&](int hv, int s) {
        if constexpr (ZLDS) return as_bf16x8(zlds[(hv * 2 * MT + s) * 64 + lane]);
        else return zt[hv][s];
    };

    const bf16_t *kb = k + tok_base(ts, bh, H);
    bf16_t *yb = y + tok_base(ts_y, bh, H);
    const int tiles = (N + 31) / 32;
    const int stride = gridDim.x * 4;
    int tile = gp.x * 4 + wave;
    bf16x8 kt[KS], ktn[KS];
    // hi part of the scores of latent tile t against the keys kk, without a stabiliser
    auto qk_hi = [&](int t, const bf16x8 (&kk)[KS]) {
        f32x16 r = splat16(0.f);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) r = mfma_s<F>(qh[t][ks], kk[ks], r);
        return r;
    };
    // The stabiliser of a token tile is the maximum of the hi product of its FIRST latent tile (any value is exact
    // as long as no weight overflows and the largest does not underflow; this one is <= the true maximum).  The
    // scores of that latent tile are the same product minus the stabiliser, plus the lo product.
    auto tile_max = [&](const f32x16 &hi) {
        const float m = max16(hi, -INFINITY);
        return fmaxf(m, __shfl_xor(m, 32));
    };
    auto first_scores = [&](f32x16 hi, float m, const bf16x8 (&kk)[KS]) {
        if constexpr (PRE) {
#pragma unroll
            for (int i = 0; i < 16; ++i) hi[i] -= m;
            if constexpr (!PACK) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) hi = mfma_s<F>(ql[0][ks], kk[ks], hi);
            }
        }
        return hi;
    };
    // carried from one token tile of the wave to its next: the keys, the stabiliser, the scores of latent tile 0
    float mx = 0.f;
    f32x16 s_cur0 = splat16(0.f);
    if (tile < tiles) {
        const int nld = min(tile * 32 + l32, N - 1);
#pragma unroll
        for (int s = 0; s < KS; ++s)
            kt[s] = as_bf16x8(row8_bf16<DR>(kb + tok_off(ts, nld), PACK ? 0 : (D / 2) * hh + 8 * s));
        const f32x16 hi = qk_hi(0, kt);
        mx = tile_max(hi);
        s_cur0 = first_scores(hi, mx, kt);
    }
    for (; tile < tiles; tile += stride) {
        const int n = tile * 32 + l32;
        {   // prefetch the keys of this wave's next tile (the last tile is simply loaded again)
            const int tn = (tile + stride < tiles) ? tile + stride : tile;
            const int nld = min(tn * 32 + l32, N - 1);
#pragma unroll
            for (int s = 0; s < KS; ++s)
                ktn[s] = as_bf16x8(row8_bf16<DR>(kb + tok_off(ts, nld), PACK ? 0 : (D / 2) * hh + 8 * s));
        }
        // MODE 1: this lane's quartets of the tile's dY rows, used after the sweep (for delta).  Requested here, a
        // whole tile before their use -- except at d = 32, where their eight registers would cost the kernel its
        // third wave per SIMD: there they are requested where they are used.
        constexpr bool EARLY_G = D <= 16;
        u32x2 gq[MODE == 1 ? HV : 1][2];
        auto request_g = [&]() {
            const bf16_t *gr = dy + tok_base(ts, bh, H) + tok_off(ts, min(n, N - 1));
#pragma unroll
            for (int hv = 0; hv < HV; ++hv) {
                gq[hv][0] = u32x2{0u, 0u};
                gq[hv][1] = u32x2{0u, 0u};
                if (quartet_inside<DR>(hv, hh, 0)) gq[hv][0] = *reinterpret_cast<const u32x2 *>(gr + 16 * hv + 4 * hh);
                if (quartet_inside<DR>(hv, hh, 1)) gq[hv][1] = *reinterpret_cast<const u32x2 *>(gr + 16 * hv + 8 + 4 * hh);
            }
        };
        if constexpr (MODE == 1 && EARLY_G) request_g();
        // An opaque copy of the keys for the hi products, so that the compiler keeps them apart from the lo ones.
        bf16x8 kt2[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 w = __builtin_bit_cast(u32x4, kt[ks]);
            asm volatile("" : "+v"(w));
            kt2[ks] = as_bf16x8(w);
        }
        f32x16 acc[HV];
        f32x16 s_ahead = splat16(0.f);   // hi product of the NEXT token tile's first latent tile
        float b2 = mx * ac2;
        // One sweep over the latent tiles: 2^x, pack, value product per tile.  s_cur: the scores of latent tile 0;
        // cinit: -b as the starting value of the other tiles' score accumulators (PRE), or folded into the fma.
        // AHEAD: the last latent tile, which has no next scores to request, requests the first hi product of
        // the wave's next token tile instead, so that its stabiliser is known when this tile's output is stored.
        auto sweep = [&](f32x16 s_cur, const f32x16 cinit, auto ahead_tag) {
            constexpr bool AHEAD = decltype(ahead_tag)::value;
            auto qk_full = [&](int t) {
                f32x16 r = cinit;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) r = mfma_s<F>(qh[t][ks], kt2[ks], r);
                if constexpr (PRE && !PACK) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) r = mfma_s<F>(ql[t][ks], kt[ks], r);
                }
                return r;
            };
            f32x16 s_next = s_cur;
#pragma unroll
            for (int hv = 0; hv < HV; ++hv) acc[hv] = splat16(0.f);
            sched_fence();
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                // SPLIT (d = 16, q' as a hi + lo pair): the two dependent score products of tile t+1 and the two
                // dependent value products of tile t alternate (hi, value, lo, value), so that each finds its
                // predecessor's result ready instead of waiting for the matrix pipe to drain
                constexpr bool SPLIT = PRE && D == 16 && !PACK;
                if (t + 1 < MT) {
                    if constexpr (SPLIT) s_next = mfma_s<F>(qh[t + 1][0], kt2[0], cinit);
                    else s_next = qk_full(t + 1);
                } else if constexpr (AHEAD) {
                    s_next = qk_hi(0, ktn);
                }
                // d = 32 with the stabiliser as C operand: groups for the tile's 8 products (-1.3 % of the forward at
                // 4096 tokens and 128 latents; the variant with Z in LDS and 6 products a tile lost 1 % with its groups)
                constexpr bool GROUPS32 = D == 32 && !PACK && PRE;
                if constexpr (!(PRE && D == 16) && !GROUPS32) sched_fence();
                if constexpr (!PRE) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) s_cur[i] = fmaf(s_cur[i], ac2, -b2);
                }
                bf16x8 p0, p1;
                exp_pack(s_cur, p0, p1);
                if constexpr (SPLIT) {
                    acc[0] = mfma(z_op(0, 2 * t), p0, acc[0]);
                    if (t + 1 < MT) s_next = mfma_s<F>(ql[t + 1][0], kt[0], s_next);
                    acc[0] = mfma(z_op(0, 2 * t + 1), p1, acc[0]);
                } else {
#pragma unroll
                    for (int hv = 0; hv < HV; ++hv) {
                        acc[hv] = mfma(z_op(hv, 2 * t), p0, acc[hv]);
                        acc[hv] = mfma(z_op(hv, 2 * t + 1), p1, acc[hv]);
                    }
                }
                if constexpr (PRE && D == 16) {
                    // order within the tile: the two score products of tile t+1 (one when q' is packed) and the
                    // two value products of tile t, each followed by a share of the 16 exponentials and 8 packs
                    // of tile t
                    if (PACK && t + 1 < MT) {
                        FLARE_GROUP_TRANS(4);
                        FLARE_GROUP_MFMA(1);
                        FLARE_GROUP_TRANS(4);
                        FLARE_GROUP_VALU(4);
                        FLARE_GROUP_MFMA(1);
                        FLARE_GROUP_TRANS(8);
                        FLARE_GROUP_VALU(4);
                        FLARE_GROUP_MFMA(1);
                    } else if (t + 1 < MT) {
                        FLARE_GROUP_TRANS(4);
                        FLARE_GROUP_MFMA(1);      // hi product of the next scores
                        FLARE_GROUP_TRANS(4);
                        FLARE_GROUP_VALU(4);
                        FLARE_GROUP_MFMA(1);      // first value product
                        FLARE_GROUP_TRANS(4);
                        FLARE_GROUP_MFMA(1);      // lo product
                        FLARE_GROUP_TRANS(4);
                        FLARE_GROUP_VALU(4);
                        FLARE_GROUP_MFMA(1);      // second value product
                    } else if (AHEAD) {
                        FLARE_GROUP_TRANS(4);
                        FLARE_GROUP_MFMA(1);      // hi product of the next token tile
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
                }
                if constexpr (GROUPS32) {
                    // score products of the next tile (KS hi k-steps, and KS lo ones when q' is a pair), then the four
                    // value products, each group followed by a share of the tile's vector work
                    constexpr int NS = (PRE ? 2 : 1) * KS;
                    if (t + 1 < MT || AHEAD) {
                        const int ns = (t + 1 < MT) ? NS : KS;
#pragma unroll
                        for (int i = 0; i < NS; ++i) {
                            if (i < ns) {
                                FLARE_GROUP_MFMA(1);
                                if constexpr (!PRE) FLARE_GROUP_VALU(4);
                                FLARE_GROUP_TRANS(NS == 4 ? 2 : 4);
                            }
                        }
                        if (ns < NS) FLARE_GROUP_TRANS(4);
                    } else {
                        if constexpr (!PRE) FLARE_GROUP_VALU(8);
                        FLARE_GROUP_TRANS(8);
                    }
                    FLARE_GROUP_VALU(PRE ? 4 : 12);   // (the rest of the scaling,) the first four packs
                    FLARE_GROUP_MFMA(1);
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_MFMA(1);
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_VALU(4);
                    FLARE_GROUP_MFMA(1);
                    FLARE_GROUP_MFMA(1);
                }
                sched_fence();
                s_cur = s_next;
            }
            return s_cur;
        };
        s_ahead = sweep(s_cur0, splat16(PRE ? -mx : 0.f), PlainTag<true>{});
        // A later latent tile beat the first one by more than 2^64 for some token (its denominator, row 16,
        // is huge or not finite): once more with the exact maximum.  Exponent field >= 127 + 64.
        if (__any((__float_as_uint(acc[0][8]) & 0x7f800000u) >= ((127u + 64u) << 23))) {
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
            b2 = mx * ac2;
            (void)sweep(first_scores(hi0, mx, kt), splat16(PRE ? -mx : 0.f), PlainTag<false>{});
            s_ahead = qk_hi(0, ktn);
        }
        // The next tile's stabiliser and first scores, before this tile's output: their latencies (a cross-lane
        // exchange, a matrix product) pass while the output below is normalised, packed and stored.
        const float mx_next = tile_max(s_ahead);
        s_cur0 = first_scores(s_ahead, mx_next, ktn);
        // row 16 (register 8 of the lower lane half) is the softmax denominator
        const float den = __shfl(acc[0][8], l32);
        const float inv = 1.f / den;
        if constexpr (MODE == 1) {
            const size_t row = (size_t)bh * N + min(n, N - 1);
            if constexpr (!EARLY_G) request_g();
            float part = 0.f;
#pragma unroll
            for (int hv = 0; hv < HV; ++hv) {
                const u32x2 g0 = gq[hv][0], g1 = gq[hv][1];
                if constexpr (DR <= 8) {   // rows 8 + j: the lo part of column j (zero unless z_lo), same lane
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[hv][i] += acc[hv][4 + i];
                }
                part = fmaf(acc[hv][0] * inv, dy_lo<F>(g0[0]), part);
                part = fmaf(acc[hv][1] * inv, dy_hi<F>(g0[0]), part);
                part = fmaf(acc[hv][2] * inv, dy_lo<F>(g0[1]), part);
                part = fmaf(acc[hv][3] * inv, dy_hi<F>(g0[1]), part);
                part = fmaf(acc[hv][4] * inv, dy_lo<F>(g1[0]), part);
                part = fmaf(acc[hv][5] * inv, dy_hi<F>(g1[0]), part);
                part = fmaf(acc[hv][6] * inv, dy_lo<F>(g1[1]), part);
                part = fmaf(acc[hv][7] * inv, dy_hi<F>(g1[1]), part);
            }
            part += __shfl_xor(part, 32);
            // the stabiliser that was actually subtracted
            const float used = PRE ? mx : b2;
            if (n < N && hh == 0) {
                lse_dec2[row] = used + log2f(den);
                delta[row] = part;
            }
        } else if (n < N) {
            if (lse_dec2 && hh == 0) {   // optional saved statistic of the forward, natural log
                const float used = PRE ? mx : b2;
                lse_dec2[(size_t)bh * N + n] = (used + log2f(den)) * kLn2;
            }
            if constexpr (DR <= 8) {   // rows 8 + j: the lo part of column j (zero unless z_lo), same lane
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[0][i] += acc[0][4 + i];
            }
            if (y32) {
                float *yf = reinterpret_cast<float *>(y) + tok_base(ts_y, bh, H) + tok_off(ts_y, n);
#pragma unroll
                for (int hv = 0; hv < HV; ++hv)
#pragma unroll
                    for (int up = 0; up < 2; ++up)
                        if (quartet_inside<DR>(hv, hh, up))
                            *reinterpret_cast<float4 *>(yf + 16 * hv + 8 * up + 4 * hh) =
                                make_float4(acc[hv][4 * up] * inv, acc[hv][4 * up + 1] * inv, acc[hv][4 * up + 2] * inv,
                                            acc[hv][4 * up + 3] * inv);
            } else
#pragma unroll
            for (int hv = 0; hv < HV; ++hv) {
                u32x2 w0, w1;
                w0[0] = pack_elems<F>(acc[hv][0] * inv, acc[hv][1] * inv);
                w0[1] = pack_elems<F>(acc[hv][2] * inv, acc[hv][3] * inv);
                w1[0] = pack_elems<F>(acc[hv][4] * inv, acc[hv][5] * inv);
                w1[1] = pack_elems<F>(acc[hv][6] * inv, acc[hv][7] * inv);
                if (quartet_inside<DR>(hv, hh, 0)) *reinterpret_cast<u32x2 *>(yb + tok_off(ts_y, n) + 16 * hv + 4 * hh) = w0;
                if (quartet_inside<DR>(hv, hh, 1))
                    *reinterpret_cast<u32x2 *>(yb + tok_off(ts_y, n) + 16 * hv + 8 + 4 * hh) = w1;
            }
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) kt[s] = ktn[s];
        mx = mx_next;
    }
}

// ============================================================================================
// Encode partials.  A workgroup has up to 4 waves; wave w works on latent group w % G (NB tiles
// of 32 latents) and on every TG-th 32-token tile of the chunk, starting at tile w / G.  Per tile
// and latent tile:
//   S2^T - c = K . Q'^T  (rows = tokens, columns = latents; -c rides in a k-step of its own:
//   key side 1 in slot 0, query side -c in slot 0, so that every lo term of q' stays in),
//   lazy online softmax: c moves only when a score exceeds it by more than kLazy (or on the
//   first tile), then O is rescaled; 2^x, pack; O^T += Vaug^T . P^T, Vaug = [V | 1].
// V^T is formed through a wave-private, double-buffered LDS tile (no workgroup barrier in the
// encode; the dZ kernel lines its waves up every 32 tiles): the values of tile j+1 are written
// while tile j is computed and read back at its end.  Keys and values are requested two tiles
// ahead; the value rows of consecutive tiles alternate between two sets of registers (a copy of
// a load in flight would be waited for in the tile that issued it).  The MFMAs of the next
// latent tile (or of the next token tile) are issued before the vector work on the current one.
// Output per wave: (c, row sums, unnormalised O) for its latents = one partial slot.
// ============================================================================================
// MODE 1 (second step of the backward) reuses the same machinery for dZ = R^T dY: the values are
// dY, the weights are R^T[n][m] = 2^(S2 - lse_dec2[n]) with the per-token -lse_dec2 as the value the score
// accumulators start from (exact in fp32; no k-step of its own), and there is no
// softmax state: only the unnormalised sums are written.  lse_dec2 is read as ld_mul * lse_dec2[n]
// (ld_mul = log2 e when the array holds the forward's natural-log statistic).  When y_tok is given,
// every wave also forms delta[n] = <dY_n, Y_n> from the rows it streams anyway (no branch in the
// loop), and the waves of latent group 0 store it to delta_out for the two kernels that follow.
// Those waves also record the smallest and largest lse_dec2 they met, ld_range[part] = (min, max),
// from which bwd_one_exp_ok decides which variant of the next two kernels may run.
template <int DR, int NB, int MINB, int MODE, bool F, bool Y32 = false>
__global__ __launch_bounds__(256, MINB) void encode_mfma_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const float *__restrict__ lse_dec2, float ld_mul, const bf16_t *__restrict__ y_tok,
    float *__restrict__ delta_out, float *__restrict__ ld_range,
    float *__restrict__ m_part, float *__restrict__ l_part, float *__restrict__ o_part,
    TokStride ts, int H, int N, int M, int chunk_len, int parts, int G, int TG, float c2)
{
    // Y32 (MODE 1, d <= 8 only): y_tok points to fp32 rows (flare_shape.y_f32) instead of rows of the storage type
    static_assert(!Y32 || (MODE == 1 && DR <= 8), "fp32 rows of y: written for the statistics of d <= 8");
    constexpr int D = padded_dim(DR);
    constexpr int KS = D / 16;
    // d = 32: the value operand's 32 rows are the 32 columns of V, so there is no free row for the ones that sum
    // the weights at d <= 16.  The encode's denominators then come from the vector ALU instead: one v_dot2c per
    // packed pair of weights adds the same rounded weights that enter the matrix product (eight instructions a
    // tile instead of the two extra matrix products of a second column group with its own ones row).
    constexpr bool WIDE = D == 32;
    constexpr bool ROWSUM = WIDE && MODE == 0;
    constexpr int HV = 1;
    // The value tile of a token tile lives in LDS as it is loaded, row = token: D columns of values, then a column
    // of ones (the softmax denominator's row of the operand), then 15 columns of zeros; 8 more pad the row to a
    // stride that keeps the 16-byte stores aligned.  The operand wants it transposed (row = column of V, eight
    // tokens per lane): that is what the transposing LDS read delivers.
    constexpr int RS = D + 16 + 8;              // uint16 per row
    // dZ kernel: -lse_dec2 of the tokens is what the score accumulators start from (no correction k-step)
    constexpr bool CINIT = MODE == 1;
    constexpr bool PACK = pack_dim(DR);         // q' hi | lo in one operand, keys repeated in both lane halves
    constexpr int BUF = 32 * RS;                // uint16 per buffer
    __shared__ __attribute__((aligned(16))) uint16_t vt_all[4][2 * BUF];

    const int lane = threadIdx.x & 63, l32 = lane & 31, hh = lane >> 5;
    // (read from the first lane: the compiler then knows it is the same for the whole wave and keeps everything derived
    // from it -- token groups, tile indices, loop bounds -- on the scalar unit)
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int g = wave % G, tg = wave / G;
    const GridPos gp = grid_pos(ts, H, DR * 2);
    const int bh = gp.y, h = bh % H, chunk = gp.x;
    const uint32_t keep0 = hh == 0 ? 0xffff0000u : 0xffffffffu;
    uint16_t *vt = vt_all[wave];

    // constant columns of the value tile, in both buffers: two lanes per row, eight columns each
    {
        u32x4 w;
        w[0] = (lane & 1) == 0 ? 0x3f80u : 0u; w[1] = 0u; w[2] = 0u; w[3] = 0u;
        uint16_t *c = vt + (lane >> 1) * RS + D + 8 * (lane & 1);
        *reinterpret_cast<u32x4 *>(c) = w;
        *reinterpret_cast<u32x4 *>(c + BUF) = w;
    }

    const int lat0 = 32 * NB * (G * (int)blockIdx.z + g);   // a workgroup owns NB*G tiles of latents
    bf16x8 qh[NB][KS], ql[NB][KS];
#pragma unroll
    for (int b = 0; b < NB; ++b) {   // padding latents (at or beyond M): zero queries, nothing stored
        const int m = lat0 + 32 * b + l32;
        load_q_operand<DR, true, F, PACK>(q + (size_t)h * ts.sq + (size_t)min(m, M - 1) * DR, hh, c2, false, qh[b],
                                          ql[b]);
        if (m >= M) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) { qh[b][ks] = zero_operand(); ql[b][ks] = zero_operand(); }
        }
    }
    u32x4 wzero;
    wzero[0] = 0u; wzero[1] = 0u; wzero[2] = 0u; wzero[3] = 0u;
    bf16x8 caug[MODE == 0 ? NB : 1];             // query side of the stabiliser k-step: slot 0 := -c
    caug[0] = as_bf16x8(wzero);

    const bf16_t *kb = k + tok_base(ts, bh, H);
    const bf16_t *vb = v + tok_base(ts, bh, H);
    const int n0 = chunk * chunk_len;
    const int n1 = min(N, n0 + chunk_len);
    const int tiles = (n1 - n0 + 31) / 32;
    const int cnt = (tiles > tg) ? (tiles - tg + TG - 1) / TG : 0;   // tiles of this wave

    float c[NB];
    float l[NB];                                   // ROWSUM: this lane's share of the denominators
    float nl_min = INFINITY, nl_max = -INFINITY;   // range of -lse_dec2 over this wave's tokens (MODE 1)
    f32x16 o[NB][HV];
#pragma unroll
    for (int b = 0; b < NB; ++b) {   // what a wave without tiles stores
        c[b] = 0.f;
        l[b] = 0.f;
#pragma unroll
        for (int hv = 0; hv < HV; ++hv) o[b][hv] = splat16(0.f);
    }

    // Transposing read of the value operand: this lane's chunk of the tile.  Lanes 16-31 and 48-63 supply rows
    // 16-31 of the operand (d <= 16: the ones, then zeros; d = 32: columns 16-31 of V); the others rows 0-15
    // (columns 0-15 of V).  Row within a group of four tokens: (lane % 16) / 4; the lane half takes tokens 4-7 of
    // every eight.
    const int tr_row = 4 * hh + (lane & 15) / 4;
    const bool tr_upper = (lane & 16) != 0;
    const int tr_piece = 4 * (lane & 3);

    // keys: A operand, row = token.  values: 32 tokens x D in 16-byte pieces, two lanes per token.
    constexpr int PIECES = D / 8;          // 16-byte pieces per token row
    constexpr int LOADS = PIECES / 2;      // pieces per lane (64 lanes cover 32 tokens x 2 pieces)
    const int vtok = lane >> 1;
    auto tile_tok0 = [&](int j) { return n0 + 32 * (tg + min(j, cnt - 1) * TG); };   // j-th tile of this wave
    auto load_k = [&](int j, bf16x8 (&kk)[KS]) {
        const int nk = min(tile_tok0(j) + l32, N - 1);
#pragma unroll
        for (int s = 0; s < KS; ++s)
            kk[s] = as_bf16x8(row8_bf16<DR>(kb + tok_off(ts, nk), PACK ? 0 : (D / 2) * hh + 8 * s));
    };
    auto load_v = [&](int j, u32x4 (&vv)[LOADS]) {
        const int nv = min(tile_tok0(j) + vtok, N - 1);
#pragma unroll
        for (int i = 0; i < LOADS; ++i)
            vv[i] = row8_bf16<DR>(vb + tok_off(ts, nv), 8 * ((lane & 1) * LOADS + i));
    };
    auto write_vt = [&](const u32x4 (&vv)[LOADS], uint16_t *buf) {   // as loaded: row = token, one 16-byte store a piece
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int d0 = 8 * ((lane & 1) * LOADS + i);
            // the value side of the second product is bf16
            *reinterpret_cast<u32x4 *>(buf + vtok * RS + d0) = to_bf16_row<F>(vv[i]);
        }
    };
    auto read_va = [&](const uint16_t *buf, bf16x8 (&va)[HV][2]) {
#pragma unroll
        for (int hv = 0; hv < HV; ++hv)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                // k-step s2 of the operand: tokens 16 s2 + 4 hh + (0..3) and + 8 of them, column = this lane's row
                const uint16_t *src = buf + (16 * s2 + tr_row) * RS + (tr_upper ? (WIDE ? 16 : D) : 16 * hv) + tr_piece;
                const u32x2 a = lds_read_tr16(src);
                const u32x2 b = lds_read_tr16(src + 8 * RS);
                u32x4 w;
                w[0] = a[0]; w[1] = a[1]; w[2] = b[0]; w[3] = b[1];
                va[hv][s2] = as_bf16x8(w);
            }
    };
    // scores minus the stabiliser of latent tile b against the token tile (kk; kk0a = key side of the correction k-step)
    // (plain: without the correction k-step -- the encode's sweep that needs no stabiliser)
    // c0: what the score accumulators start from -- zero, or (CINIT) minus lse_dec2 of the register's token, which
    // then needs no correction k-step
    auto qk = [&](int b, const bf16x8 (&kk)[KS], bf16x8 kk0a, bool plain, const f32x16 &c0) {
        f32x16 r = c0;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) r = mfma_s<F>(kk[ks], qh[b][ks], r);
        if constexpr (!PACK) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) r = mfma_s<F>(kk[ks], ql[b][ks], r);
        }
        if (!CINIT && !plain) r = mfma_s<F>(kk0a, caug[MODE == 0 ? b : 0], r);
        return r;
    };
    // The same in two parts (d = 16, q' as a hi + lo pair), for the tiles that spread their matrix instructions:
    // the correction k-step and the hi product first, the lo product on top of them later.
    auto qk_first = [&](int b, const bf16x8 (&kk)[KS], bf16x8 kk0a, bool plain, const f32x16 &c0) {
        f32x16 r = c0;
        if (!CINIT && !plain) r = mfma_s<F>(kk0a, caug[MODE == 0 ? b : 0], r);
        return mfma_s<F>(kk[0], qh[b][0], r);
    };
    auto qk_second = [&](int b, const bf16x8 (&kk)[KS], f32x16 r) { return mfma_s<F>(kk[0], ql[b][0], r); };
    // The same at d = 32 in four parts: part 0 the correction k-step (unless plain) and the hi product's k-step 0,
    // part 1 its k-step 1, parts 2 and 3 the lo product's k-steps.
    auto qk_part = [&](int b, const bf16x8 (&kk)[KS], bf16x8 kk0a, bool plain, int part, f32x16 r) {
        if (!CINIT && part == 0 && !plain) r = mfma_s<F>(kk0a, caug[MODE == 0 ? b : 0], r);
        return mfma_s<F>(kk[part % KS], part < 2 ? qh[b][part % KS] : ql[b][part % KS], r);
    };
    const uint32_t one0 = hh == 0 ? kOne<F> : 0u;
    const float *lb = (MODE == 1) ? lse_dec2 + (size_t)bh * N : nullptr;
    // Key operand of the encode's stabiliser k-step: slot 0 := 1, else zero.
    auto k_aug = [&](bf16x8 k0, float neg_lse) { return with_slot0(as_bf16x8(wzero), keep0, one0); };
    auto load_lse = [&](int j) {   // lse_dec2 (as stored) of this lane's token in the wave's j-th tile (MODE 1)
        if constexpr (MODE == 1) return lb[min(tile_tok0(j) + l32, N - 1)];
        else return 0.f;
    };
    // CINIT: the accumulators of a score tile start from -lse_dec2 (scaled) of their tokens: register r of a lane
    // holds token 8 (r / 4) + 4 hh + r % 4 of the tile.  Every lane has its own token's value (load_lse); the 32
    // values of a tile go through 128 bytes of wave-private LDS and come back as four 16-byte reads per lane.
    __shared__ __attribute__((aligned(16))) float ld_all[CINIT ? 4 : 1][32];
    float *ldw = ld_all[CINIT ? wave : 0];
    auto put_ld = [&](float neg_lse) {
        if constexpr (CINIT) {
            if (hh == 0) ldw[l32] = neg_lse;
        }
    };
    auto get_ld = [&](f32x16 &t) {
        if constexpr (CINIT) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4 x = *reinterpret_cast<const float4 *>(ldw + 4 * hh + 8 * i);
                t[4 * i] = x.x; t[4 * i + 1] = x.y; t[4 * i + 2] = x.z; t[4 * i + 3] = x.w;
            }
        }
    };
    // delta of the wave's j-th tile (j < cnt) from its dY and Y rows: two lanes per token
    const bool do_delta = (MODE == 1) && y_tok != nullptr && blockIdx.z == 0;
    const bf16_t *yb = (MODE == 1 && y_tok != nullptr) ? y_tok + tok_base(ts, bh, H) : vb;
    // fp32 rows of y (d <= 8: one 16-byte piece of dY per token, in the even lane of its pair): the even lane
    // takes columns 0-3, the odd lane columns 4-7 (d = 8), four floats each -- the same registers as a
    // 16-bit piece -- and the odd lane fetches its half of the dY piece from its neighbour
    auto load_y = [&](int j, u32x4 (&yy)[LOADS]) {
        const int nv = min(tile_tok0(j) + vtok, N - 1);
        if constexpr (Y32) {
            {
                const float *yf = reinterpret_cast<const float *>(y_tok) + tok_base(ts, bh, H) + tok_off(ts, nv);
                u32x4 w;
                w[0] = 0u; w[1] = 0u; w[2] = 0u; w[3] = 0u;
                if (DR == 8 || (lane & 1) == 0) w = *reinterpret_cast<const u32x4 *>(yf + 4 * (lane & 1));
                yy[0] = w;
                return;
            }
        }
#pragma unroll
        for (int i = 0; i < LOADS; ++i)
            yy[i] = row8_bf16<DR>(yb + tok_off(ts, nv), 8 * ((lane & 1) * LOADS + i));
    };
    auto put_delta = [&](int j, const u32x4 (&gv)[LOADS], const u32x4 (&yy)[LOADS]) {
        float part = 0.f;
        bool done = false;
        if constexpr (Y32) {
            {
                const uint32_t n2 = (uint32_t)__builtin_amdgcn_mov_dpp((int)gv[0][2], 0xB1, 0xf, 0xf, true);
                const uint32_t n3 = (uint32_t)__builtin_amdgcn_mov_dpp((int)gv[0][3], 0xB1, 0xf, 0xf, true);
                const uint32_t g0 = (lane & 1) ? n2 : gv[0][0], g1 = (lane & 1) ? n3 : gv[0][1];
                part = dy_lo<F>(g0) * __uint_as_float(yy[0][0]);
                part = fmaf(dy_hi<F>(g0), __uint_as_float(yy[0][1]), part);
                part = fmaf(dy_lo<F>(g1), __uint_as_float(yy[0][2]), part);
                part = fmaf(dy_hi<F>(g1), __uint_as_float(yy[0][3]), part);
                done = true;
            }
        }
        if constexpr (!F && !Y32) {   // bf16 rows on both sides: one dot instruction per pair of elements
#pragma unroll
            for (int i = 0; i < LOADS; ++i) part = dot8_bf16(gv[i], yy[i], part);
            done = true;
        }
        if (!done) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                part = fmaf(dy_lo<F>(gv[i][e]), elem_lo<F>(yy[i][e]), part);
                part = fmaf(dy_hi<F>(gv[i][e]), elem_hi<F>(yy[i][e]), part);
            }
        }
        // the other half of the row is in the neighbouring lane: quad_perm [1,0,3,2]
        part += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(part), 0xB1, 0xf, 0xf, true));
        const int n = n0 + 32 * (tg + j * TG) + vtok;
        if (do_delta && j < cnt && g == 0 && (lane & 1) == 0 && n < n1) delta_out[(size_t)bh * N + n] = part;
    };

    // The waves of a workgroup that share token tiles (one per latent group) read the same rows; nothing else keeps
    // them together, and once they are more tiles apart than the L2 holds, the later one fetches its rows a second
    // time.  The dZ kernel therefore lines its waves up every kSyncTiles tiles (a wave passes the same number of
    // barriers whatever its number of tiles: those its sweep does not reach follow after it).
    constexpr bool SYNC = MODE == 1;
    constexpr int kSyncTiles = 32;
    // One sweep over this wave's token tiles.  PLAIN (encode only): the weights are 2^S2 as they come, with no
    // stabiliser (c = 0: no running maximum, no correction k-step, no rescaling) -- right whenever the row sums
    // end up in a range that shows that nothing overflowed and nothing that matters was flushed to zero, which
    // the caller checks afterwards; otherwise the same tiles are swept again with the lazy online softmax.
    auto sweep = [&](auto plain_tag) {
        constexpr bool PLAIN = decltype(plain_tag)::value;
        static_assert(!PLAIN || MODE == 0, "only the encode has a softmax state to leave out");
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            c[b] = 0.f;
            l[b] = 0.f;
#pragma unroll
            for (int hv = 0; hv < HV; ++hv) o[b][hv] = splat16(0.f);
            if constexpr (MODE == 0) caug[b] = as_bf16x8(wzero);
        }
        // keys: requested two token tiles ahead (ktf), like the values: the next tile's keys are needed before the
        // current tile ends (by the first score product of the next one), a request made at the top of the same
        // tile would have three quarters of a tile, or half of one at d = 32, to arrive
        bf16x8 kt[KS], ktn[KS], ktf[KS], va[HV][2];
        u32x4 vr1[LOADS], vr2[LOADS], yr1[LOADS], yr2[LOADS];
        f32x16 S[NB];
        bool first = true;

        // prologue: tile 0 fully staged, tile 1's values in flight
        // -lse_dec2 of the current tile's token and of the next tile's; the values are requested two tiles ahead
        // (la, lb2 alternate like the row registers), so that nothing waits for a request of the same tile
        float nl = -load_lse(0) * ld_mul, nln = 0.f;
        float la = load_lse(1), lb2 = 0.f;
        load_k(0, kt);
        load_k(1, ktn);
        load_v(0, vr1);
        if (do_delta) {
            load_y(0, yr1);
            put_delta(0, vr1, yr1);
            load_y(1, yr1);
        }
        compiler_fence();
        write_vt(vr1, vt);
        compiler_fence();
        read_va(vt, va);
        load_v(1, vr1);
#pragma unroll
        for (int b = 0; b < NB; ++b) S[b] = splat16(0.f);
        // MODE 1: the score accumulators' starting values of the current and of the next token tile; the tiles
        // alternate between the two (no copy at the end of a tile)
        f32x16 c_a = splat16(0.f), c_b = splat16(0.f);
        put_ld(nl);
        compiler_fence();
        get_ld(c_a);
        S[0] = qk(0, kt, k_aug(kt[0], nl), PLAIN, c_a);

        // One token tile.  TAIL: the wave's last tile, the only one that can reach past the chunk's end (its rows
        // beyond n1 are masked); the tiles before it carry no mask code, so that their matrix and vector
        // instructions form one scheduling region.
        // vn, yn: the rows of token tile j+1 (requested a tile ago); vf, yf: receive those of tile j+2.  Consecutive
        // tiles swap the two sets, so that no register of a load in flight is ever copied (a copy would make the
        // wave wait for the load in the tile that issued it).
        auto tile = [&](int j, auto tail_tag, const f32x16 &c_cur, f32x16 &c_nxt, u32x4 (&vn)[LOADS],
                        u32x4 (&vf)[LOADS], u32x4 (&yn)[LOADS], u32x4 (&yf)[LOADS], const float &ln, float &lf) {
            constexpr bool TAIL = decltype(tail_tag)::value;
            // SPREAD: the score products of the next latent tile and the value products of this one are issued
            // between the exponentials and packs of this tile instead of in one burst before and after them
            constexpr bool SPREAD = !TAIL && D == 16 && !PACK && (PLAIN || MODE == 1);
            // the same at d = 32 (two k-steps per score product, two column groups of values: eight products a tile),
            // in the dZ kernel only: there it gains 3 % (192 -> 186 us at 262144 tokens), the encode loses 1 % with it
            constexpr bool SPREAD32 = !TAIL && D == 32 && MODE == 1;
            const int tok0 = tile_tok0(j);
            uint16_t *buf_next = vt + ((j + 1) & 1) * BUF;
            lf = load_lse(j + 2);
            nln = -ln * ld_mul;
            load_k(j + 2, ktf);
            load_v(j + 2, vf);
            if constexpr (MODE == 1) {
                // (when y_tok is NULL, yb aliases the dY rows: the loads stay in bounds, nothing is stored)
                load_y(j + 2, yf);
                put_delta(j + 1, vn, yn);     // rows of tile j+1 (nothing stored past the last tile)
            }
            compiler_fence();
            write_vt(vn, buf_next);           // values of tile j+1
            compiler_fence();
            const bf16x8 kt0a = k_aug(kt[0], nl);

            // register r of this lane holds token tok0 + 8*(r/4) + 4*hh + r%4: valid iff 8*(r/4) + r%4 < rem
            const int rem = n1 - tok0 - 4 * hh;
            const bool partial = TAIL && tok0 + 32 > n1;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                // issue the next score product first: the next latent tile, or tile 0 of the next tokens
                f32x16 nxt;
                if constexpr (CINIT) {
                    // the next tile's values (requested two tiles ago) go into LDS at the top of the tile and are
                    // read back one latent tile before the next tile's first score product starts from them
                    if (b == 0) put_ld(nln);
                    if (b == (NB >= 2 ? NB - 2 : 0)) {
                        compiler_fence();
                        get_ld(c_nxt);
                    }
                }
                if constexpr (SPREAD) {
                    if (b + 1 < NB) nxt = qk_first(b + 1, kt, kt0a, PLAIN, c_cur);
                    else nxt = qk_first(0, ktn, k_aug(ktn[0], nln), PLAIN, c_nxt);
                } else if constexpr (SPREAD32) {
                    if (b + 1 < NB) nxt = qk_part(b + 1, kt, kt0a, PLAIN, 0, c_cur);
                    else nxt = qk_part(0, ktn, k_aug(ktn[0], nln), PLAIN, 0, c_nxt);
                } else {
                    if (b + 1 < NB) nxt = qk(b + 1, kt, kt0a, PLAIN, c_cur);
                    else nxt = qk(0, ktn, k_aug(ktn[0], nln), PLAIN, c_nxt);
                    sched_fence();
                }
                f32x16 sc = S[b];
                if (partial) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (8 * (r / 4) + (r % 4) >= rem) sc[r] = -INFINITY;
                }
                float mx = (MODE == 0 && !PLAIN) ? max16(sc, -INFINITY) : 0.f;
                if (MODE == 0 && !PLAIN && (first || __any(mx > kLazy))) {
                    mx = fmaxf(mx, __shfl_xor(mx, 32));   // both lane halves hold tokens of the same latent
                    const float cn = elem_round<F>(c[b] + (first ? mx : fmaxf(mx, 0.f)));
                    const float shift = cn - c[b];
                    if (!first) {
                        const float f = fast_exp2(-shift);
#pragma unroll
                        for (int hv = 0; hv < HV; ++hv)
#pragma unroll
                            for (int i = 0; i < 16; ++i) o[b][hv][i] *= f;
                        l[b] *= f;
                    }
                    c[b] = cn;
                    caug[b] = with_slot0(caug[b], keep0, hh == 0 ? rne_elem<F>(-cn) : 0u);
#pragma unroll
                    for (int i = 0; i < 16; ++i) sc[i] -= shift;
                    if constexpr (NB == 1) {   // the product already in flight is for this same latent tile
#pragma unroll
                        for (int i = 0; i < 16; ++i) nxt[i] -= shift;
                    }
                }
                bf16x8 p0, p1;
                if constexpr (ROWSUM) exp_pack_sum(sc, p0, p1, l[b]);
                else exp_pack(sc, p0, p1);
                if constexpr (SPREAD) {
                    // dependent pairs alternate (hi, value, lo, value): each finds its predecessor's result ready
                    o[b][0] = mfma(va[0][0], p0, o[b][0]);
                    if (b + 1 < NB) nxt = qk_second(b + 1, kt, nxt);
                    else nxt = qk_second(0, ktn, nxt);
                    o[b][0] = mfma(va[0][1], p1, o[b][0]);
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_MFMA(1);      // hi product of the next scores
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_VALU(4);
                    FLARE_GROUP_MFMA(1);      // first value product
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_MFMA(1);      // lo product
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_VALU(4);
                    FLARE_GROUP_MFMA(1);      // second value product
                } else if constexpr (SPREAD32) {
                    // six products, each dependent pair apart: (hi k-step 0 above), hi k-step 1, value (p0),
                    // lo k-step 0, lo k-step 1, value (p1)
                    nxt = (b + 1 < NB) ? qk_part(b + 1, kt, kt0a, PLAIN, 1, nxt) : qk_part(0, ktn, kt0a, PLAIN, 1, nxt);
                    o[b][0] = mfma(va[0][0], p0, o[b][0]);
                    nxt = (b + 1 < NB) ? qk_part(b + 1, kt, kt0a, PLAIN, 2, nxt) : qk_part(0, ktn, kt0a, PLAIN, 2, nxt);
                    nxt = (b + 1 < NB) ? qk_part(b + 1, kt, kt0a, PLAIN, 3, nxt) : qk_part(0, ktn, kt0a, PLAIN, 3, nxt);
                    o[b][0] = mfma(va[0][1], p1, o[b][0]);
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_MFMA(1);      // hi, k-step 0
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_VALU(4);
                    FLARE_GROUP_MFMA(1);      // hi, k-step 1
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_MFMA(1);      // value (p0)
                    FLARE_GROUP_TRANS(4);
                    FLARE_GROUP_VALU(4);
                    FLARE_GROUP_MFMA(1);      // lo, k-step 0
                    FLARE_GROUP_MFMA(1);      // lo, k-step 1
                    FLARE_GROUP_MFMA(1);      // value (p1)
                } else {
#pragma unroll
                    for (int hv = 0; hv < HV; ++hv) {
                        o[b][hv] = mfma(va[hv][0], p0, o[b][hv]);
                        o[b][hv] = mfma(va[hv][1], p1, o[b][hv]);
                    }
                }
                sched_fence();
                S[(b + 1) % NB] = nxt;
            }
            first = false;
            if constexpr (MODE == 1) { nl_min = fminf(nl_min, nl); nl_max = fmaxf(nl_max, nl); }
            nl = nln;
            compiler_fence();
            read_va(buf_next, va);            // value operand of tile j+1 (written at the top of this iteration)
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                kt[s] = ktn[s];
                ktn[s] = ktf[s];
            }
        };
        int j = 0;
        for (; j + 2 < cnt; j += 2) {
            if (SYNC && j > 0 && (j & (kSyncTiles - 1)) == 0) __syncthreads();
            tile(j, PlainTag<false>{}, c_a, c_b, vr1, vr2, yr1, yr2, la, lb2);
            tile(j + 1, PlainTag<false>{}, c_b, c_a, vr2, vr1, yr2, yr1, lb2, la);
        }
        if (j + 1 < cnt) {
            tile(j, PlainTag<false>{}, c_a, c_b, vr1, vr2, yr1, yr2, la, lb2);
            tile(j + 1, PlainTag<true>{}, c_b, c_a, vr2, vr1, yr2, yr1, lb2, la);
        } else {
            tile(j, PlainTag<true>{}, c_a, c_b, vr1, vr2, yr1, yr2, la, lb2);
        }
    };
    if constexpr (SYNC) {
        // the barriers this wave's sweep does not reach (it has one tile fewer than the longest, or none at all)
        const int cnt_max = (tiles + TG - 1) / TG;
        const int mine = cnt >= 3 ? (cnt - 3) / kSyncTiles : 0, all = cnt_max >= 3 ? (cnt_max - 3) / kSyncTiles : 0;
        if (cnt > 0) sweep(PlainTag<false>{});
        for (int i = mine; i < all; ++i) __syncthreads();
    } else if (cnt > 0) {
        if constexpr (MODE == 0) {
            sweep(PlainTag<true>{});
            // Row sums (register 8 of the lower lane half) between 2^-80 and 2^100: no weight overflowed, and the
            // largest score of the latent in this slot is above -94, so whatever was flushed to zero is below
            // 2^-32 of it.  Anything else (also NaN, inf): the slot is swept again with a stabiliser.
            bool redo = false;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float den = ROWSUM ? l[b] + __shfl_xor(l[b], 32) : o[b][0][8];
                const uint32_t e = (__float_as_uint(den) >> 23) & 0xffu;
                redo |= hh == 0 && lat0 + 32 * b + l32 < M && (e < 127u - 80u || e > 127u + 100u);
            }
            if (__any(redo)) sweep(PlainTag<false>{});
        } else {
            sweep(PlainTag<false>{});
        }
    }

    if constexpr (ROWSUM) {   // the two lane halves hold the sums over different tokens of the same latent
#pragma unroll
        for (int b = 0; b < NB; ++b) l[b] += __shfl_xor(l[b], 32);
    }
    // partial slot of this wave: (bh, chunk*TG + tg), latents lat0 .. lat0 + 32*NB
    if (tg >= TG) return;
    const size_t part = (size_t)bh * parts + (size_t)chunk * TG + tg;
    if (MODE == 1 && ld_range != nullptr && g == 0 && blockIdx.z == 0) {
#pragma unroll
        for (int off = 1; off < 32; off <<= 1) {   // both lane halves hold the same tokens
            nl_min = fminf(nl_min, __shfl_xor(nl_min, off));
            nl_max = fmaxf(nl_max, __shfl_xor(nl_max, off));
        }
        if (lane == 0) {   // a wave without tiles leaves (+inf, -inf): neutral
            ld_range[2 * part] = -nl_max;
            ld_range[2 * part + 1] = -nl_min;
        }
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (lat0 + 32 * b + l32 >= M) continue;
        const size_t slot = part * M + lat0 + 32 * b + l32;
        if (MODE == 0 && hh == 0) {
            m_part[slot] = (cnt > 0) ? c[b] : -INFINITY;
            l_part[slot] = ROWSUM ? l[b] : o[b][0][8];
        }
#pragma unroll
        for (int hv = 0; hv < HV; ++hv) {
            float4 lo4 = make_float4(o[b][hv][0], o[b][hv][1], o[b][hv][2], o[b][hv][3]);
            float4 hi4 = make_float4(o[b][hv][4], o[b][hv][5], o[b][hv][6], o[b][hv][7]);
            if (quartet_inside<DR>(hv, hh, 0)) *reinterpret_cast<float4 *>(o_part + slot * DR + 16 * hv + 4 * hh) = lo4;
            if (quartet_inside<DR>(hv, hh, 1)) *reinterpret_cast<float4 *>(o_part + slot * DR + 16 * hv + 8 + 4 * hh) = hi4;
            if constexpr (WIDE) {   // registers 8-15: columns 16-31 of the same layout
                float *dst = o_part + slot * DR + 16 + 4 * hh;
                *reinterpret_cast<float4 *>(dst) = make_float4(o[b][0][8], o[b][0][9], o[b][0][10], o[b][0][11]);
                *reinterpret_cast<float4 *>(dst + 8) = make_float4(o[b][0][12], o[b][0][13], o[b][0][14], o[b][0][15]);
            }
        }
    }
}

// ============================================================================================
// Companion matrix of the spectral analysis (Appendix C.1, Algorithm 1, steps 1-4 and the product of
// step 5):   G = J J^T,   J[m][n] = exp(S[m][n] - (lse_enc[m] + lse_dec[n]) / 2) = (P[m][n] R[n][m])^(1/2).
// A workgroup has one wave per 32-latent tile and walks over the 32-token tiles of its chunk.  Per
// token tile every wave forms its own J^T tile (rows = tokens, columns = its latents; both
// half-normalisers ride in one correction k-step), rounds it to bf16 and publishes it in LDS; after
// one barrier it multiplies its tile with every wave's tile: the packed accumulator layout is at
// once a valid A operand (row = latent) and B operand (column = latent) over the same permuted
// token order.  LDS is double-buffered, so one barrier per token tile suffices.
// Output: the chunk's partial G, [b*h][chunk][M][M] fp32, summed in chunk order afterwards.
// ============================================================================================
template <int DR, int MT>
__global__ __launch_bounds__(64 * MT) void gram_mfma_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const float *__restrict__ lse_enc,
    const float *__restrict__ lse_dec, float *__restrict__ g_part, TokStride ts, int H, int N, int chunk_len,
    int chunks, float c2)
{
    constexpr int D = padded_dim(DR);
    constexpr int KS = D / 16;
    constexpr int M = 32 * MT;
    __shared__ __attribute__((aligned(16))) u32x4 jt[2][MT][2][64];
    const int lane = threadIdx.x & 63, l32 = lane & 31, hh = lane >> 5;
    const int wave = threadIdx.x >> 6;
    const GridPos gp = grid_pos(ts, H, DR * 2);
    const int bh = gp.y, h = bh % H, chunk = gp.x;
    const bool lower = hh == 0;

    bf16x8 qh[KS], ql[KS];
    load_q_operand<DR, true, false>(q + (size_t)h * ts.sq + (size_t)(32 * wave + l32) * DR, hh, c2, false, qh, ql);
    u32x4 wq;
    wq[0] = lower ? split_bf16_pair(-0.5f * kLog2e * lse_enc[(size_t)bh * M + 32 * wave + l32]) : 0u;
    wq[1] = lower ? 0x3f803f80u : 0u;      // slots 2,3 := 1 (pick the token's half-normaliser)
    wq[2] = 0u; wq[3] = 0u;
    const bf16x8 q_aug = as_bf16x8(wq);

    const bf16_t *kb = k + tok_base(ts, bh, H);
    const float *lb = lse_dec + (size_t)bh * N;
    const int n0 = chunk * chunk_len;
    const int n1 = min(N, n0 + chunk_len);
    const int tiles = (n1 - n0 + 31) / 32;
    f32x16 acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = splat16(0.f);

    // keys and lse_dec of a tile are requested one tile ahead (the last tile requests itself again: in bounds, unused)
    bf16x8 kt[KS], ktn[KS];
    float ld = 0.f, ldn = 0.f;
    auto request = [&](int j, bf16x8 (&kk)[KS], float &l) {
        const int n = min(n0 + 32 * min(j, tiles - 1) + l32, N - 1);
#pragma unroll
        for (int s = 0; s < KS; ++s) kk[s] = as_bf16x8(row8_bf16<DR>(kb + tok_off(ts, n), (D / 2) * hh + 8 * s));
        l = lb[n];
    };
    if (tiles > 0) request(0, kt, ld);
    for (int j = 0; j < tiles; ++j) {
        const int tok0 = n0 + 32 * j;
        request(j + 1, ktn, ldn);
        u32x4 wk;
        wk[0] = lower ? 0x3f803f80u : 0u;                                      // slots 0,1 := 1
        wk[1] = lower ? split_bf16_pair(-0.5f * kLog2e * ld) : 0u;             // slots 2,3 := -lse_dec2[n] / 2
        wk[2] = 0u; wk[3] = 0u;
        f32x16 x = splat16(0.f);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) x = mfma(kt[ks], qh[ks], x);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) x = mfma(kt[ks], ql[ks], x);
        x = mfma(as_bf16x8(wk), q_aug, x);
        if (tok0 + 32 > n1) {   // rows past the chunk's end contribute nothing
            const int rem = n1 - tok0 - 4 * hh;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (8 * (r / 4) + (r % 4) >= rem) x[r] = -INFINITY;
        }
        bf16x8 p0, p1;
        exp_pack(x, p0, p1);
        u32x4 (*buf)[2][64] = jt[j & 1];
        buf[wave][0][lane] = __builtin_bit_cast(u32x4, p0);
        buf[wave][1][lane] = __builtin_bit_cast(u32x4, p1);
        __syncthreads();
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            acc[t] = mfma(p0, as_bf16x8(buf[t][0][lane]), acc[t]);
            acc[t] = mfma(p1, as_bf16x8(buf[t][1][lane]), acc[t]);
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) kt[s] = ktn[s];
        ld = ldn;
    }
    float *out = g_part + ((size_t)bh * chunks + chunk) * M * M;
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 32 * wave + 8 * (r / 4) + 4 * hh + (r % 4);
            out[(size_t)row * M + 32 * t + l32] = acc[t][r];
        }
}

}  // namespace

bool mfma_supported(const flare_shape &s)
{
    if (s.dtype != FLARE_BF16 && s.dtype != FLARE_F16) return false;
    if (s.d != 4 && s.d != 8 && s.d != 16 && s.d != 32) return false;   // d < 16 runs padded to 16
    // A handful of tokens: every Z_m lies in the span of those few value rows, so c - delta = <dY_n, Z_m - Y_n>
    // and a - eps cancel almost completely and the bf16 operands' rounding shows in dQ and dK (two tokens,
    // fp16 storage, d = 16: up to 1.6e-1 measured; 9 and 12 tokens under more than a thousand latents: 2.1e-2 and 2.9e-2).
    // The fp32 kernels take such shapes; they cost nothing there.
    if (s.N < 16) return false;
    return s.M <= 2048;   // any number of latents: tiles of 32, the last ones padded
}

MfmaPlan mfma_plan(const flare_shape &s)
{
    MfmaPlan p;
    const EncGeom e = enc_geom(lat_eff(s.M), padded_dim(s.d));
    const int BH = s.B * s.H;
    // each chunk gives every token group at least 8 tiles of 32 tokens
    p.enc = plan_split(s.N, BH, 256 * e.TG, kEncodeTargetBlocks);
    p.parts = p.enc.chunks * e.TG;
    return p;
}

size_t mfma_fwd_bytes(const flare_shape &s)
{
    const MfmaPlan p = mfma_plan(s);
    Split sp;
    sp.chunks = p.parts;
    sp.chunk_len = 0;
    return valu_fwd_layout(s, sp, nullptr, nullptr, nullptr, nullptr);
}

int mfma_encode(const flare_shape &s, const void *q, const void *k, const void *v, float *z, float *lse_enc,
                float scale, void *ws, hipStream_t stream)
{
    const MfmaPlan p = mfma_plan(s);
    const EncGeom e = enc_geom(lat_eff(s.M), padded_dim(s.d));
    Split sp;
    sp.chunks = p.parts;
    sp.chunk_len = 0;
    float *m_part, *l_part, *o_part;
    valu_fwd_layout(s, sp, ws, &m_part, &l_part, &o_part);
    const int BH = s.B * s.H;
    const float c2 = scale * kLog2e;
    const dim3 grid(p.enc.chunks, BH, lat_chunks(s.M));
    const bf16_t *qq = (const bf16_t *)q, *kk = (const bf16_t *)k, *vv = (const bf16_t *)v;
    {
        LaunchTimer t(KID_ENCODE_PARTIAL, stream);
        const bool f16 = s.dtype == FLARE_F16;
#define FLARE_ENC(DD, NBB)                                                                                        \
    do {                                                                                                          \
        if (f16)                                                                                                  \
            encode_mfma_kernel<DD, NBB, 2, 0, true><<<grid, e.threads, 0, stream>>>(                              \
                qq, kk, vv, nullptr, 1.f, nullptr, nullptr, nullptr, m_part, l_part, o_part, tok_stride(s), s.H,  \
                s.N, s.M, p.enc.chunk_len, p.parts, e.G, e.TG, c2);                                               \
        else                                                                                                      \
            encode_mfma_kernel<DD, NBB, 2, 0, false><<<grid, e.threads, 0, stream>>>(                             \
                qq, kk, vv, nullptr, 1.f, nullptr, nullptr, nullptr, m_part, l_part, o_part, tok_stride(s), s.H,  \
                s.N, s.M, p.enc.chunk_len, p.parts, e.G, e.TG, c2);                                               \
    } while (0)
#define FLARE_ENC_NB(DD)                   \
    do {                                   \
        if (e.NB == 1) FLARE_ENC(DD, 1);   \
        else if (e.NB == 2) FLARE_ENC(DD, 2); \
        else FLARE_ENC(DD, 4);             \
    } while (0)
        switch (s.d) {
            case 4: FLARE_ENC_NB(4); break;
            case 8: FLARE_ENC_NB(8); break;
            case 16: FLARE_ENC_NB(16); break;
            default:
                if (e.NB == 1) FLARE_ENC(32, 1);
                else FLARE_ENC(32, 2);
        }
#undef FLARE_ENC_NB
#undef FLARE_ENC
    }
    if (check_launch() != FLARE_OK) return FLARE_ELAUNCH;
    return launch_encode_merge(s, m_part, l_part, o_part, z, lse_enc, p.parts, stream);
}

// dZ partials of the backward (the encode machinery with values dY and weights R^T)
int mfma_dz_partial(const flare_shape &s, const void *q, const void *k, const void *dy, const float *lse_dec2,
                    float ld_mul, const void *y, float *delta_out, float *ld_range, float *dz_part, float scale,
                    hipStream_t stream)
{
    const MfmaPlan p = mfma_plan(s);
    const EncGeom e = enc_geom(lat_eff(s.M), padded_dim(s.d));
    const int BH = s.B * s.H;
    const float c2 = scale * kLog2e;
    const dim3 grid(p.enc.chunks, BH, lat_chunks(s.M));
    const bf16_t *qq = (const bf16_t *)q, *kk = (const bf16_t *)k, *gg = (const bf16_t *)dy;
    LaunchTimer t(KID_BWD_DZ_PARTIAL, stream);
    const bool f16 = s.dtype == FLARE_F16;
    if (y != nullptr && s.y_f32 && s.d > 8) return FLARE_EUNSUPPORTED;   // the caller forms delta itself there
    const int y32 = (y != nullptr && s.y_f32) ? 1 : 0;
#define FLARE_DZ_ARGS                                                                                            \
    qq, kk, gg, lse_dec2, ld_mul, (const bf16_t *)y, delta_out, ld_range, nullptr, nullptr, dz_part, tok_stride(s), \
        s.H, s.N, s.M, p.enc.chunk_len, p.parts, e.G, e.TG, c2
#define FLARE_DZ(DD, NBB)                                                                                         \
    do {                                                                                                          \
        if constexpr (DD <= 8) {                                                                                  \
            if (y32 && f16) {                                                                                     \
                encode_mfma_kernel<DD, NBB, 2, 1, true, true><<<grid, e.threads, 0, stream>>>(FLARE_DZ_ARGS);     \
                break;                                                                                            \
            } else if (y32) {                                                                                     \
                encode_mfma_kernel<DD, NBB, 2, 1, false, true><<<grid, e.threads, 0, stream>>>(FLARE_DZ_ARGS);    \
                break;                                                                                            \
            }                                                                                                     \
        }                                                                                                         \
        if (f16)                                                                                                  \
            encode_mfma_kernel<DD, NBB, 2, 1, true><<<grid, e.threads, 0, stream>>>(FLARE_DZ_ARGS);               \
        else                                                                                                      \
            encode_mfma_kernel<DD, NBB, 2, 1, false><<<grid, e.threads, 0, stream>>>(FLARE_DZ_ARGS);              \
    } while (0)
#define FLARE_DZ_NB(DD)                   \
    do {                                  \
        if (e.NB == 1) FLARE_DZ(DD, 1);   \
        else if (e.NB == 2) FLARE_DZ(DD, 2); \
        else FLARE_DZ(DD, 4);             \
    } while (0)
    switch (s.d) {
        case 4: FLARE_DZ_NB(4); break;
        case 8: FLARE_DZ_NB(8); break;
        case 16: FLARE_DZ_NB(16); break;
        default:
            if (e.NB == 1) FLARE_DZ(32, 1);
            else FLARE_DZ(32, 2);
    }
#undef FLARE_DZ_NB
#undef FLARE_DZ
#undef FLARE_DZ_ARGS
    return check_launch();
}

template <int MODE>
static int launch_decode_family(const flare_shape &s, const void *q, const void *k, const float *z, void *y,
                                TokStride ts_y, const void *dy, float *lse_dec2, float *delta, int m0, int Mc,
                                float scale, hipStream_t stream, int flags = 0)
{
    const int BH = s.B * s.H;
    const int tiles = (s.N + 31) / 32;
    // d = 32 with 192 or 256 latents (Z in LDS, 168 registers): three workgroups fit a CU
    const bool three = padded_dim(s.d) == 32 && Mc > 128;
    int blocks = ((three ? 768 : kDecodeTargetBlocks) + BH - 1) / BH;
    if (blocks > (tiles + 3) / 4) blocks = (tiles + 3) / 4;
    const dim3 grid(blocks, BH);
    const float c2 = scale * kLog2e;
    const bf16_t *qq = (const bf16_t *)q, *kk = (const bf16_t *)k, *gg = (const bf16_t *)dy;
    bf16_t *yy = (bf16_t *)y;
    LaunchTimer t(MODE == 0 ? KID_DECODE : KID_BWD_TOKEN_STATS, stream);
    const bool f16 = s.dtype == FLARE_F16;
#define FLARE_DEC_ARGS qq, kk, z, yy, gg, lse_dec2, delta, tok_stride(s), ts_y, s.H, s.N, s.M, m0, c2, flags
#define FLARE_DEC(DD, MTT, PREE, MINB)                                                                          \
    do {                                                                                                        \
        if (f16)                                                                                                \
            decode_mfma_kernel<DD, MTT, PREE, MINB, MODE, true><<<grid, 256, 0, stream>>>(FLARE_DEC_ARGS);      \
        else                                                                                                    \
            decode_mfma_kernel<DD, MTT, PREE, MINB, MODE, false><<<grid, 256, 0, stream>>>(FLARE_DEC_ARGS);     \
    } while (0)
    const int MT = Mc / 32;
#define FLARE_DEC_MT(DD)                               \
    switch (MT) {                                      \
        case 1: FLARE_DEC(DD, 1, true, 2); break;      \
        case 2: FLARE_DEC(DD, 2, true, 2); break;      \
        case 4: FLARE_DEC(DD, 4, true, 2); break;      \
        case 6: FLARE_DEC(DD, 6, true, 2); break;      \
        case 8: FLARE_DEC(DD, 8, true, 2); break;      \
        default: return FLARE_EUNSUPPORTED;            \
    }
    if (s.d == 4) {
        FLARE_DEC_MT(4)
    } else if (s.d == 8) {
        FLARE_DEC_MT(8)
    } else if (s.d == 16) {
        FLARE_DEC_MT(16)
    } else {
        switch (MT) {
            case 1: FLARE_DEC(32, 1, true, 2); break;
            case 2: FLARE_DEC(32, 2, true, 2); break;
            case 4: FLARE_DEC(32, 4, true, 2); break;
            case 6: FLARE_DEC(32, 6, false, 2); break;
            case 8: FLARE_DEC(32, 8, false, 2); break;
            default: return FLARE_EUNSUPPORTED;
        }
    }
#undef FLARE_DEC_MT
#undef FLARE_DEC
#undef FLARE_DEC_ARGS
    return check_launch();
}

namespace {
// Combine the per-chunk results of the decode (M > 256): for token n of (b,h),
//   lse = log sum_c exp(lse_c),   y = sum_c exp(lse_c - lse) y_c        (softmax over all M latents).
// Writes y in the caller's layout and, when asked, lse_dec (natural log).
// thread = token; the partial rows are [chunk][b*h][n][DR] in the storage type, the partial lse [chunk][b*h][n].
template <int DR, bool F>
__global__ __launch_bounds__(256) void decode_merge_kernel(
    const bf16_t *__restrict__ y_part, const float *__restrict__ lse_part, int chunks, bf16_t *__restrict__ y,
    float *__restrict__ lse_out, TokStride ts, int H, int N, size_t rows_all)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    const int bh = blockIdx.y;
    const size_t row = (size_t)bh * N + n;
    float mx = -INFINITY;
    for (int c = 0; c < chunks; ++c) mx = fmaxf(mx, lse_part[(size_t)c * rows_all + row]);
    float acc[DR], tot = 0.f;
#pragma unroll
    for (int j = 0; j < DR; ++j) acc[j] = 0.f;
    for (int c = 0; c < chunks; ++c) {
        const float w = __expf(lse_part[(size_t)c * rows_all + row] - mx);
        tot += w;
        const bf16_t *src = y_part + ((size_t)c * rows_all + row) * DR;
#pragma unroll
        for (int j = 0; j < DR; j += 4) {
            const u32x2 t = *reinterpret_cast<const u32x2 *>(src + j);
            acc[j] = fmaf(w, elem_lo<F>(t[0]), acc[j]);
            acc[j + 1] = fmaf(w, elem_hi<F>(t[0]), acc[j + 1]);
            acc[j + 2] = fmaf(w, elem_lo<F>(t[1]), acc[j + 2]);
            acc[j + 3] = fmaf(w, elem_hi<F>(t[1]), acc[j + 3]);
        }
    }
    const float inv = 1.f / tot;
    const size_t trow = tok_base(ts, bh, H) + tok_off(ts, n);
#pragma unroll
    for (int j = 0; j < DR; j += 4) {
        u32x2 w;
        w[0] = pack_elems<F>(acc[j] * inv, acc[j + 1] * inv);
        w[1] = pack_elems<F>(acc[j + 2] * inv, acc[j + 3] * inv);
        *reinterpret_cast<u32x2 *>(y + trow + j) = w;
    }
    if (lse_out) lse_out[row] = mx + __logf(tot);
}

// The same for fp32 rows (flare_shape.y_f32): fp32 partial rows in, fp32 y out.
template <int DR>
__global__ __launch_bounds__(256) void decode_merge_f32_kernel(
    const float *__restrict__ y_part, const float *__restrict__ lse_part, int chunks, float *__restrict__ y,
    float *__restrict__ lse_out, TokStride ts, int H, int N, size_t rows_all)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    const int bh = blockIdx.y;
    const size_t row = (size_t)bh * N + n;
    float mx = -INFINITY;
    for (int c = 0; c < chunks; ++c) mx = fmaxf(mx, lse_part[(size_t)c * rows_all + row]);
    float acc[DR], tot = 0.f;
#pragma unroll
    for (int j = 0; j < DR; ++j) acc[j] = 0.f;
    for (int c = 0; c < chunks; ++c) {
        const float w = __expf(lse_part[(size_t)c * rows_all + row] - mx);
        tot += w;
        const float *src = y_part + ((size_t)c * rows_all + row) * DR;
#pragma unroll
        for (int j = 0; j < DR; j += 4) {
            const float4 t = *reinterpret_cast<const float4 *>(src + j);
            acc[j] = fmaf(w, t.x, acc[j]);
            acc[j + 1] = fmaf(w, t.y, acc[j + 1]);
            acc[j + 2] = fmaf(w, t.z, acc[j + 2]);
            acc[j + 3] = fmaf(w, t.w, acc[j + 3]);
        }
    }
    const float inv = 1.f / tot;
    float *dst = y + tok_base(ts, bh, H) + tok_off(ts, n);
#pragma unroll
    for (int j = 0; j < DR; j += 4)
        *reinterpret_cast<float4 *>(dst + j) = make_float4(acc[j] * inv, acc[j + 1] * inv, acc[j + 2] * inv, acc[j + 3] * inv);
    if (lse_out) lse_out[row] = mx + __logf(tot);
}

// Combine the per-chunk token statistics of the backward (M > 256).  Chunk c gives, for token n,
// lse2_c = log2 sum_{m in c} 2^S2[m][n] and delta_c = <dY_n, Y_n^c> with Y_n^c the decode over the chunk's
// latents alone, formed in fp32 registers; then
//   lse_dec2 = log2 sum_c 2^lse2_c,   delta = sum_c 2^(lse2_c - lse_dec2) delta_c.
// (Going through 16-bit rows of Y^c instead would put their rounding into delta, and c - delta is a
// difference that must cancel: measured 2.9e-2 against 7e-3 in dq_lat at d = 4.)  thread = token row.
__global__ __launch_bounds__(256) void stats_merge_kernel(const float *__restrict__ lse_part,
                                                          const float *__restrict__ delta_part, int chunks,
                                                          float *__restrict__ lse_out, float *__restrict__ delta,
                                                          size_t rows)
{
    const size_t row = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= rows) return;
    float mx = -INFINITY;
    for (int c = 0; c < chunks; ++c) mx = fmaxf(mx, lse_part[(size_t)c * rows + row]);
    float tot = 0.f, dl = 0.f;
    for (int c = 0; c < chunks; ++c) {
        const float w = fast_exp2(lse_part[(size_t)c * rows + row] - mx);
        tot += w;
        dl = fmaf(w, delta_part[(size_t)c * rows + row], dl);
    }
    lse_out[row] = mx + log2f(tot);
    delta[row] = dl / tot;
}
}  // namespace

// bytes of the per-chunk partial results of the token-major forward kernels (0 when M <= 256)
size_t mfma_tok_part_bytes(const flare_shape &s)
{
    if (s.M <= kLatChunk) return 0;
    const size_t rows = (size_t)s.B * s.H * s.N * lat_chunks(s.M);
    return ((rows * s.d * (s.y_f32 ? 4 : 2) + 255) & ~(size_t)255) + ((rows * 4 + 255) & ~(size_t)255);
}

// decode (MODE 0) or token statistics (MODE 1) over all latents, in chunks of 256 when there are more
template <int MODE>
static int decode_all(const flare_shape &s, const void *q, const void *k, const float *z, void *y, const void *dy,
                      float *lse_out, float *delta, float scale, void *ws, hipStream_t stream, int flags = 0)
{
    if (s.M <= kLatChunk)
        return launch_decode_family<MODE>(s, q, k, z, y, tok_stride(s), dy, lse_out, delta, 0, lat_eff(s.M), scale,
                                          stream, flags);
    const int C = lat_chunks(s.M);
    const size_t rows = (size_t)s.B * s.H * s.N;
    const size_t es = s.y_f32 ? 4 : 2;          // bytes per element of the partial rows
    float *lse_part = reinterpret_cast<float *>(static_cast<char *>(ws) + ((rows * C * s.d * es + 255) & ~(size_t)255));
    if constexpr (MODE == 1) {
        // per-chunk statistics in fp32 (delta_c in the space of the partial rows, which this mode does not need)
        float *delta_part = static_cast<float *>(ws);
        for (int c = 0; c < C; ++c) {
            const int rc = launch_decode_family<1>(s, q, k, z, nullptr, tok_stride(s), dy, lse_part + (size_t)c * rows,
                                                   delta_part + (size_t)c * rows, c * kLatChunk, kLatChunk, scale,
                                                   stream, flags);
            if (rc != FLARE_OK) return rc;
        }
        LaunchTimer t(KID_DECODE_MERGE, stream);
        stats_merge_kernel<<<(unsigned)((rows + 255) / 256), 256, 0, stream>>>(lse_part, delta_part, C, lse_out, delta,
                                                                              rows);
        return check_launch();
    } else {
        bf16_t *y_part = static_cast<bf16_t *>(ws);
        const TokStride tp{(long long)s.H * s.N * s.d, (long long)s.N * s.d, s.d, 0};   // partial rows: [b][h][n][d]
        for (int c = 0; c < C; ++c) {
            void *part_c = static_cast<char *>(ws) + (size_t)c * rows * s.d * es;
            const int rc = launch_decode_family<0>(s, q, k, z, part_c, tp, nullptr, lse_part + (size_t)c * rows, nullptr,
                                                   c * kLatChunk, kLatChunk, scale, stream, flags);
            if (rc != FLARE_OK) return rc;
        }
        const dim3 grid((s.N + 255) / 256, s.B * s.H);
        LaunchTimer t(KID_DECODE_MERGE, stream);
        if (s.y_f32) {
            const float *yp = static_cast<const float *>(ws);
            switch (s.d) {
                case 4: decode_merge_f32_kernel<4><<<grid, 256, 0, stream>>>(yp, lse_part, C, (float *)y, lse_out, tok_stride(s), s.H, s.N, rows); break;
                case 8: decode_merge_f32_kernel<8><<<grid, 256, 0, stream>>>(yp, lse_part, C, (float *)y, lse_out, tok_stride(s), s.H, s.N, rows); break;
                case 16: decode_merge_f32_kernel<16><<<grid, 256, 0, stream>>>(yp, lse_part, C, (float *)y, lse_out, tok_stride(s), s.H, s.N, rows); break;
                default: decode_merge_f32_kernel<32><<<grid, 256, 0, stream>>>(yp, lse_part, C, (float *)y, lse_out, tok_stride(s), s.H, s.N, rows); break;
            }
            return check_launch();
        }
        const bool f16 = s.dtype == FLARE_F16;
#define FLARE_DM(DD)                                                                                              \
    do {                                                                                                          \
        if (f16)                                                                                                  \
            decode_merge_kernel<DD, true><<<grid, 256, 0, stream>>>(y_part, lse_part, C, (bf16_t *)y, lse_out,    \
                                                                    tok_stride(s), s.H, s.N, rows);               \
        else                                                                                                      \
            decode_merge_kernel<DD, false><<<grid, 256, 0, stream>>>(y_part, lse_part, C, (bf16_t *)y, lse_out,   \
                                                                     tok_stride(s), s.H, s.N, rows);              \
    } while (0)
        switch (s.d) {
            case 4: FLARE_DM(4); break;
            case 8: FLARE_DM(8); break;
            case 16: FLARE_DM(16); break;
            default: FLARE_DM(32); break;
        }
#undef FLARE_DM
        return check_launch();
    }
}

// partial companion matrices [b*h][chunk][M][M]; the split of the token axis is returned in *sp
bool mfma_gram_supported(const flare_shape &s)
{
    return mfma_supported(s) && s.dtype == FLARE_BF16 && (s.M == 32 || s.M == 64 || s.M == 128 || s.M == 256);
}

int mfma_gram_partial(const flare_shape &s, const Split &sp, const void *q, const void *k, const float *lse_enc,
                      const float *lse_dec, float *g_part, float scale, hipStream_t stream)
{
    const dim3 grid(sp.chunks, s.B * s.H);
    const float c2 = scale * kLog2e;
    const bf16_t *qq = (const bf16_t *)q, *kk = (const bf16_t *)k;
    LaunchTimer t(KID_SPECTRAL_GRAM, stream);
#define FLARE_GRAM(DD, MTT)                                                                                  \
    gram_mfma_kernel<DD, MTT><<<grid, 64 * MTT, 0, stream>>>(qq, kk, lse_enc, lse_dec, g_part, tok_stride(s), s.H, \
                                                             s.N, sp.chunk_len, sp.chunks, c2)
#define FLARE_GRAM_MT(DD)                       \
    switch (s.M / 32) {                         \
        case 1: FLARE_GRAM(DD, 1); break;       \
        case 2: FLARE_GRAM(DD, 2); break;       \
        case 4: FLARE_GRAM(DD, 4); break;       \
        default: FLARE_GRAM(DD, 8); break;      \
    }
    switch (s.d) {
        case 4: FLARE_GRAM_MT(4) break;
        case 8: FLARE_GRAM_MT(8) break;
        case 16: FLARE_GRAM_MT(16) break;
        default: FLARE_GRAM_MT(32) break;
    }
#undef FLARE_GRAM_MT
#undef FLARE_GRAM
    return check_launch();
}

int mfma_decode(const flare_shape &s, const void *q, const void *k, const float *z, void *y, float *lse_dec,
                float scale, void *ws, hipStream_t stream)
{
    // an fp32 y is what the backward will form delta from: at d <= 8 its rows carry Z as the
    // hi + lo pair that the backward's c chain carries (see mfma_token_stats)
    const int flags = s.y_f32 ? (2 | (s.d <= 8 ? 1 : 0)) : 0;
    return decode_all<0>(s, q, k, z, y, nullptr, lse_dec, nullptr, scale, ws, stream, flags);
}

int mfma_token_stats(const flare_shape &s, const void *q, const void *k, const float *z, const void *dy,
                     float *lse_dec2, float *delta, float scale, void *ws, hipStream_t stream)
{
    // d <= 8: delta from rows of Y that carry Z as a hi + lo pair, where every kernel that subtracts it from
    // c = <Z_m, dY_n> carries that pair too (c - delta must cancel where one latent dominates a token): the
    // dQ kernel does, the dK/dV kernel that also forms dQ does, and the plain dK/dV kernel does at d = 4 only.
    const bool z_lo = s.d == 4 || (s.d == 8 && mfma_dkdv_supported(s) && mfma_dq_fused(s));
    return decode_all<1>(s, q, k, z, nullptr, dy, lse_dec2, delta, scale, ws, stream, z_lo ? 1 : 0);
}

}  // namespace flare
