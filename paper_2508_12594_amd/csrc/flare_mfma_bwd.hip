// Matrix-core kernels of the second backward pass: dQ, dK, dV (one kernel at d <= 16, two otherwise),
// the per-(b,h) choice between the one- and two-exponential variants, and the fp32 sums of latent chunks.
// Operand layouts, helpers and the tile geometry are in flare_mfma_common.h.
#include "flare_mfma_common.h"

namespace flare {
namespace {

// ============================================================================================
// Backward, dQ partials (latent-major, same wave geometry as the encode).  For its NB latent tiles
// a wave keeps, as B operands (column = latent, contraction over d): q' hi and lo, dZ (bf16-exact: it is
// rounded where it is merged, before eps is formed) and Z in bf16 (hi and, at d = 16, lo).  Per 32-token tile it streams K, V and dY as A operands
// (row = token) and forms, all on the matrix cores,
//     S2 - lse_enc2[m]   (one more k-step: -lse_enc2 as a hi+lo pair in slots 0,1, against 1,1)
//     S2 - lse_dec2[n]   (likewise -lse_dec2 in slots 2,3 of the token-side operand)
//     a[n][m] = <V_n, dZ_m> - eps[m]      (-eps rides in one more, otherwise empty, k-step)
//     c[n][m] = <dY_n, Z_m> - delta[n]    (-delta likewise)
// then dS^T = 2^(..) a + 2^(..) c in fp32, rounds it to bf16 and accumulates
//     dQ^T[dd][m] += K^T[dd][n] dS^T[n][m]
// with K^T read back from a wave-private, double-buffered LDS tile.  Masked tokens have both
// exponents at -inf, so their dS is exactly zero.
//
// ONE = true is the variant with one exponential per score, P~ = 2^S2 without a normaliser:
//     P = P~ e[m],  R = P~ w[n],   e[m] = 2^-lse_enc2[m],  w[n] = 2^-lse_dec2[n],
// so dS^T = P~ (e[m] (a - eps) + w[n] (c - delta)).  e[m] arrives folded into dZ and eps (the kernel that merges
// the dZ partials scales dZ before it rounds it and forms eps), so the a chain needs nothing new and the score
// products need no correction k-step; w[n] is a per-row factor that goes from the token's lane to the rows of
// the accumulator layout through 128 bytes of LDS (and multiplies delta in the correction k-step).  It is exact
// as long as both log-sum-exps stay within +-60, which bwd_one_exp_ok checks per (b,h) (plan[bh] = 1);
// otherwise the ONE = false variant runs.  Each variant returns at once when the plan names the other.
// ============================================================================================
template <int DR, int NB, int MINB, bool ONE, bool F>
__device__ __forceinline__ void dq_body(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const bf16_t *__restrict__ dy, const float *__restrict__ z, const float *__restrict__ lse_enc,
    const float *__restrict__ dz, const float *__restrict__ eps, const float *__restrict__ lse_dec2,
    const float *__restrict__ delta, float ld_mul, const int *__restrict__ plan, float *__restrict__ dq_part,
    TokStride ts, int H, int N, int M, int chunk_len, int parts, int G, int TG, float c2)
{
    constexpr int D = padded_dim(DR);
    constexpr int KS = D / 16;
    // Row blocks of the dQ accumulation.  d <= 16: one 32x32 product per 16 columns (rows 16-31 of the K^T
    // operand are zero).  d = 32: the 32 columns fill the 32 rows of ONE product (WIDE).
    constexpr bool WIDE = (D == 32);
    constexpr int HV = WIDE ? 1 : D / 16;
    constexpr int QUARTS = WIDE ? 4 : 2;        // 4-column pieces per lane and accumulator: columns 8 q + 4 hh (+ 16 hv)
    constexpr int ROWS = D + 1;                 // K^T rows, then a row of zeros
    // d <= 8: the upper half of the padded contraction carries what otherwise needs products of its own:
    // q' lo and Z lo (K and dY rows repeated in both lane halves) and -eps (against ones in the V operand).
    constexpr bool PACK = pack_dim(DR);
    // d = 32: the key tile goes to LDS as loaded, row = token (kKwStride uint16 a row: 80 B, two 16-byte stores per
    // lane), and the transposing read forms the K^T operand; d <= 16: transposed on the way in, two bytes a store.
    constexpr int kKwStride = 40;
    constexpr int BUF = WIDE ? 32 * kKwStride : ROWS * kVtStride;
    __shared__ __attribute__((aligned(16))) uint16_t kt_all[4][2 * BUF];
    __shared__ __attribute__((aligned(16))) float wl_all[ONE ? 4 : 1][2][32];   // w[n] of a token tile

    const int lane = threadIdx.x & 63, l32 = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // known to be wave-uniform: scalar unit
    const int g = wave % G, tg = wave / G;
    const GridPos gp = grid_pos(ts, H, DR * 2);
    const int bh = gp.y, h = bh % H, chunk = gp.x;
    if ((plan[bh] != 0) != ONE) return;         // the other variant owns this (b,h)
    const bool lower = hh == 0;
    uint16_t *lds = kt_all[wave];
    float (*wl)[32] = wl_all[ONE ? wave : 0];
    constexpr float kap = 0.f;                  // w[n] = 2^(kap - lse_dec2[n])
    if (!WIDE && lane < kVtStride) {
        lds[D * kVtStride + lane] = 0;
        lds[BUF + D * kVtStride + lane] = 0;
        if constexpr (PACK) {   // K^T rows 8-15 are never written: zero, so that the unused output rows stay finite
#pragma unroll
            for (int r = 8; r < 16; ++r) {
                lds[r * kVtStride + lane] = 0;
                lds[BUF + r * kVtStride + lane] = 0;
            }
        }
    }

    // ---- per-latent operands ----
    const int lat0 = 32 * NB * (G * (int)blockIdx.z + g);   // a workgroup owns NB*G tiles of latents
    constexpr bool LO2 = (D == 16);             // carry the lo term of Z as well (dZ arrives bf16-exact)
    bf16x8 qh[NB][KS], ql[NB][KS], q_aug[NB], dzb[NB][KS], zb[NB][KS], zl[NB][KS], dz_aug[NB];
    bf16x8 u_aug[ONE ? NB : 1];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        // padding latents (at or beyond M): every operand zero, loads clamped to the last real latent
        const bool real = lat0 + 32 * b + l32 < M;
        const int m = min(lat0 + 32 * b + l32, M - 1);
        load_q_operand<DR, true, F, PACK>(q + (size_t)h * ts.sq + (size_t)m * DR, hh, c2, false, qh[b], ql[b]);
        if (!real) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) { qh[b][ks] = zero_operand(); ql[b][ks] = zero_operand(); }
        }
        const float le2 = real ? lse_enc[(size_t)bh * M + m] * kLog2e : 0.f;
        const float um = 1.f;                       // (a per-latent factor of the c chain: none in either variant)
        if constexpr (ONE) {
            const uint32_t us = split_bf16_pair(um);          // slots 0,1,2 := u hi, u hi, u lo
            u32x4 wu;
            wu[0] = lower ? ((us & 0xffffu) | (us << 16)) : 0u;
            wu[1] = lower ? (us >> 16) : 0u;
            // slots 4,5 := -eps (hi + lo): with one exponential the a chain's correction rides in the same
            // product as the c chain's (against ones in the token operand), see the tile loop
            wu[2] = (!PACK && lower) ? split_bf16_pair(real ? -eps[(size_t)bh * M + m] : 0.f) : 0u;
            wu[3] = 0u;
            u_aug[b] = as_bf16x8(wu);
        }
        u32x4 wq;
        wq[0] = lower ? split_pair<F>(-le2) : 0u;       // slots 0,1 := -lse_enc2 (hi + lo)
        wq[1] = lower ? kOnePair<F> : 0u;               // slots 2,3 := 1
        wq[2] = 0u; wq[3] = 0u;
        q_aug[b] = as_bf16x8(wq);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            float zr[8], dr[8];
            row8_f32<DR>(z + ((size_t)bh * M + m) * DR, PACK ? 0 : (D / 2) * hh + 8 * s, zr);
            row8_f32<DR>(dz + ((size_t)bh * M + m) * DR, (D / 2) * hh + 8 * s, dr);
            if (!real) {
#pragma unroll
                for (int i = 0; i < 8; ++i) { zr[i] = 0.f; dr[i] = 0.f; }
            }
            u32x4 wz, wd, wzl;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float za = zr[2 * i] * um, zc = zr[2 * i + 1] * um;
                const uint32_t z0 = rne_bf16(za), z1 = rne_bf16(zc);
                const uint32_t d0 = rne_bf16(dr[2 * i]), d1 = rne_bf16(dr[2 * i + 1]);
                wz[i] = z0 | (z1 << 16);
                wd[i] = d0 | (d1 << 16);
                wzl[i] = rne_bf16(za - __uint_as_float(z0 << 16)) |
                         (rne_bf16(zc - __uint_as_float(z1 << 16)) << 16);
            }
            zb[b][s] = as_bf16x8((PACK && !lower) ? wzl : wz);
            dzb[b][s] = as_bf16x8(wd);
            zl[b][s] = as_bf16x8(wzl);
        }
        u32x4 we;
        we[0] = (lower != PACK) ? split_bf16_pair(real ? -eps[(size_t)bh * M + m] : 0.f) : 0u;
        we[1] = 0u; we[2] = 0u; we[3] = 0u;
        dz_aug[b] = as_bf16x8(we);
        if constexpr (PACK) {   // slots 8,9 of the dZ operand := -eps (the rest of its upper half is zero)
            u32x4 wd = __builtin_bit_cast(u32x4, dzb[b][0]);
            if (!lower) wd[0] = we[0];
            dzb[b][0] = as_bf16x8(wd);
        }
    }
    u32x4 w11;
    w11[0] = lower ? 0x3f803f80u : 0u;
    w11[1] = 0u; w11[2] = 0u; w11[3] = 0u;
    const bf16x8 ones_aug = as_bf16x8(w11);      // slots 0,1 = 1 in the lower lane half, else 0
    w11[0] = lower ? kOnePair<F> : 0u;
    const bf16x8 ones_s = as_bf16x8(w11);        // the same in the type of the score products
    auto to_bf16 = [](bf16x8 x) { return as_bf16x8(to_bf16_row<F>(__builtin_bit_cast(u32x4, x))); };
    // V rows as the operand of the a product; PACK: slots 8,9 := 1 (the upper lane half loaded zeros)
    auto v_operand = [&](bf16x8 x) {
        u32x4 w = to_bf16_row<F>(__builtin_bit_cast(u32x4, x));
        if (PACK && !lower) w[0] = 0x3f803f80u;
        return as_bf16x8(w);
    };

    const bf16_t *kb = k + tok_base(ts, bh, H);
    const bf16_t *vb = v + tok_base(ts, bh, H);
    const bf16_t *gb = dy + tok_base(ts, bh, H);
    const float *lb = lse_dec2 + (size_t)bh * N;
    const float *db = delta + (size_t)bh * N;
    const int n0 = chunk * chunk_len;
    const int n1 = min(N, n0 + chunk_len);
    const int tiles = (n1 - n0 + 31) / 32;
    const int cnt = (tiles > tg) ? (tiles - tg + TG - 1) / TG : 0;

    f32x16 acc[NB][HV];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int hv = 0; hv < HV; ++hv) acc[b][hv] = splat16(0.f);

    int krow[HV];
#pragma unroll
    for (int hv = 0; hv < HV; ++hv) krow[hv] = WIDE ? l32 : ((l32 < 16) ? 16 * hv + l32 : D);

    auto tile_tok0 = [&](int j) { return n0 + 32 * (tg + min(j, cnt - 1) * TG); };
    // A operand: row = token.  rep (PACK only): both lane halves get elements 0-7 of the row.
    auto load_rows = [&](const bf16_t *base, int j, bf16x8 (&t)[KS], bool rep) {
        const int n = min(tile_tok0(j) + l32, N - 1);
#pragma unroll
        for (int s = 0; s < KS; ++s)
            t[s] = as_bf16x8(row8_bf16<DR>(base + tok_off(ts, n), (PACK && rep) ? 0 : (D / 2) * hh + 8 * s));
    };
    auto write_kt = [&](const bf16x8 (&t)[KS], uint16_t *buf) {   // transposed: row = d-index, column = token
        if (PACK && !lower) return;   // the upper lane half holds a copy of the same elements
        if constexpr (WIDE) {
#pragma unroll
            for (int s = 0; s < KS; ++s)
                *reinterpret_cast<u32x4 *>(buf + l32 * kKwStride + (D / 2) * hh + 8 * s) =
                    to_bf16_row<F>(__builtin_bit_cast(u32x4, t[s]));
            return;
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const u32x4 w = to_bf16_row<F>(__builtin_bit_cast(u32x4, t[s]));   // K as a value: bf16
            const int d0 = (D / 2) * hh + 8 * s;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                buf[(d0 + 2 * e) * kVtStride + l32] = (uint16_t)(w[e] & 0xffffu);
                buf[(d0 + 2 * e + 1) * kVtStride + l32] = (uint16_t)(w[e] >> 16);
            }
        }
    };
    auto read_kT = [&](const uint16_t *buf, bf16x8 (&kT)[HV][2]) {
#pragma unroll
        for (int hv = 0; hv < HV; ++hv)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                if constexpr (WIDE) {
                    // lanes 16 i .. 16 i + 15 hand in four rows (tokens) of 16 columns (d-indices 16 (i & 1) ..) and
                    // lane c of them receives column c of the four: tokens 16 s2 + 4 hh + 0..3, then + 8..11
                    const int c16 = lane & 15;
                    const uint16_t *src =
                        buf + (16 * s2 + 4 * hh + (c16 >> 2)) * kKwStride + 16 * (l32 >> 4) + 4 * (c16 & 3);
                    const u32x2 a = lds_read_tr16(src), b = lds_read_tr16(src + 8 * kKwStride);
                    kT[hv][s2] = as_bf16x8(u32x4{a[0], a[1], b[0], b[1]});
                    continue;
                }
                const uint16_t *row = buf + krow[hv] * kVtStride + 16 * s2 + 4 * hh;
                const u32x2 a = *reinterpret_cast<const u32x2 *>(row);
                const u32x2 b = *reinterpret_cast<const u32x2 *>(row + 8);
                u32x4 w;
                w[0] = a[0]; w[1] = a[1]; w[2] = b[0]; w[3] = b[1];
                kT[hv][s2] = as_bf16x8(w);
            }
    };

    // w[n] of a tile: written by the token's lane, read back as the 16 rows of this lane's registers
    auto read_w = [&](const float *buf, float (&wr)[16]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 t = *reinterpret_cast<const float4 *>(buf + 8 * i + 4 * hh);
            wr[4 * i] = t.x; wr[4 * i + 1] = t.y; wr[4 * i + 2] = t.z; wr[4 * i + 3] = t.w;
        }
    };

    if (cnt > 0) {
        // The rows of a token tile (keys, values, dY, as loaded) and its two statistics are requested as soon as
        // the tile three places earlier is done with its registers: a tile of this kernel is short (one or two
        // latent tiles), and a request has to be older than the memory latency when its rows are needed (the keys
        // two tiles later, the rest three).  Three sets of registers take turns as current tile, next tile and in
        // flight, so that no register of a load in flight is ever copied.
        struct Rows {
            bf16x8 k[KS], v[KS], g[KS];
            float l, d;   // lse_dec2 as stored, delta
        };
        auto request = [&](int j, Rows &r) {
            load_rows(kb, j, r.k, true);
            load_rows(vb, j, r.v, false);
            load_rows(gb, j, r.g, true);
            const int n = min(tile_tok0(j) + l32, N - 1);
            r.l = lb[n];
            r.d = db[n];
        };
        Rows ra, rb, rc;
        bf16x8 kT[HV][2];
        float wrow[ONE ? 16 : 1];
        request(0, ra);
        request(1, rb);
        request(2, rc);
        compiler_fence();
        write_kt(ra.k, lds);
        if constexpr (ONE) wl[0][l32] = fast_exp2(kap - ra.l * ld_mul);
        compiler_fence();
        read_kT(lds, kT);
        if constexpr (ONE) read_w(wl[0], wrow);

        // tile j: cur holds its rows (and receives those of tile j+3 at the end), nxt those of tile j+1
        auto tile = [&](int j, Rows &cur, const Rows &nxt) {
            const int tok0 = tile_tok0(j);
            uint16_t *buf_next = lds + ((j + 1) & 1) * BUF;
            const float nld = -cur.l * ld_mul, dl = cur.d;
            bf16x8 vt[KS], gt[KS];   // V and dY meet bf16 operands
#pragma unroll
            for (int s = 0; s < KS; ++s) { vt[s] = v_operand(cur.v[s]); gt[s] = to_bf16(cur.g[s]); }

            // token-side operands of the correction k-steps (zero outside the named slots)
            u32x4 wb;
            wb[0] = 0u; wb[2] = 0u; wb[3] = 0u;
            wb[1] = lower ? split_pair<F>(nld) : 0u;             // slots 2,3 := -lse_dec2[n]
            const bf16x8 kt_a = ones_s, kt_b = as_bf16x8(wb);    // slots 0,1 := 1 picks -lse_enc2
            // One exponential (d >= 16): dS = P (a + w c) and w[n] is this lane's token's, so ONE product serves
            // both corrections: slots 0,1,2 = -w delta (hi, lo, hi) meet u (hi, hi, lo) and slots 4,5 = 1 pick
            // -eps; the a chain starts from it and the c chain from zero.
            constexpr bool MERGED = ONE && !PACK;
            u32x4 wg;
            const uint32_t ds_ = split_bf16_pair(MERGED ? -dl * fast_exp2(kap + nld) : -dl);
            wg[0] = lower ? ds_ : 0u;
            wg[1] = (ONE && lower) ? (ds_ & 0xffffu) : 0u;       // ONE: slots 0,1,2 := -delta hi, lo, hi
            wg[2] = (MERGED && lower) ? 0x3f803f80u : 0u;
            wg[3] = 0u;
            const bf16x8 g_aug = as_bf16x8(wg);

            const int rem = n1 - tok0 - 4 * hh;
            const bool partial = tok0 + 32 > n1;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                f32x16 x = splat16(0.f);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) x = mfma_s<F>(cur.k[ks], qh[b][ks], x);
                if constexpr (!PACK) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) x = mfma_s<F>(cur.k[ks], ql[b][ks], x);
                }
                f32x16 s1 = x;                  // one exponential: the scores as they are
                if constexpr (!ONE) s1 = mfma_s<F>(kt_a, q_aug[b], x);
                f32x16 s2 = s1;
                if constexpr (!ONE) s2 = mfma_s<F>(kt_b, q_aug[b], x);
                f32x16 av = splat16(0.f), cv = splat16(0.f);
                if constexpr (MERGED) {
                    av = mfma(g_aug, u_aug[ONE ? b : 0], av);
                } else {
                    if constexpr (!PACK) av = mfma(ones_aug, dz_aug[b], av);
                    cv = mfma(g_aug, ONE ? u_aug[ONE ? b : 0] : ones_aug, cv);
                }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    av = mfma(vt[ks], dzb[b][ks], av);
                    cv = mfma(gt[ks], zb[b][ks], cv);
                    if constexpr (LO2 && !PACK) cv = mfma(gt[ks], zl[b][ks], cv);
                }
                if (partial) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (8 * (r / 4) + (r % 4) >= rem) { s1[r] = -INFINITY; s2[r] = -INFINITY; }
                }
                f32x16 ds;
                if constexpr (ONE) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) ds[i] = fast_exp2(s1[i]) * fmaf(cv[i], wrow[i], av[i]);
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) ds[i] = fmaf(fast_exp2(s2[i]), cv[i], fast_exp2(s1[i]) * av[i]);
                }
                u32x4 w0, w1;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    w0[i] = cvt_pk_bf16(ds[2 * i], ds[2 * i + 1]);
                    w1[i] = cvt_pk_bf16(ds[8 + 2 * i], ds[8 + 2 * i + 1]);
                }
#pragma unroll
                for (int hv = 0; hv < HV; ++hv) {
                    acc[b][hv] = mfma(kT[hv][0], as_bf16x8(w0), acc[b][hv]);
                    acc[b][hv] = mfma(kT[hv][1], as_bf16x8(w1), acc[b][hv]);
                }
            }
            // The next tile's K^T and w go through LDS here, at the end of the tile: its rows were requested two
            // tiles ago, and what is read back is first needed by the last products of the next tile.
            compiler_fence();
            write_kt(nxt.k, buf_next);
            if constexpr (ONE) wl[(j + 1) & 1][l32] = fast_exp2(kap - nxt.l * ld_mul);
            compiler_fence();
            request(j + 3, cur);
            read_kT(buf_next, kT);
            if constexpr (ONE) read_w(wl[(j + 1) & 1], wrow);
            sched_fence();   // consecutive tiles are not interleaved (their temporaries would not fit the registers)
        };
        int j = 0;
        for (; j + 3 <= cnt; j += 3) {
            tile(j, ra, rb);
            tile(j + 1, rb, rc);
            tile(j + 2, rc, ra);
        }
        if (j < cnt) {
            tile(j, ra, rb);
            if (j + 1 < cnt) tile(j + 1, rb, rc);
        }
    }

    const size_t part = (size_t)bh * parts + (size_t)chunk * TG + tg;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (lat0 + 32 * b + l32 >= M) continue;
        const size_t slot = part * M + lat0 + 32 * b + l32;
#pragma unroll
        for (int hv = 0; hv < HV; ++hv)
#pragma unroll
            for (int qd = 0; qd < QUARTS; ++qd) {
                const int o = 16 * hv + 8 * qd + 4 * hh;
                if (o >= DR) continue;
                *reinterpret_cast<float4 *>(dq_part + slot * DR + o) = make_float4(
                    acc[b][hv][4 * qd], acc[b][hv][4 * qd + 1], acc[b][hv][4 * qd + 2], acc[b][hv][4 * qd + 3]);
            }
    }
}

// Both variants in one launch: each workgroup takes the one that the plan names for its (b,h) (a second launch whose
// workgroups all leave at once would still cost 4-6 us).  The two bodies share the kernel's registers; their LDS adds up.
template <int DR, int NB, int MINB, bool F>
__global__ __launch_bounds__(256, MINB) void bwd_dq_mfma_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const bf16_t *__restrict__ dy, const float *__restrict__ z, const float *__restrict__ lse_enc,
    const float *__restrict__ dz, const float *__restrict__ eps, const float *__restrict__ lse_dec2,
    const float *__restrict__ delta, float ld_mul, const int *__restrict__ plan, float *__restrict__ dq_part,
    TokStride ts, int H, int N, int M, int chunk_len, int parts, int G, int TG, float c2)
{
    const int bh = grid_pos(ts, H, DR * 2).y;
    if (plan[bh] != 0)
        dq_body<DR, NB, MINB, true, F>(q, k, v, dy, z, lse_enc, dz, eps, lse_dec2, delta, ld_mul, plan, dq_part, ts, H, N,
                                       M, chunk_len, parts, G, TG, c2);
    else
        dq_body<DR, NB, MINB, false, F>(q, k, v, dy, z, lse_enc, dz, eps, lse_dec2, delta, ld_mul, plan, dq_part, ts, H, N,
                                        M, chunk_len, parts, G, TG, c2);
}

// ============================================================================================
// Backward, dK and dV (token-major, like the decode: one wave owns 32 tokens at a time and walks
// over all latent tiles).  Everything that depends on the latents only is prepared once per
// workgroup as MFMA-ready operand images in LDS (one (b,h) per workgroup, 8 waves share it):
//   A-type images (row = latent, contraction over d): q' hi, q' lo, dZ hi (and lo), Z hi (and
//     lo), and a correction operand (slots 0,1 = -lse_enc2 as a hi+lo pair, slots 2,3 = 1,1; slots
//     8,9 = -eps as a hi+lo pair; slots 10,11 = 1,1 or, with one exponential, slots 4-6 = u: they
//     pick -delta[n] out of the token-side operand of the c chain's correction k-step);
//   row images (row = output column, contraction over the 32 latents in accumulator order):
//     RW1 = [dZ^T ; 0]   and   RW2 = [q^T ; 0]   (d = 32: all 32 rows are columns of dZ and q).
// Per token tile and latent tile:  P = 2^(S2 - lse_enc2[m]), R = 2^(S2 - lse_dec2[n]),
//   a = <dZ_m, V_n> - eps[m],  c = <Z_m, dY_n> - delta[n],  dS = P a + R c  (fp32), then
//   acc1 += RW1 . P   (rows 0-15: dV^T)
//   acc2 += RW2 . dS  (rows 0-15: (sum_m dS q_m)^T)
// and at the end  dV = acc1[0:16],  dK = scale * acc2[0:16].
// (eps is subtracted inside the a chain, by one more product, so that a - eps = <dZ_m, V_n - Z_m>
// cancels before dS is rounded: where a latent attends sharply to tokens of similar values the two
// terms agree to several digits, and carrying -eps q separately through bf16 roundings lost them.)
// No lo terms of dZ and Z for dK and dV: dZ arrives bf16-exact, and the rounding of Z_m is one error per
// latent, which the sums of dK_n and dV_n over the latents average out (measured: dK error up by
// 5-10 %, time down by 9 %) -- unlike in dQ, whose sums run over the tokens of one latent and add that
// error up coherently (the DQ variant below therefore carries the lo term of Z at d <= 8, and at d = 16 where the
// shape calls for it: ZL).
// ONE: one exponential per score, as in the dQ kernel: R = P u[m] w[n]; u is folded into the Z images
// (and into slots 4-6 of the correction image, against -delta in the token operand), w[n] is a
// per-lane scalar here, and dS' = P (a + w c).  Runs only where plan[bh] = 1.
// ============================================================================================
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kDsStride = 36;   // uint16 per row of the dS tile [token][latent] (72 B: conflict-free 8-byte stores)
constexpr int kKtStride = 16;   // uint16 per row of the key tile [token][d] of the fused dQ product (rows as loaded)
constexpr int kFusedWaveLds = 32 * kDsStride + 32 * kKtStride;   // uint16 per wave: dS tile, then the key tile

// WV: waves per workgroup (one workgroup per CU).  Eight, or twelve where the kernel fits 168 registers (three waves
// per SIMD): d = 32 with one exponential.
template <int DR, int MT, bool DQ, bool ONE, bool F, int WV = 8, bool ZL = false>
__device__ __forceinline__ void dkdv_body(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const bf16_t *__restrict__ dy, const float *__restrict__ z, const float *__restrict__ lse_enc,
    const float *__restrict__ dz, const float *__restrict__ eps, const float *__restrict__ lse_dec2,
    const float *__restrict__ delta, float ld_mul, const int *__restrict__ plan, bf16_t *__restrict__ dk,
    bf16_t *__restrict__ dv, float *__restrict__ acc32, float *__restrict__ dq_part, TokStride ts, int H, int N,
    int Mtot, int m0, float c2, float scale)
{
    // DQ (d <= 16): the kernel also forms the dQ partials, so that the scores, a, c and dS of a tile
    // pair are computed once for all three gradients.  dS of a tile reaches the dQ product transposed
    // (contraction over the tokens) through a wave-private LDS tile, and that product is
    //     dQ^T[dd][m] += K^T[dd][n] dS^T[n][m]     with v_mfma_f32_16x16x32_bf16
    // (16 output rows = d: no wasted rows, four accumulator registers per 16 latents), so a wave keeps
    // dQ of all 32*MT latents in 8*MT registers.  At the end the eight waves add their partials in a
    // fixed order through LDS and the workgroup writes slot x (its grid position) of dq_part
    // ([(b*h) * gridDim.x + x][Mtot][d], summed and scaled by dq_reduce_kernel).  The c chain
    // then carries the lo term of Z at d <= 8 (ZPACK below) and, with ZL, at d = 16 (dQ sums dS over the tokens of
    // one latent and adds up its rounding coherently, see the dQ kernel).
    // The kernel works on the latents m0 .. m0 + M of the head's Mtot.  With acc32 given (more than one
    // latent chunk) it adds its dV and dK rows in fp32 to acc32[0][b*h][n][DR] and acc32[1][...] (the
    // chunk with m0 = 0 stores instead); the last chunk adds what is there to its own rows and rounds the
    // sums to dk and dv.  The chunks run as launches in a row on one stream, so the order of the sum is fixed.
    constexpr int D = padded_dim(DR);
    constexpr int KS = D / 16;
    // Row blocks of the two accumulations.  d <= 16: one 32x32 product per 16 columns (rows 16-31 of its
    // operand image are zero).  d = 32: the 32 columns fill the 32 rows of ONE product (WIDE), half the
    // matrix instructions of two half-empty ones.
    constexpr bool WIDE = (D == 32);
    constexpr int HV = WIDE ? 1 : D / 16;
    constexpr int QUARTS = WIDE ? 4 : 2;        // 4-column pieces per lane and accumulator: columns 8 q + 4 hh (+ 16 hv)
    static_assert(!DQ || DR <= 16, "the fused dQ product is written for d <= 16 (16 output rows)");
    // ZL (DQ at d = 16, shapes with fewer tokens than latents): the c chain carries the lo term of Z as one more image
    // and product (at d <= 8 it rides in the free upper half of the Z image, ZPACK below).  dQ sums dS over the tokens
    // of one latent, so the rounding of Z_m adds up coherently there, and on rows whose halves cancel it shows:
    // mesh-like inputs, 692 latents over 242 tokens, dq_lat 2.4e-2 without it, 1.1e-2 with it (1539 over 427: 2.5e-2
    // and 7e-3).  It costs 5 % of the kernel's time; of the random shapes with at least as many tokens as latents one
    // in 30 000 left the bar, and that one for another reason (delta from the saved bf16 y), the lo term or not.
    constexpr bool ZLO = DQ && !pack_dim(DR) && ZL;
    static_assert(!ZL || (DQ && !pack_dim(DR)), "the extra image is for the fused dQ product at d = 16");
    constexpr int NA = (ZLO ? 5 : 4) * KS + 1;  // A-type images per latent tile (the last one: corrections)
    constexpr int NR = 4 * HV;                  // row images per latent tile (RW1, RW2) x 2 k-steps
    constexpr int PER_TILE = NA + NR;
    constexpr bool PIPE = (D == 16);            // look one latent tile ahead where registers allow
    // d <= 8: the upper half of the padded contraction carries what otherwise needs products of its own.
    // Images: q' hi | lo in one (keys repeated in both lane halves), slots 8,9 of the dZ image = -eps
    // (against ones in the V operand), slots 8-10 of the Z image = u, u, u lo or 1, 1 (against -delta in
    // the dY operand).  The q' lo image and the a / c parts of the correction image are then unused.
    constexpr bool PACK = pack_dim(DR);
    // PACK with DQ: the upper half of the Z image carries the lo term of Z instead (dY rows repeated in both
    // lane halves), as the separate dQ kernel has it at d <= 8, and -delta comes in through the correction
    // image as at d = 16: dQ sums dS over the tokens of one latent, and with so few terms per dot product
    // the rounding of Z_m showed (9.7e-3 against 2.6e-3 on a 1500-token case).  The delta it subtracts
    // comes from rows of Y formed with the same hi + lo pair (the token-statistics kernel at d <= 8), so
    // c - delta cancels where one latent dominates a token, down to a single latent.
    constexpr bool ZPACK = PACK && DQ;
    extern __shared__ __attribute__((aligned(16))) u32x4 img[];   // [MT][PER_TILE][64 lanes]

    const int tid = threadIdx.x;
    const int lane = tid & 63, l32 = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // known to be wave-uniform: scalar unit
    const GridPos gp = grid_pos(ts, H, DR * 2);
    const int bh = gp.y, h = bh % H;
    const bool lower = hh == 0;
    if ((plan[bh] != 0) != ONE) return;         // the other variant owns this (b,h); uniform over the workgroup
    constexpr float kap = 0.f;                  // w[n] = 2^(kap - lse_dec2[n])

    // ---- build the operand images ----
    {
        const bf16_t *qh_ = q + (size_t)h * ts.sq + (size_t)m0 * DR;
        const float *zb = z + ((size_t)bh * Mtot + m0) * DR;
        const float *dzb = dz + ((size_t)bh * Mtot + m0) * DR;
        const float *eb = eps + (size_t)bh * Mtot + m0;
        const float *leb = lse_enc + (size_t)bh * Mtot + m0;
        // Padding latents (at or beyond Mtot; mleft = real ones from m0 on): loads are clamped to the last
        // real latent and every value that could reach dK or dV is zero -- q, Z, dZ, eps, u and the ones
        // that pick -delta -- so that a = c = 0 and dS = 0 whatever P and R come out as.
        const int mleft = Mtot - m0;
        for (int idx = tid; idx < MT * PER_TILE * 64; idx += 64 * WV) {
            const int ln = idx & 63, sid = (idx >> 6) % PER_TILE, t = (idx >> 6) / PER_TILE;
            const int r32 = ln & 31, hf = ln >> 5;
            u32x4 w;
            if (sid == NA - 1) {
                // correction operand: slots 0,1 = -lse_enc2 (hi + lo pair), slots 2,3 = 1, else zero
                const bool real = 32 * t + r32 < mleft;
                const int mc = min(32 * t + r32, mleft - 1);
                const float le2 = real ? leb[mc] * kLog2e : 0.f;
                w[0] = hf == 0 ? split_pair<F>(-le2) : 0u;
                w[1] = hf == 0 ? kOnePair<F> : 0u;
                w[2] = 0u; w[3] = 0u;
                // Slots 4-6 belong to the c product and slots 8,9 to the a product, whose operands are bf16
                // whatever the storage type; the score products meet them with zeros in the token operand
                // (and the a and c products meet slots 0-3 with zeros).  u <= 1 and finite 16-bit patterns of either type read as finite values
                // of the other, so the foreign slots contribute exact zeros.
                if constexpr (ONE) {   // slots 4,5,6 := u hi, u hi, u lo
                    const uint32_t us = split_bf16_pair(real ? 1.f : 0.f);   // (the latent's factor of the c chain: 1)
                    w[2] = hf == 0 ? ((us & 0xffffu) | (us << 16)) : 0u;
                    w[3] = hf == 0 ? (us >> 16) : 0u;
                }
                if (hf == 1) {
                    w[0] = split_bf16_pair(real ? -eb[mc] : 0.f);          // slots 8,9 := -eps (bf16: the a chain)
                    if (!ONE && real) w[1] = 0x3f803f80u;                  // slots 10,11 := 1 (picks -delta, two exponentials)
                }
            } else if (sid < NA) {
                const int kind = sid / KS, ks = sid % KS;          // 0 q' hi, 1 q' lo, 2 dZ, 3 Z hi, 4 Z lo (DQ only)
                const bool real = 32 * t + r32 < mleft;
                const int m = min(32 * t + r32, mleft - 1);
                const int d0 = (D / 2) * hf + 8 * ks;
                float x[8];
                if (kind <= 1) {
                    const u32x4 raw = row8_bf16<DR>(qh_ + (size_t)m * DR, PACK ? 0 : d0);
#pragma unroll
                    for (int i = 0; i < 4; ++i) { x[2 * i] = elem_lo<F>(raw[i]) * c2; x[2 * i + 1] = elem_hi<F>(raw[i]) * c2; }
                } else {
                    const bool is_z = kind >= 3;
                    row8_f32<DR>((is_z ? zb : dzb) + (size_t)m * DR, (ZPACK && is_z) ? 0 : d0, x);
                }
                if (!real) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) x[i] = 0.f;
                }
                const bool want_lo = (kind == 1 || kind >= 4 || (PACK && kind == 0 && hf == 1) ||
                                      (ZPACK && kind == 3 && hf == 1));
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint32_t a, b;
                    if (kind <= 1) {   // q' feeds the score products: storage type
                        a = rne_elem<F>(x[2 * i]); b = rne_elem<F>(x[2 * i + 1]);
                        if (want_lo) {
                            a = rne_elem<F>(x[2 * i] - elem_value<F>(a));
                            b = rne_elem<F>(x[2 * i + 1] - elem_value<F>(b));
                        }
                    } else {
                        a = rne_bf16(x[2 * i]); b = rne_bf16(x[2 * i + 1]);
                        if (want_lo) {
                            a = rne_bf16(x[2 * i] - __uint_as_float(a << 16));
                            b = rne_bf16(x[2 * i + 1] - __uint_as_float(b << 16));
                        }
                    }
                    w[i] = a | (b << 16);
                }
                if constexpr (DR == 4 && !ZPACK) {   // slots 4-7 of the Z image := its lo part (dY repeated there)
                    if (kind == 3 && hf == 0) {
#pragma unroll
                        for (int i = 0; i < 2; ++i) {
                            const uint32_t a = rne_bf16(x[2 * i] - __uint_as_float(w[i] << 16));
                            const uint32_t b = rne_bf16(x[2 * i + 1] - __uint_as_float(w[i] & 0xffff0000u));
                            w[2 + i] = a | (b << 16);
                        }
                    }
                }
                if (PACK && hf == 1 && kind == 2 && real) w[0] = split_bf16_pair(-eb[m]);   // slots 8,9 := -eps
                if (PACK && !ZPACK && hf == 1 && kind == 3 && real) {                // slots 8,9,10 := u, u, u lo / 1, 1
                    if constexpr (ONE) {
                        const uint32_t us = split_bf16_pair(1.f);
                        w[0] = (us & 0xffffu) | (us << 16);
                        w[1] = us >> 16;
                    } else {
                        w[0] = 0x3f803f80u;
                    }
                }
            } else {
                const int rsid = sid - NA;                          // (which, hv, s2)
                const int which = rsid / (2 * HV), hv = (rsid / 2) % HV, s2 = rsid % 2;
                const int dd = WIDE ? r32 : 16 * hv + (r32 & 15);
                const bool row_live = WIDE || r32 < 16;
#pragma unroll
                for (int i = 0; i < 8; i += 2) {
                    float a, b;
                    const int ma = 32 * t + perm_index(s2, hf, i), mb = 32 * t + perm_index(s2, hf, i + 1);
                    const bool in = dd < DR;   // beyond the real head dimension every row image is zero
                    const bool ina = in && ma < mleft, inb = in && mb < mleft;
                    const float q0 = ina ? elem_value<F>(qh_[(size_t)ma * DR + dd]) : 0.f;
                    const float q1 = inb ? elem_value<F>(qh_[(size_t)mb * DR + dd]) : 0.f;
                    if (which == 0) {
                        a = (row_live && ina) ? dzb[(size_t)ma * DR + dd] : 0.f;
                        b = (row_live && inb) ? dzb[(size_t)mb * DR + dd] : 0.f;
                    } else {
                        a = row_live ? q0 : 0.f;
                        b = row_live ? q1 : 0.f;
                    }
                    w[i / 2] = rne_bf16(a) | (rne_bf16(b) << 16);
                }
            }
            img[idx] = w;
        }
    }
    __syncthreads();

    u32x4 w11;
    w11[1] = 0u; w11[2] = 0u; w11[3] = 0u;
    w11[0] = lower ? kOnePair<F> : 0u;
    const bf16x8 ones_s = as_bf16x8(w11);        // the same in the type of the score products
    w11[0] = lower ? 0u : 0x3f803f80u;
    const bf16x8 ones_eps = as_bf16x8(w11);      // slots 8,9 = 1 (bf16): picks -eps out of the correction image
    auto to_bf16 = [](bf16x8 x) { return as_bf16x8(to_bf16_row<F>(__builtin_bit_cast(u32x4, x))); };

    const bf16_t *kb = k + tok_base(ts, bh, H);
    const bf16_t *vb = v + tok_base(ts, bh, H);
    const bf16_t *gb = dy + tok_base(ts, bh, H);
    const float *lb = lse_dec2 + (size_t)bh * N;
    const float *db = delta + (size_t)bh * N;
    const int tiles = (N + 31) / 32;
    static_assert(!DQ || WV == 8, "the fused dQ reduction is written for eight waves");
    const int stride = gridDim.x * WV;
    // B operand: column = token.  rep (PACK only): both lane halves get elements 0-7 of the row.
    auto load_cols = [&](const bf16_t *base, int tile, bf16x8 (&t)[KS], bool rep) {
        const int n = min(tile * 32 + l32, N - 1);
#pragma unroll
        for (int s = 0; s < KS; ++s)
            t[s] = as_bf16x8(row8_bf16<DR>(base + tok_off(ts, n), (PACK && rep) ? 0 : (D / 2) * hh + 8 * s));
    };
    // V rows as the operand of the a product; PACK: slots 8,9 := 1 (the upper lane half loaded zeros)
    auto v_operand = [&](bf16x8 x) {
        u32x4 w = to_bf16_row<F>(__builtin_bit_cast(u32x4, x));
        if (PACK && !lower) w[0] = 0x3f803f80u;
        return as_bf16x8(w);
    };
    auto image = [&](int t, int sid) { return as_bf16x8(img[(t * PER_TILE + sid) * 64 + lane]); };

    // fused dQ: wave-private LDS tiles and the accumulators dQ^T[dd = 4 (lane / 16) + r][m = 32 t + 16 jb + lane % 16]
    uint16_t *ds_t = reinterpret_cast<uint16_t *>(img + MT * PER_TILE * 64) + (DQ ? wave * kFusedWaveLds : 0);
    uint16_t *k_t = ds_t + 32 * kDsStride;
    if constexpr (DQ && PACK) {   // columns 8-15 of the key tile are never written at d <= 8: zero (the output rows 8-15 are dropped)
        if (lane < 32) *reinterpret_cast<u32x4 *>(k_t + lane * kKtStride + 8) = u32x4{0u, 0u, 0u, 0u};
    }
    f32x4 dqa[DQ ? MT : 1][2];
#pragma unroll
    for (int t = 0; t < (DQ ? MT : 1); ++t)
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) dqa[t][jb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int c16 = lane & 15, g16 = lane >> 4;

    int tile = gp.x * WV + wave;
    bf16x8 kt[KS], vt[KS], gt[KS], ktn[KS], vtn[KS], gtn[KS];
    if (tile < tiles) {
        load_cols(kb, tile, kt, true);
        load_cols(vb, tile, vt, false);
        load_cols(gb, tile, gt, ZPACK);
#pragma unroll
        for (int s = 0; s < KS; ++s) { vt[s] = v_operand(vt[s]); gt[s] = to_bf16(gt[s]); }
    }
    // The token statistics (lse_dec2, delta) are requested one tile ahead like the rows: a request made where its
    // value is needed would also wait for the rows requested just before it (loads complete in order), and every
    // token tile would begin with a full memory latency.
    float lse_next = 0.f, delta_next = 0.f;
    if (tile < tiles) {
        const size_t row0 = (size_t)min(tile * 32 + l32, N - 1);
        lse_next = lb[row0];
        delta_next = db[row0];
    }
    // (the first tile's rows and statistics have arrived before the loop starts: inside it, nothing waits for
    // anything but what the loop itself requested a tile earlier)
    float nld_cur = pinned(-lse_next * ld_mul), dl_cur = pinned(delta_next);
#pragma unroll
    for (int s = 0; s < KS; ++s) { kt[s] = pinned(kt[s]); vt[s] = pinned(vt[s]); gt[s] = pinned(gt[s]); }
    for (; tile < tiles; tile += stride) {
        const int n = tile * 32 + l32;
        const int tn = (tile + stride < tiles) ? tile + stride : tile;
        load_cols(kb, tn, ktn, true);
        load_cols(vb, tn, vtn, false);
        load_cols(gb, tn, gtn, ZPACK);
        const float nld = nld_cur, dl = dl_cur;
        {
            const size_t rown = (size_t)min(tn * 32 + l32, N - 1);
            lse_next = lb[rown];
            delta_next = db[rown];
        }
        const float wn = ONE ? fast_exp2(kap + nld) : 0.f;

        u32x4 wb;
        wb[0] = 0u; wb[2] = 0u; wb[3] = 0u;
        wb[1] = lower ? split_pair<F>(nld) : 0u;             // slots 2,3 := -lse_dec2[n]
        const bf16x8 kt_a = ones_s, kt_b = as_bf16x8(wb);    // slots 0,1 := 1 picks -lse_enc2
        // Token side of the correction k-step(s).  Two exponentials: g_aug picks -delta for the c chain
        // (slots 10,11 against the image's ones) and ones_eps picks -eps for the a chain.  One exponential:
        // dS = P (a + w c), and w[n] is this lane's scalar, so ONE product serves both chains: slots 8,9 = 1
        // pick -eps and slots 4,5,6 = -w delta (hi, lo, hi) meet u (hi, hi, lo); the a chain starts from
        // it and the c chain from zero.
        u32x4 wg;
        const uint32_t ds_ = split_bf16_pair(ONE ? -dl * wn : -dl);
        wg[0] = (ONE && !lower && !PACK) ? 0x3f803f80u : 0u;
        wg[1] = (!ONE && !lower) ? ds_ : 0u;                 // two exponentials: slots 10,11 := -delta (hi, lo)
        wg[2] = (ONE && lower) ? ds_ : 0u;                   // one: slots 4,5,6 := -w delta hi, lo, hi
        wg[3] = (ONE && lower) ? (ds_ & 0xffffu) : 0u;
        const bf16x8 g_aug = as_bf16x8(wg);
        bf16x8 gc[KS];   // dY operand of the c product; PACK: slots 8,9,10 := -delta hi, lo, hi
#pragma unroll
        for (int s = 0; s < KS; ++s) gc[s] = gt[s];
        if constexpr (PACK && !ZPACK) {
            u32x4 w = __builtin_bit_cast(u32x4, gt[0]);
            const uint32_t dp_ = split_bf16_pair(-dl);   // here c keeps its own correction: -delta unscaled
            if (!lower) { w[0] = dp_; w[1] = ONE ? (dp_ & 0xffffu) : 0u; }
            if (DR == 4 && lower) { w[2] = w[0]; w[3] = w[1]; }   // against the lo part of Z in slots 4-7
            gc[0] = as_bf16x8(w);
        }

        f32x16 acc1[HV], acc2[HV];
#pragma unroll
        for (int hv = 0; hv < HV; ++hv) { acc1[hv] = splat16(0.f); acc2[hv] = splat16(0.f); }

        // fused dQ: K^T of this token tile as the A operand of the 16x16x32 product (row = dd = lane % 16,
        // tokens 8 (lane / 16) .. + 7), through the wave's LDS tile; rows of tokens past N are zero
        bf16x8 k_op = zero_operand();
        if constexpr (DQ) {
            const u32x4 w = (n < N) ? to_bf16_row<F>(__builtin_bit_cast(u32x4, kt[0])) : __builtin_bit_cast(u32x4, zero_operand());
            // the tile as loaded, row = token (one 16-byte store per lane); the transposing read hands lane c16 of block
            // g16 column c16 of the rows 8 g16 .. + 3 (second read: + 4 .. + 7), as for the dS tile below
            if (!(PACK && hh))     // d <= 8: the upper lane half holds a copy of the same elements
                *reinterpret_cast<u32x4 *>(k_t + l32 * kKtStride + 8 * hh) = w;
            compiler_fence();
            const uint16_t *src = k_t + (8 * g16 + c16 / 4) * kKtStride + 4 * (c16 % 4);
            const u32x2 lo2 = lds_read_tr16(src), hi2 = lds_read_tr16(src + 4 * kKtStride);
            u32x4 ka;
            ka[0] = lo2[0]; ka[1] = lo2[1]; ka[2] = hi2[0]; ka[3] = hi2[1];
            k_op = as_bf16x8(ka);
        }

        // Score products of latent tile t (minus lse_enc2 / minus lse_dec2): 2*KS + 2 MFMAs.
        auto scores = [&](int t, f32x16 &s1, f32x16 &s2) {
            f32x16 x = splat16(0.f);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) x = mfma_s<F>(image(t, 0 * KS + ks), kt[ks], x);
            if constexpr (!PACK) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) x = mfma_s<F>(image(t, 1 * KS + ks), kt[ks], x);
            }
            if constexpr (ONE) {
                s1 = x;                         // one exponential: the scores as they are
            } else {
                const bf16x8 qa = image(t, NA - 1);
                s1 = mfma_s<F>(qa, kt_a, x);
                s2 = mfma_s<F>(qa, kt_b, x);
            }
        };
        // One latent tile, software-pipelined: the a and c products of tile t and the score products
        // of tile t+1 are issued first and run on the matrix cores while the vector ALUs
        // exponentiate the scores of tile t (s1, s2, computed one step earlier).
        auto tile_step = [&](int t, f32x16 &s1, f32x16 &s2, f32x16 &s1n, f32x16 &s2n) {
            // The wave takes issue priority over its SIMD's other wave while it feeds the matrix cores (the a and
            // c products, the next tile's scores) and drops it for the vector block: the matrix pipe starts
            // at once and the other wave's vector instructions fill the gaps (measured -4.5 % at d = 16, -2 to
            // -6 % at the other shapes; holding the priority over the accumulation products as well was
            // slower, and the same switch in the encode kernel changed nothing, in the dQ kernel it cost 5 %).
            __builtin_amdgcn_s_setprio(1);
            if constexpr (!PIPE) scores(t, s1, s2);   // not enough registers at d = 32: no look-ahead
            f32x16 av = splat16(0.f), cv = splat16(0.f);
            if constexpr (ONE) {
                if constexpr (!PACK || ZPACK) av = mfma(image(t, NA - 1), g_aug, av);
            } else {
                if constexpr (!PACK) av = mfma(image(t, NA - 1), ones_eps, av);
                if constexpr (!PACK || ZPACK) cv = mfma(image(t, NA - 1), g_aug, cv);
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                av = mfma(image(t, 2 * KS + ks), vt[ks], av);
                cv = mfma(image(t, 3 * KS + ks), gc[ks], cv);
                if constexpr (ZLO) cv = mfma(image(t, 4 * KS + ks), gc[ks], cv);
            }
            if constexpr (PIPE) {
                if (t + 1 < MT) scores(t + 1, s1n, s2n);
            }
            bf16x8 rw[NR];
#pragma unroll
            for (int r = 0; r < NR; ++r) rw[r] = image(t, NA + r);
            sched_fence();
            __builtin_amdgcn_s_setprio(0);
            f32x16 pv, rv;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                pv[i] = fast_exp2(s1[i]);
                if constexpr (ONE) rv[i] = pv[i] * fmaf(cv[i], wn, av[i]);     // dS' = P (a + w[n] u[m] c)
                else rv[i] = fmaf(fast_exp2(s2[i]), cv[i], pv[i] * av[i]);     // dS' = P a + R c
            }
            u32x4 p0, p1, d0, d1;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                p0[i] = cvt_pk_bf16(pv[2 * i], pv[2 * i + 1]);
                p1[i] = cvt_pk_bf16(pv[8 + 2 * i], pv[8 + 2 * i + 1]);
                d0[i] = cvt_pk_bf16(rv[2 * i], rv[2 * i + 1]);
                d1[i] = cvt_pk_bf16(rv[8 + 2 * i], rv[8 + 2 * i + 1]);
            }
#pragma unroll
            for (int hv = 0; hv < HV; ++hv) {
                acc1[hv] = mfma(rw[(0 * HV + hv) * 2 + 0], as_bf16x8(p0), acc1[hv]);
                acc1[hv] = mfma(rw[(0 * HV + hv) * 2 + 1], as_bf16x8(p1), acc1[hv]);
                acc2[hv] = mfma(rw[(1 * HV + hv) * 2 + 0], as_bf16x8(d0), acc2[hv]);
                acc2[hv] = mfma(rw[(1 * HV + hv) * 2 + 1], as_bf16x8(d1), acc2[hv]);
            }
            if constexpr (DQ) {
                // dS (this lane: token l32, latents 8 (r/4) + 4 hh + r%4 for r = 0..15) -> LDS as it is, row = token:
                // four 8-byte stores of four latents each.  The product wants it the other way round (column =
                // latent, 8 consecutive tokens per lane): four transposing reads, each four tokens of one latent.
                uint16_t *drow = ds_t + l32 * kDsStride + 4 * hh;
                *reinterpret_cast<u32x2 *>(drow) = u32x2{d0[0], d0[1]};
                *reinterpret_cast<u32x2 *>(drow + 8) = u32x2{d0[2], d0[3]};
                *reinterpret_cast<u32x2 *>(drow + 16) = u32x2{d1[0], d1[1]};
                *reinterpret_cast<u32x2 *>(drow + 24) = u32x2{d1[2], d1[3]};
                compiler_fence();
#pragma unroll
                for (int jb = 0; jb < 2; ++jb) {
                    // lane c16 of block g16: chunk row = token 8 g16 (+ 4) + c16 / 4, piece = latents 16 jb + 4 (c16 % 4)
                    const uint16_t *src = ds_t + (8 * g16 + c16 / 4) * kDsStride + 16 * jb + 4 * (c16 % 4);
                    const u32x2 b_lo = lds_read_tr16(src), b_hi = lds_read_tr16(src + 4 * kDsStride);
                    const u32x4 bop = u32x4{b_lo[0], b_lo[1], b_hi[0], b_hi[1]};
                    dqa[t][jb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k_op, as_bf16x8(bop), dqa[t][jb], 0, 0, 0);
                }
                compiler_fence();
            }
            // (the fused one-exponential kernel of d = 16 is 0.6 % faster without this fence between its latent tiles)
            if constexpr (!(DQ && ONE && D == 16)) sched_fence();
        };
        {
            f32x16 sa1 = splat16(0.f), sa2 = splat16(0.f), sb1 = splat16(0.f), sb2 = splat16(0.f);
            if constexpr (PIPE) scores(0, sa1, sa2);
            if constexpr (MT == 1) {
                tile_step(0, sa1, sa2, sb1, sb2);
            } else if constexpr (DQ) {   // unrolled: the dQ accumulators are indexed by the latent tile
#pragma unroll
                for (int t = 0; t < MT; t += 2) {
                    tile_step(t, sa1, sa2, sb1, sb2);
                    tile_step(t + 1, sb1, sb2, sa1, sa2);
                }
            } else {
#pragma unroll 1
                for (int t = 0; t < MT; t += 2) {
                    tile_step(t, sa1, sa2, sb1, sb2);
                    tile_step(t + 1, sb1, sb2, sa1, sa2);
                }
            }
        }
        // What was requested at the top of this tile is taken over here, ahead of the tile's stores: memory
        // operations complete in order, so taking it over after them (at the top of the next tile) would make the
        // wave wait for its own stores once per tile.
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            kt[s] = pinned(ktn[s]);
            vt[s] = pinned(v_operand(vtn[s]));
            gt[s] = pinned(to_bf16(gtn[s]));
        }
        nld_cur = pinned(-lse_next * ld_mul);
        dl_cur = pinned(delta_next);
        compiler_fence();
        // registers 4 q .. 4 q + 3 of an accumulator: columns (16 hv +) 8 q + 4 hh .. + 3 of this lane's token
        // More than one latent chunk: all but the first add what the chunks before them left in acc32, and all but
        // the head's last one leave their sums there; the last one rounds and stores them like a single chunk.
        const bool from_acc = acc32 != nullptr && m0 != 0;
        const bool to_acc = acc32 != nullptr && m0 + 32 * MT < Mtot;
        if (n < N) {
#pragma unroll
            for (int hv = 0; hv < HV; ++hv)
#pragma unroll
                for (int qd = 0; qd < QUARTS; ++qd) {
                    const int o = 16 * hv + 8 * qd + 4 * hh;
                    if (o >= DR) continue;
                    float4 a = make_float4(acc1[hv][4 * qd], acc1[hv][4 * qd + 1], acc1[hv][4 * qd + 2],
                                           acc1[hv][4 * qd + 3]);
                    float4 b = make_float4(scale * acc2[hv][4 * qd], scale * acc2[hv][4 * qd + 1],
                                           scale * acc2[hv][4 * qd + 2], scale * acc2[hv][4 * qd + 3]);
                    if (from_acc || to_acc) {
                        float *dvr = acc32 + ((size_t)bh * N + n) * DR + o;
                        float *dkr = dvr + (size_t)gridDim.y * N * DR;
                        if (from_acc) {
                            const float4 pa = *reinterpret_cast<const float4 *>(dvr);
                            const float4 pb = *reinterpret_cast<const float4 *>(dkr);
                            a.x += pa.x; a.y += pa.y; a.z += pa.z; a.w += pa.w;
                            b.x += pb.x; b.y += pb.y; b.z += pb.z; b.w += pb.w;
                        }
                        if (to_acc) {
                            *reinterpret_cast<float4 *>(dvr) = a;
                            *reinterpret_cast<float4 *>(dkr) = b;
                        }
                    }
                    if (!to_acc) {
                        const size_t at = tok_base(ts, bh, H) + tok_off(ts, n) + o;
                        u32x2 w;
                        w[0] = pack_elems<F>(a.x, a.y);
                        w[1] = pack_elems<F>(a.z, a.w);
                        *reinterpret_cast<u32x2 *>(dv + at) = w;
                        w[0] = pack_elems<F>(b.x, b.y);
                        w[1] = pack_elems<F>(b.z, b.w);
                        *reinterpret_cast<u32x2 *>(dk + at) = w;
                    }
                }
        }
    }

    if constexpr (DQ) {
        // The eight waves add their dQ partials in wave order (fixed, so the bits are reproducible) in a
        // [32*MT][16] fp32 buffer that reuses the image memory, then the workgroup stores its slot.
        float *red = reinterpret_cast<float *>(img);
        for (int w = 0; w < 8; ++w) {
            __syncthreads();   // first pass: every wave is done with the images
            if (wave == w) {
#pragma unroll
                for (int t = 0; t < MT; ++t)
#pragma unroll
                    for (int jb = 0; jb < 2; ++jb) {
                        float4 *cell = reinterpret_cast<float4 *>(red + (32 * t + 16 * jb + c16) * 16 + 4 * g16);
                        float4 x = make_float4(dqa[t][jb][0], dqa[t][jb][1], dqa[t][jb][2], dqa[t][jb][3]);
                        if (w > 0) {
                            const float4 o = *cell;
                            x.x += o.x; x.y += o.y; x.z += o.z; x.w += o.w;
                        }
                        *cell = x;
                    }
            }
        }
        __syncthreads();
        const int mleft = Mtot - m0;
        float *out = dq_part + (((size_t)bh * gridDim.x + gp.x) * Mtot + m0) * DR;
        constexpr int PCS = DR / 4;                             // float4 pieces of a DR-element row
        for (int i = tid; i < 32 * MT * PCS; i += 512) {        // latent i / PCS, columns 4 (i % PCS) ..
            const int lat = i / PCS, pc = i % PCS;
            if (lat < mleft)
                *reinterpret_cast<float4 *>(out + (size_t)lat * DR + 4 * pc) =
                    *reinterpret_cast<const float4 *>(red + (size_t)lat * 16 + 4 * pc);
        }
    }
}

#define FLARE_DKDV_PARAMS                                                                                        \
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,                    \
        const bf16_t *__restrict__ dy, const float *__restrict__ z, const float *__restrict__ lse_enc,           \
        const float *__restrict__ dz, const float *__restrict__ eps, const float *__restrict__ lse_dec2,         \
        const float *__restrict__ delta, float ld_mul, const int *__restrict__ plan, bf16_t *__restrict__ dk,    \
        bf16_t *__restrict__ dv, float *__restrict__ acc32, float *__restrict__ dq_part, TokStride ts, int H,    \
        int N, int Mtot, int m0, float c2, float scale
#define FLARE_DKDV_PASS \
    q, k, v, dy, z, lse_enc, dz, eps, lse_dec2, delta, ld_mul, plan, dk, dv, acc32, dq_part, ts, H, N, Mtot, m0, c2, scale

// One variant per launch (the workgroups of a (b,h) that the plan gives to the other variant leave at once) ...
template <int DR, int MT, bool DQ, bool ONE, bool F, int WV = 8>
__global__ __launch_bounds__(64 * WV, 1) void bwd_dkdv_mfma_kernel(FLARE_DKDV_PARAMS)
{
    dkdv_body<DR, MT, DQ, ONE, F, WV>(FLARE_DKDV_PASS);
}

// ... or both in one launch, each workgroup taking the variant that the plan names for its (b,h): one launch less per
// step (a launch whose workgroups all leave at once still costs 4-6 us).  Both bodies share the kernel's registers,
// which at one workgroup per CU costs nothing.
template <int DR, int MT, bool DQ, bool F, bool ZL = false>
__global__ __launch_bounds__(512, 1) void bwd_dkdv_planned_kernel(FLARE_DKDV_PARAMS)
{
    const int bh = grid_pos(ts, H, DR * 2).y;
    if (plan[bh] != 0) dkdv_body<DR, MT, DQ, true, F, 8, ZL>(FLARE_DKDV_PASS);
    else dkdv_body<DR, MT, DQ, false, F, 8, ZL>(FLARE_DKDV_PASS);
}
#undef FLARE_DKDV_PASS
#undef FLARE_DKDV_PARAMS

}  // namespace

// dQ partials of the backward; slot layout as the encode partials: [(b*h) * parts + part][M][d]
int mfma_dq_partial(const flare_shape &s, const void *q, const void *k, const void *v, const void *dy,
                    const float *z, const float *lse_enc, const float *dz, const float *eps,
                    const float *lse_dec2, const float *delta, float ld_mul, const int *plan, float *dq_part,
                    float scale, hipStream_t stream)
{
    const MfmaPlan p = mfma_plan(s);
    int zdim;
    const EncGeom e = dq_geom(s, &zdim);
    const int BH = s.B * s.H;
    const float c2 = scale * kLog2e;
    const int parts = p.enc.chunks * e.TG;
    const dim3 grid(p.enc.chunks, BH, zdim);
    const bf16_t *qq = (const bf16_t *)q, *kk = (const bf16_t *)k, *vv = (const bf16_t *)v, *gg = (const bf16_t *)dy;
    LaunchTimer t(KID_BWD_DQ_PARTIAL, stream);
    const bool f16 = s.dtype == FLARE_F16;
#define FLARE_DQ_ARGS                                                                                            \
    qq, kk, vv, gg, z, lse_enc, dz, eps, lse_dec2, delta, ld_mul, plan, dq_part, tok_stride(s), s.H, s.N, s.M,   \
        p.enc.chunk_len, parts, e.G, e.TG, c2
#define FLARE_DQ(DD, NBB, MINB)                                                                                  \
    do {                                                                                                         \
        if (f16) bwd_dq_mfma_kernel<DD, NBB, MINB, true><<<grid, e.threads, 0, stream>>>(FLARE_DQ_ARGS);         \
        else bwd_dq_mfma_kernel<DD, NBB, MINB, false><<<grid, e.threads, 0, stream>>>(FLARE_DQ_ARGS);            \
    } while (0)
#define FLARE_DQ_NB(DD)                      \
    do {                                     \
        if (e.NB == 1) FLARE_DQ(DD, 1, 2);   \
        else FLARE_DQ(DD, 2, 2);             \
    } while (0)
    switch (s.d) {
        case 4: FLARE_DQ_NB(4); break;
        case 8: FLARE_DQ_NB(8); break;
        case 16: FLARE_DQ_NB(16); break;
        default:
            if (e.NB == 1) FLARE_DQ(32, 1, 2);
            else FLARE_DQ(32, 2, 1);
    }
#undef FLARE_DQ_NB
#undef FLARE_DQ
#undef FLARE_DQ_ARGS
    return check_launch();
}

// dK and dV of the backward.  One workgroup of 8 waves per (b,h) slice and block of token tiles;
// the operand images need (4 or 6)*KS + 1 + 4*HV KiB of LDS per latent tile.
bool mfma_dkdv_supported(const flare_shape &s)
{
    return mfma_supported(s);
}

// workgroups per (b,h) of the dK/dV kernel (= dQ partial slots per (b,h) when it also forms dQ)
int mfma_dkdv_blocks(const flare_shape &s)
{
    const int BH = s.B * s.H;
    const int tiles = (s.N + 31) / 32;
    int blocks = (256 + BH - 1) / BH;                 // one 8-wave workgroup per CU
    if (blocks > (tiles + 7) / 8) blocks = (tiles + 7) / 8;
    return blocks;
}

// The dK/dV kernel can form the dQ partials as well (one pass over the scores for all three gradients);
// written for and used at d <= 16 (at d = 32 the dQ accumulators alone would take 128 registers).  At d <= 8
// it carries the lo term of Z in the upper half of its Z image (ZPACK in the kernel), like the token-statistics
// kernel that forms the delta it subtracts.  flare_shape.variant with FLARE_VARIANT_SEPARATE_DQ keeps the separate dQ
// kernel (tests, measurements).
bool mfma_dq_fused(const flare_shape &s)
{
    if (!mfma_supported(s) || s.d == 32) return false;
    return (s.variant & FLARE_VARIANT_SEPARATE_DQ) == 0;
}

int mfma_dkdv(const flare_shape &s, const void *q, const void *k, const void *v, const void *dy, const float *z,
              const float *lse_enc, const float *dz, const float *eps, const float *lse_dec2, const float *delta,
              float ld_mul, const int *plan, void *dk, void *dv, float *acc32, float *dq_part, int m0, float scale,
              hipStream_t stream)
{
    // Both variants (one or two exponentials per score, whichever the plan names for a (b,h)) for the latent chunk
    // that starts at m0.  dq_part != NULL: also write the dQ partials (mfma_dq_fused(s) must hold), slot layout
    // [(b*h) * mfma_dkdv_blocks(s) + block][M][d]
    const int BH = s.B * s.H;
    const dim3 grid(mfma_dkdv_blocks(s), BH);
    const bool fuse = dq_part != nullptr;
    if (fuse && !mfma_dq_fused(s)) return FLARE_EUNSUPPORTED;
    const float c2 = scale * kLog2e;
    const int MT = lat_eff(s.M) == 192 ? 8 : lat_eff(s.M) / 32;   // instantiated for 1, 2, 4, 8 tiles
    const int pd = padded_dim(s.d);
    const int KS = pd / 16, HV = (pd == 32) ? 1 : pd / 16;   // d = 32: one 32-row block of row images
    // dQ from this kernel at d = 16 with fewer tokens than latents: one more image, the lo term of Z (see the kernel)
    const bool zlo = fuse && s.d == 16 && s.N < s.M;
    const int na = (zlo ? 5 : 4) * KS + 1;
    const size_t lds = (size_t)MT * (na + 4 * HV) * 1024 + (fuse ? 8 * kFusedWaveLds * 2 : 0);
    const bf16_t *qq = (const bf16_t *)q, *kk = (const bf16_t *)k, *vv = (const bf16_t *)v, *gg = (const bf16_t *)dy;
    const bool f16 = s.dtype == FLARE_F16;
#define FLARE_DKDV_LAUNCH(KERN, THREADS)                                                                         \
    do {                                                                                                         \
        auto kern = KERN;                                                                                        \
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                (int)lds) != hipSuccess)                                                         \
            return FLARE_ELAUNCH;                                                                                \
        kern<<<grid, THREADS, lds, stream>>>(qq, kk, vv, gg, z, lse_enc, dz, eps, lse_dec2, delta, ld_mul, plan, \
                                             (bf16_t *)dk, (bf16_t *)dv, acc32, dq_part, tok_stride(s), s.H,     \
                                             s.N, s.M, m0, c2, scale);                                           \
    } while (0)
    if (s.d == 32 && MT == 8) {
        // d = 32, 256 latents: the one-exponential variant fits 168 registers, so twelve waves (three per SIMD) share
        // its images; the two-exponential variant keeps eight.  One launch each.
        {
            LaunchTimer t(KID_BWD_DKDV, stream);
            if (f16) FLARE_DKDV_LAUNCH((bwd_dkdv_mfma_kernel<32, 8, false, true, true, 12>), 768);
            else FLARE_DKDV_LAUNCH((bwd_dkdv_mfma_kernel<32, 8, false, true, false, 12>), 768);
        }
        if (check_launch() != FLARE_OK) return FLARE_ELAUNCH;
        LaunchTimer t(KID_BWD_DKDV_2EXP, stream);
        if (f16) FLARE_DKDV_LAUNCH((bwd_dkdv_mfma_kernel<32, 8, false, false, true, 8>), 512);
        else FLARE_DKDV_LAUNCH((bwd_dkdv_mfma_kernel<32, 8, false, false, false, 8>), 512);
        return check_launch();
    }
    LaunchTimer t(KID_BWD_DKDV, stream);
#define FLARE_DKDV(DD, MTT, LO)                                                                 \
    do {                                                                                        \
        if (f16) FLARE_DKDV_LAUNCH((bwd_dkdv_planned_kernel<DD, MTT, LO, true>), 512);          \
        else FLARE_DKDV_LAUNCH((bwd_dkdv_planned_kernel<DD, MTT, LO, false>), 512);             \
    } while (0)
#define FLARE_DKDV_MT(DD, LO)                       \
    switch (MT) {                                   \
        case 1: FLARE_DKDV(DD, 1, LO); break;       \
        case 2: FLARE_DKDV(DD, 2, LO); break;       \
        case 4: FLARE_DKDV(DD, 4, LO); break;       \
        case 8: FLARE_DKDV(DD, 8, LO); break;       \
        default: return FLARE_EUNSUPPORTED;         \
    }
    if (s.d == 4 && fuse) {
        FLARE_DKDV_MT(4, true)
    } else if (s.d == 8 && fuse) {
        FLARE_DKDV_MT(8, true)
    } else if (s.d == 16 && fuse && zlo) {
#define FLARE_DKDV_Z(MTT)                                                                          \
    do {                                                                                           \
        if (f16) FLARE_DKDV_LAUNCH((bwd_dkdv_planned_kernel<16, MTT, true, true, true>), 512);     \
        else FLARE_DKDV_LAUNCH((bwd_dkdv_planned_kernel<16, MTT, true, false, true>), 512);        \
    } while (0)
        switch (MT) {
            case 1: FLARE_DKDV_Z(1); break;
            case 2: FLARE_DKDV_Z(2); break;
            case 4: FLARE_DKDV_Z(4); break;
            case 8: FLARE_DKDV_Z(8); break;
            default: return FLARE_EUNSUPPORTED;
        }
#undef FLARE_DKDV_Z
    } else if (s.d == 16 && fuse) {
        FLARE_DKDV_MT(16, true)
    } else if (s.d == 4) {
        FLARE_DKDV_MT(4, false)
    } else if (s.d == 8) {
        FLARE_DKDV_MT(8, false)
    } else if (s.d == 16) {
        FLARE_DKDV_MT(16, false)
    } else {
        switch (MT) {   // d = 32 (with 256 latents: above)
            case 1: FLARE_DKDV(32, 1, false); break;
            case 2: FLARE_DKDV(32, 2, false); break;
            case 4: FLARE_DKDV(32, 4, false); break;
            default: return FLARE_EUNSUPPORTED;
        }
    }
#undef FLARE_DKDV_MT
#undef FLARE_DKDV
#undef FLARE_DKDV_LAUNCH
    return check_launch();
}

size_t mfma_dkdv_acc_bytes(const flare_shape &s)
{
    if (s.M <= kLatChunk) return 0;
    return ((size_t)s.B * s.H * s.N * s.d * 4 * 2 + 255) & ~(size_t)255;
}

// partial slots per (b,h) that mfma_dq_partial writes
int mfma_dq_parts(const flare_shape &s)
{
    const MfmaPlan p = mfma_plan(s);
    int zdim;
    return p.enc.chunks * dq_geom(s, &zdim).TG;
}

}  // namespace flare
