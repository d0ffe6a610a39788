// Matrix-core (MFMA) kernels of the FLARE mixer for bf16 and fp16 storage on gfx950.
//
// The kernels are built from v_mfma_f32_32x32x16_bf16 and keep the M x N weights in
// registers only.  The softmax work per score is one v_exp_f32, half a v_cvt_pk_bf16_f32 and
// half a v_max3_f32: the score MFMAs already deliver  S2 - stabiliser  because
//   * q is pre-multiplied by scale*log2(e) and split into two bf16 terms (hi + lo), so the
//     product is exact to ~2^-17 and the exponential is a bare 2^x;
//   * the stabiliser rides in the matrix instruction: as the C operand the score products start
//     from (decode: one splat of -max per token tile), or in a k-step of its own whose operands
//     hold it as a hi + lo pair against ones (encode, and the log-sum-exp normalisers, -eps and
//     -delta of the backward).
// The probabilities are rounded to bf16 once and feed the second MFMA straight from the
// accumulator layout: the contraction index of the second product (tokens in the encode,
// latents in the decode) is order-free, so the value operand is simply loaded in the
// permuted order the accumulator layout dictates.  Row sums come out of the same MFMA from
// a row of ones appended to the value operand, so numerator and denominator use identical
// rounded weights.
//
// Register layouts of v_mfma_f32_32x32x16_bf16 (lane l, l32 = l % 32, hh = l / 32):
//   A operand: row l32, contraction slots 8*hh .. 8*hh+7 (8 bf16 = 4 VGPRs)
//   B operand: column l32, contraction slots 8*hh .. 8*hh+7
//   C/D:       column l32, register r (0..15) holds row 8*(r/4) + 4*hh + r%4
//
// fp16 storage (template flag F): the score products and everything that rides in their
// contraction (q' hi + lo, stabilisers, log-sum-exp pairs) use v_mfma_f32_32x32x16_f16 on the raw
// fp16 keys, so the scores are as exact as with bf16 storage.  The softmax weights, dS and the
// operands they are multiplied with stay bf16 (their range is needed: normalised weights of a
// million tokens are far below the smallest fp16 number), so the V, dY (and, where K is a value,
// K) rows are rounded to bf16 after the load; outputs are rounded to fp16 from fp32.
//
// Equations: Section 3.1, Eq. flare_encode / Eq. flare_decode; Appendix F.
#ifndef FLARE_MFMA_COMMON_H
#define FLARE_MFMA_COMMON_H

#include "flare_internal.h"

namespace flare {
namespace {

// a compile-time flag passed to a generic lambda (decltype(tag)::value)
template <bool B>
struct PlainTag { static constexpr bool value = B; };

typedef uint16_t bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 w) { return __builtin_bit_cast(bf16x8, w); }
__device__ __forceinline__ uint32_t rne_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
// two fp32 -> packed bf16 (low half = a, high half = b), round to nearest even: one
// v_cvt_pk_bf16_f32.  Left to the compiler (no inline asm) so that it keeps the wait state a
// VALU read of a transcendental result needs.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b)
{
    f32x2 v;
    v[0] = a;
    v[1] = b;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// Score-chain product: operands hold 8 elements of the storage type (bf16, or fp16 when F); they
// are carried as bf16x8 registers either way.
template <bool F>
__device__ __forceinline__ f32x16 mfma_s(bf16x8 a, bf16x8 b, f32x16 c)
{
    if constexpr (F)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c,
                                                      0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// ---- 16-bit elements of the storage type ----
// value of the low / high half of a word
template <bool F>
__device__ __forceinline__ float elem_lo(uint32_t w)
{
    if constexpr (F) return (float)__builtin_bit_cast(f16x2, w)[0];
    else return __uint_as_float(w << 16);
}
template <bool F>
__device__ __forceinline__ float elem_hi(uint32_t w)
{
    if constexpr (F) return (float)__builtin_bit_cast(f16x2, w)[1];
    else return __uint_as_float(w & 0xffff0000u);
}
// fp32 -> 16 bits, round to nearest even, and back
template <bool F>
__device__ __forceinline__ uint32_t rne_elem(float f)
{
    if constexpr (F) return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
    else return rne_bf16(f);
}
template <bool F>
__device__ __forceinline__ float elem_value(uint32_t bits)
{
    if constexpr (F) return (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
    else return __uint_as_float(bits << 16);
}
template <bool F>
__device__ __forceinline__ float elem_round(float x) { return elem_value<F>(rne_elem<F>(x)); }
// two fp32 -> one packed word of the storage type (one v_cvt_pk_{bf16,f16}_f32)
template <bool F>
__device__ __forceinline__ uint32_t pack_elems(float a, float b)
{
    if constexpr (F) {
        f32x2 v;
        v[0] = a;
        v[1] = b;
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
    } else {
        return cvt_pk_bf16(a, b);
    }
}
// Value of a stored dY element as the c product sees it: with fp16 storage the rows are rounded to
// bf16 before they meet Z, and delta[n] = <dY_n, Y_n> must be formed from the same rounded values, or
// c - delta = <dY_n, Z_m - Y_n> would not cancel where the latents agree (one latent: exactly zero).
template <bool F>
__device__ __forceinline__ float dy_lo(uint32_t w)
{
    if constexpr (F) return __uint_as_float(rne_bf16(elem_lo<true>(w)) << 16);
    else return elem_lo<false>(w);
}
template <bool F>
__device__ __forceinline__ float dy_hi(uint32_t w)
{
    if constexpr (F) return __uint_as_float(rne_bf16(elem_hi<true>(w)) << 16);
    else return elem_hi<false>(w);
}
// 1.0 in the storage type, and twice in one word
template <bool F> constexpr uint32_t kOne = F ? 0x3c00u : 0x3f80u;
template <bool F> constexpr uint32_t kOnePair = F ? 0x3c003c00u : 0x3f803f80u;
// 8 stored elements -> 8 bf16 (operands of the weight-side products); nothing to do for bf16 storage
template <bool F>
__device__ __forceinline__ u32x4 to_bf16_row(u32x4 w)
{
    if constexpr (F) {
        u32x4 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = cvt_pk_bf16(elem_lo<true>(w[i]), elem_hi<true>(w[i]));
        return r;
    } else {
        return w;
    }
}
__device__ __forceinline__ f32x16 splat16(float x)
{
    f32x16 v;
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = x;
    return v;
}
__device__ __forceinline__ float max16(const f32x16 &s, float m)
{
#pragma unroll
    for (int i = 0; i < 16; i += 2) m = fmaxf(fmaxf(m, s[i]), s[i + 1]);   // one v_max3_f32 per pair
    return m;
}
// 16 accumulator values -> 16 packed bf16 probabilities 2^x (two B operands of 8)
__device__ __forceinline__ void exp_pack(const f32x16 &dlt, bf16x8 &p0, bf16x8 &p1)
{
    u32x4 w0, w1;
#pragma unroll
    for (int i = 0; i < 4; ++i) w0[i] = cvt_pk_bf16(fast_exp2(dlt[2 * i]), fast_exp2(dlt[2 * i + 1]));
#pragma unroll
    for (int i = 0; i < 4; ++i) w1[i] = cvt_pk_bf16(fast_exp2(dlt[8 + 2 * i]), fast_exp2(dlt[8 + 2 * i + 1]));
    p0 = as_bf16x8(w0);
    p1 = as_bf16x8(w1);
}
// The same, and the sum of the 16 rounded weights added to `sum` (v_dot2c_f32_bf16 against a pair of ones: the
// products are exact and the sums fp32, so this is the sum of exactly the weights the matrix product sees).
// The dot products take the packed words as they leave the conversion, before they become vector elements.
__device__ __forceinline__ void exp_pack_sum(const f32x16 &dlt, bf16x8 &p0, bf16x8 &p1, float &sum)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const bf16x2_t ones = __builtin_bit_cast(bf16x2_t, 0x3f803f80u);
    u32x4 w0, w1;
    float acc = sum;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t w = cvt_pk_bf16(fast_exp2(dlt[2 * i]), fast_exp2(dlt[2 * i + 1]));
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w), ones, acc, false);
        w0[i] = w;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t w = cvt_pk_bf16(fast_exp2(dlt[8 + 2 * i]), fast_exp2(dlt[8 + 2 * i + 1]));
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w), ones, acc, false);
        w1[i] = w;
    }
    sum = acc;
    p0 = as_bf16x8(w0);
    p1 = as_bf16x8(w1);
}
// acc + <a, b> for eight bf16 elements a side (four packed pairs): v_dot2c_f32_bf16, exact products, fp32 sums.
// Written as one opaque block because the compiler's own form of the instruction mixes up its operands when
// they are elements of loaded vectors (hipcc 7.2), and closed by the wait states that a reader of the result
// (also a DPP move) needs after a dot instruction: inside the block the compiler inserts none.
__device__ __forceinline__ float dot8_bf16(const u32x4 &a, const u32x4 &b, float acc)
{
    asm volatile("v_dot2c_f32_bf16 %0, %1, %2\n\t"
                 "v_dot2c_f32_bf16 %0, %3, %4\n\t"
                 "v_dot2c_f32_bf16 %0, %5, %6\n\t"
                 "v_dot2c_f32_bf16 %0, %7, %8\n\t"
                 "s_nop 3"
                 : "+v"(acc)
                 : "v"(a[0]), "v"(b[0]), "v"(a[1]), "v"(b[1]), "v"(a[2]), "v"(b[2]), "v"(a[3]), "v"(b[3]));
    return acc;
}
// Nothing may be scheduled across this point: keeps the matrix-core work of the next tile issued
// ahead of the vector work of the current one.
__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }
// Ask the scheduler for the next group of `n` instructions of one class, in the order the requests are
// written (classes: matrix, transcendental, other vector ALU).  Used to spread the matrix
// instructions of a tile between its vector instructions, so that the matrix pipe (32 clocks per
// instruction) never blocks the wave's issue.
// The LDS transpose read of gfx950 (ds_read_b64_tr_b16), 16-bit elements.  Within each block of 16 lanes, lane p
// addresses a chunk of four consecutive elements E[p][0..3]; lane i of the block receives the four elements
// E[i/4][i%4], E[i/4 + 4][i%4], E[i/4 + 8][i%4], E[i/4 + 12][i%4]: with the 16 chunks laid over four rows of a
// row-major tile (chunk p = 4 (row) + (piece of four columns), row = p / 4, piece = p % 4), lane i gets column i of
// those four rows -- a column segment of a row-major tile, which is what a matrix-instruction operand wants of a
// tile that was written the other way round.  (The lane mapping was read off the instruction's output on a
// tile of distinct values.)  Returns two dwords (four elements); p must be 8-byte aligned.
__device__ __forceinline__ u32x2 lds_read_tr16(const uint16_t *p)
{
    typedef short s16x4_t __attribute__((ext_vector_type(4)));
    const s16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4_t __attribute__((address_space(3))) *)(const_cast<uint16_t *>(p)));
    return __builtin_bit_cast(u32x2, v);
}

#define FLARE_GROUP_MFMA(n) __builtin_amdgcn_sched_group_barrier(0x008, n, 0)
#define FLARE_GROUP_TRANS(n) __builtin_amdgcn_sched_group_barrier(0x400, n, 0)
#define FLARE_GROUP_VALU(n) __builtin_amdgcn_sched_group_barrier(0x002, n, 0)

// Contraction slot (8*hh + i) of k-step s2 (0 or 1) of a 32-wide tile maps to this index within
// the tile: the row that accumulator register 8*s2 + i holds.
__device__ __forceinline__ int perm_index(int s2, int hh, int i) { return 16 * s2 + 8 * (i / 4) + 4 * hh + (i % 4); }

// Head dimensions below 16 run with the contraction padded to 16: DR is the real d (the row length
// in memory), D = max(DR, 16) what the matrix cores see; the padding slots are zero in every
// operand.  The helpers below move 8 (bf16, fp32) or 4 (outputs) consecutive elements of a
// DR-element row and give zeros / skip the store beyond its end.
constexpr int padded_dim(int dr) { return dr < 16 ? 16 : dr; }
template <int DR>
__device__ __forceinline__ u32x4 row8_bf16(const bf16_t *__restrict__ row, int e0)   // e0: a multiple of 8
{
    u32x4 w;
    w[0] = 0u; w[1] = 0u; w[2] = 0u; w[3] = 0u;
    if constexpr (DR >= 16) {
        w = *reinterpret_cast<const u32x4 *>(row + e0);
    } else if constexpr (DR == 8) {
        if (e0 == 0) w = *reinterpret_cast<const u32x4 *>(row);
    } else {
        if (e0 == 0) {
            const u32x2 t = *reinterpret_cast<const u32x2 *>(row);
            w[0] = t[0]; w[1] = t[1];
        }
    }
    return w;
}
template <int DR>
__device__ __forceinline__ void row8_f32(const float *__restrict__ row, int e0, float (&x)[8])
{
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = 0.f;
    if (DR >= 16 || e0 == 0) {
#pragma unroll
        for (int i = 0; i < (DR >= 8 ? 8 : DR); ++i) x[i] = row[e0 + i];
    }
}
// Accumulator rows of one 16-wide column group: registers 0-3 hold columns 4*hh .. 4*hh+3, registers
// 4-7 columns 8 + 4*hh ... of group hv.  true iff that quartet lies inside a DR-element row.
template <int DR>
__device__ __forceinline__ bool quartet_inside(int hv, int hh, int upper)
{
    return 16 * hv + 8 * upper + 4 * hh < DR;
}

// Latent-query operand for one 32-latent tile: row/column = latent, contraction over d.
// Lane half hh covers d-indices (D/2)*hh + 8*s + i for k-step s.  The same mapping is used for
// the key operand.  PRE: multiply by c2 and split into hi + lo bf16 terms; else raw bits (sign
// flipped when c2 < 0 so that the kernel can work with |c2|).
// PACKED (d <= 8 only, where the upper half of the padded contraction is free): the lower lane half
// gets the hi terms and the upper one the lo terms of the same d-indices, so that ONE product with a
// token operand that repeats its row in both halves gives the full-precision score; lo is unused.
constexpr bool pack_dim(int dr) { return dr <= 8; }
template <int DR, bool PRE, bool F, bool PACKED = false>
__device__ __forceinline__ void load_q_operand(const bf16_t *__restrict__ q_row, int hh, float c2, bool flip,
                                               bf16x8 (&hi)[padded_dim(DR) / 16], bf16x8 (&lo)[padded_dim(DR) / 16])
{
    constexpr int D = padded_dim(DR);
    static_assert(!PACKED || (PRE && pack_dim(DR)), "packed operands need d <= 8 and the pre-scaled form");
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
        const u32x4 w = row8_bf16<DR>(q_row, PACKED ? 0 : (D / 2) * hh + 8 * s);
        if constexpr (PRE) {
            u32x4 wh, wl;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float a = elem_lo<F>(w[i]) * c2, b = elem_hi<F>(w[i]) * c2;
                const uint32_t ah = rne_elem<F>(a), bh = rne_elem<F>(b);
                const float ar = a - elem_value<F>(ah), br = b - elem_value<F>(bh);
                wh[i] = ah | (bh << 16);
                wl[i] = rne_elem<F>(ar) | (rne_elem<F>(br) << 16);
            }
            hi[s] = as_bf16x8((PACKED && hh) ? wl : wh);
            lo[s] = as_bf16x8(wl);
        } else {
            u32x4 wf = w;
            if (flip) {
#pragma unroll
                for (int i = 0; i < 4; ++i) wf[i] = w[i] ^ 0x80008000u;
            }
            hi[s] = as_bf16x8(wf);
            lo[s] = as_bf16x8(wf);
        }
    }
}

// Any number of latents runs on tiles of 32: a latent index at or beyond the head's real count is a
// padding latent.  Its operands are zeros (loads are clamped to the last real row, never past the
// tensor), its results are not stored, and where it could enter a sum over the latents (the decode's
// softmax, dK and dV) it is masked or multiplies zeros.
__device__ __forceinline__ bf16x8 zero_operand()
{
    u32x4 w;
    w[0] = 0u; w[1] = 0u; w[2] = 0u; w[3] = 0u;
    return __builtin_bit_cast(bf16x8, w);
}
// x as a hi + lo pair of storage-type values packed in one word (hi in the low half)
template <bool F>
__device__ __forceinline__ uint32_t split_pair(float x)
{
    const uint32_t hi = rne_elem<F>(x);
    return hi | (rne_elem<F>(x - elem_value<F>(hi)) << 16);
}
// x as a hi + lo pair of bf16 values packed in one word (hi in the low half)
__device__ __forceinline__ uint32_t split_bf16_pair(float x)
{
    const uint32_t hi = (__float_as_uint(x) + 0x7fffu + ((__float_as_uint(x) >> 16) & 1u)) >> 16;
    const float r = x - __uint_as_float(hi << 16);
    const uint32_t lo = (__float_as_uint(r) + 0x7fffu + ((__float_as_uint(r) >> 16) & 1u)) >> 16;
    return hi | (lo << 16);
}
// Replace contraction slot 0 (low half of word 0) of an operand; `keep` and `bits` are per-lane
// constants so that only the lower lane half (which owns slot 0) is changed.
__device__ __forceinline__ bf16x8 with_slot0(bf16x8 x, uint32_t keep, uint32_t bits)
{
    u32x4 w = __builtin_bit_cast(u32x4, x);
    w[0] = (w[0] & keep) | bits;
    return as_bf16x8(w);
}
__device__ __forceinline__ void compiler_fence() { asm volatile("" ::: "memory"); }
// The value as of this point of the program: an opaque statement takes and returns it, so that whatever produces
// it (a load's arrival, a conversion) is complete here and not wherever its first real use ends up.
__device__ __forceinline__ bf16x8 pinned(bf16x8 x)
{
    u32x4 w = __builtin_bit_cast(u32x4, x);
    asm volatile("" : "+v"(w));
    return __builtin_bit_cast(bf16x8, w);
}
__device__ __forceinline__ float pinned(float x)
{
    asm volatile("" : "+v"(x));
    return x;
}

// More than 256 latents per head are taken 256 at a time: the latent-major kernels get one more grid
// dimension (each workgroup owns one such chunk and streams the tokens again), the token-major ones
// run once per chunk and a merge kernel combines the chunks.
constexpr int kLatChunk = 256;
// Any M runs on the tile geometry of the next size the kernels are instantiated for: 32, 64, 128, 192
// (only when M is exactly 192), 256, or whole chunks of 256; the latents beyond M are padding.
inline int pad_latents(int M)
{
    if (M <= 32) return 32;
    if (M <= 64) return 64;
    if (M <= 128) return 128;
    if (M == 192) return 192;
    return (M + kLatChunk - 1) / kLatChunk * kLatChunk;
}
inline int lat_eff(int M) { return M > kLatChunk ? kLatChunk : pad_latents(M); }   // latents per chunk (padded)
inline int lat_chunks(int M) { return (M + kLatChunk - 1) / kLatChunk; }

constexpr float kLazy = 16.f;   // the stabiliser moves when a score exceeds it by this much (log2 units)
constexpr int kVtStride = 36;   // uint16 per LDS row: 32 tokens + 4 pad (72 B, conflict-free b64 reads)

// The grid position (x = token chunk, y = b*H + h) that this workgroup works on.
// With the [B,H,N,d] layout it is the workgroup's own.  With [B,N,H,d] the rows of neighbouring heads
// lie side by side within a token: 128 / (2 d) heads share each 128-byte cache line.  Workgroups go to the
// eight XCDs, each with an L2 of its own, round-robin by their linear index, so the workgroups that walk
// over the same tokens for the heads of one line would land on different XCDs, and each of those L2s
// would fetch the whole line for its own part of it (measured at d = 32: twice to three times the bytes
// of the other layout).  So the linear index is re-read as (XCD, slot within the XCD), and the heads
// of one line take consecutive slots of one XCD: they are dispatched together there and share the
// fetched lines.  A remainder that does not fill a round of the eight XCDs keeps the plain order.
// The mapping is a bijection of the grid's (x, y) plane; planes (gridDim.z) are mapped alike.
struct GridPos { int x, y; };
__device__ __forceinline__ GridPos grid_pos(const TokStride &ts, int H, int row_bytes)
{
    GridPos p{(int)blockIdx.x, (int)blockIdx.y};
    if (ts.sh >= ts.sn) return p;                 // heads are not interleaved within a token
    int hg = 128 / row_bytes;                     // heads per cache line
    while (hg > 1 && H % hg != 0) hg >>= 1;
    if (hg <= 1) return p;
    const int gx = gridDim.x, hgroups = H / hg;
    const int L = p.x + gx * p.y;
    const int groups = gx * ((int)gridDim.y / hg);          // (chunk, b, group of heads)
    const int full = (groups / 8) * 8 * hg;                 // workgroups in whole rounds of the eight XCDs
    int g, hs;
    if (L < full) {
        const int slot = L >> 3;
        hs = slot % hg;
        g = (slot / hg) * 8 + (L & 7);
    } else {
        const int r = L - full;
        g = (groups / 8) * 8 + r / hg;
        hs = r % hg;
    }
    const int yg = g / gx;                                  // b * hgroups + group of heads
    p.x = g % gx;
    p.y = (yg / hgroups) * H + (yg % hgroups) * hg + hs;
    return p;
}

inline int check_launch() { return hipGetLastError() == hipSuccess ? FLARE_OK : FLARE_ELAUNCH; }

// latent-group geometry of the encode for a given M
// NB = 32-latent tiles per wave, G = latent groups (waves) per token tile, TG = token groups.
struct EncGeom { int NB, G, TG, threads; };
inline EncGeom enc_geom(int M, int d)
{
    EncGeom e;
    const int MB = M / 32;
    if (MB == 1) e.NB = 1;
    else if (d == 16 && MB % 4 == 0) e.NB = 4;
    else e.NB = 2;
    e.G = MB / e.NB;
    e.TG = (e.G == 3) ? 1 : 4 / e.G;
    e.threads = 64 * e.G * e.TG;
    return e;
}

// Geometry of the dQ kernel, which keeps more operands per latent tile than the encode: at most two
// tiles per wave, and at d = 32 one (two waves per SIMD then fit; a workgroup covers 128 latents and
// the third grid dimension the rest).  *zdim = workgroups along the latents.
inline EncGeom dq_geom(const flare_shape &s, int *zdim)
{
    const int Me = lat_eff(s.M);
    EncGeom e = enc_geom(Me, padded_dim(s.d));
    if (e.NB == 4) {
        e.NB = 2;
        e.G = Me / 64;
        e.TG = (e.G == 3) ? 1 : 4 / e.G;
    }
    // d = 32: one latent tile per wave and two waves per SIMD beat two tiles per wave at one wave per SIMD
    // (309 against 366 us at N = 262144, M = 256) -- except with the heads interleaved within a token, where
    // the waves of a workgroup, which all read the same token rows, run into the L1's line rate: there half
    // as many waves per token tile win (345 against 460 us)
    if (s.d == 32 && Me % 128 == 0 && s.layout != FLARE_BNHD) {
        e.NB = 1;
        e.G = 4;
        e.TG = 1;
    }
    e.threads = 64 * e.G * e.TG;
    *zdim = pad_latents(s.M) / (32 * e.NB * e.G);
    return e;
}

constexpr int kEncodeTargetBlocks = 512;   // two 4-wave workgroups per CU
constexpr int kDecodeTargetBlocks = 512;

}  // namespace
}  // namespace flare

#endif  // FLARE_MFMA_COMMON_H
