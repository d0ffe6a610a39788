// fp32 vector-ALU kernels of the FLARE mixer: the fp32 path, and the general path for
// shapes the matrix-core kernels do not take (any M, d in {4,8,16,32}, f32 or bf16 storage).
//
// Two kernel shapes cover every step:
//   * one thread per LATENT, streaming tokens (encode partials, dZ partials, dQ partials):
//     the token rows k_n, v_n, dy_n have wave-uniform addresses, so they arrive through the
//     scalar data path (reads only) and cost no vector memory traffic or LDS;
//   * one thread per TOKEN, streaming latents (decode, token statistics, dK/dV): here
//     q_m, z_m, dZ_m are the wave-uniform operands.
// Scores are kept in log2 units, S2 = (scale*log2 e) * <q,k>, so that the softmax needs
// one v_exp_f32 per score.  Every cross-block reduction goes through per-chunk partials
// that are merged in a fixed order: results are bit-reproducible.
//
// Equations: Section 3.1, Eq. flare_encode / Eq. flare_decode; Appendix F per-latent and
// per-token forms.  The backward follows the formulas in include/flare.h.
#include <stdlib.h>

#include "flare_internal.h"

namespace flare {
namespace {

typedef uint16_t bf16_t;  // raw bfloat16 bits
struct f16_t { uint16_t bits; };   // raw IEEE fp16 bits (a type of its own so that the row helpers can overload)

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Load one row of D elements as floats.  `p` points at the first element of the row.
template <int D>
__device__ __forceinline__ void load_row(const float *__restrict__ p, float (&out)[D])
{
    const float4 *p4 = reinterpret_cast<const float4 *>(p);
#pragma unroll
    for (int i = 0; i < D / 4; ++i) {
        float4 t = p4[i];
        out[4 * i + 0] = t.x; out[4 * i + 1] = t.y; out[4 * i + 2] = t.z; out[4 * i + 3] = t.w;
    }
}
template <int D>
__device__ __forceinline__ void load_row(const bf16_t *__restrict__ p, float (&out)[D])
{
    if constexpr (D == 4) {
        uint2 t = *reinterpret_cast<const uint2 *>(p);
        out[0] = bf16_lo(t.x); out[1] = bf16_hi(t.x); out[2] = bf16_lo(t.y); out[3] = bf16_hi(t.y);
    } else {
        const uint4 *p4 = reinterpret_cast<const uint4 *>(p);
#pragma unroll
        for (int i = 0; i < D / 8; ++i) {
            uint4 t = p4[i];
            out[8 * i + 0] = bf16_lo(t.x); out[8 * i + 1] = bf16_hi(t.x);
            out[8 * i + 2] = bf16_lo(t.y); out[8 * i + 3] = bf16_hi(t.y);
            out[8 * i + 4] = bf16_lo(t.z); out[8 * i + 5] = bf16_hi(t.z);
            out[8 * i + 6] = bf16_lo(t.w); out[8 * i + 7] = bf16_hi(t.w);
        }
    }
}
template <int D>
__device__ __forceinline__ void load_row(const f16_t *__restrict__ p, float (&out)[D])
{
    const _Float16 *h = reinterpret_cast<const _Float16 *>(p);
    typedef _Float16 half4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int i = 0; i < D / 4; ++i) {
        const half4 t = *reinterpret_cast<const half4 *>(h + 4 * i);
        out[4 * i] = (float)t[0]; out[4 * i + 1] = (float)t[1]; out[4 * i + 2] = (float)t[2]; out[4 * i + 3] = (float)t[3];
    }
}
template <int D>
__device__ __forceinline__ void store_row(f16_t *__restrict__ p, const float (&in)[D])
{
    _Float16 *h = reinterpret_cast<_Float16 *>(p);
    typedef _Float16 half4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int i = 0; i < D / 4; ++i) {
        half4 t;
        t[0] = (_Float16)in[4 * i]; t[1] = (_Float16)in[4 * i + 1]; t[2] = (_Float16)in[4 * i + 2]; t[3] = (_Float16)in[4 * i + 3];
        *reinterpret_cast<half4 *>(h + 4 * i) = t;
    }
}
template <int D>
__device__ __forceinline__ void store_row(float *__restrict__ p, const float (&in)[D])
{
    float4 *p4 = reinterpret_cast<float4 *>(p);
#pragma unroll
    for (int i = 0; i < D / 4; ++i) p4[i] = make_float4(in[4 * i], in[4 * i + 1], in[4 * i + 2], in[4 * i + 3]);
}
template <int D>
__device__ __forceinline__ void store_row(bf16_t *__restrict__ p, const float (&in)[D])
{
    uint32_t w[D / 2];
#pragma unroll
    for (int i = 0; i < D / 2; ++i) w[i] = f32_to_bf16_rne(in[2 * i]) | (f32_to_bf16_rne(in[2 * i + 1]) << 16);
    if constexpr (D == 4) {
        *reinterpret_cast<uint2 *>(p) = make_uint2(w[0], w[1]);
    } else {
        uint4 *p4 = reinterpret_cast<uint4 *>(p);
#pragma unroll
        for (int i = 0; i < D / 8; ++i) p4[i] = make_uint4(w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]);
    }
}
template <int D>
__device__ __forceinline__ float dot(const float (&a)[D], const float (&b)[D])
{
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < D; ++j) s = fmaf(a[j], b[j], s);
    return s;
}

// The thread-per-latent kernels read the token rows through the scalar data path (the address is the same for the
// whole wave), a handful of rows per request, and a wave can use none of them before all have arrived: with the
// rows coming from HBM every group of tokens costs several full memory latencies.  So each group first touches
// the rows of a later group with one vector load that needs no register: its data goes to a few bytes of LDS
// that nobody reads (global_load_lds_dword), and the rows are in the L2 when the scalar requests come.
// Lanes 8 i + t of every 32 touch row t of the group kPrefetchTokens on in tensor i (a, b, c; i = 3: a again).
// The tensors' addresses come in a second time as plain integers (RowTouch): a pointer derived from the kernel's
// own tensor arguments would make the compiler treat the rows as possibly overwritten by this load and take
// them off the scalar data path.
constexpr int kPrefetchTokens = 16;   // two groups of kGroup ahead
struct RowTouch {
    unsigned long long a, b, c;   // addresses of up to three token tensors (element (0,0,0,0)); unused: a again
    unsigned long long f, g;      // addresses of up to two per-token fp32 arrays [b*h][N] (lanes 24-27); or 0
};
template <typename T>
__device__ __forceinline__ void touch_rows(const RowTouch &rt, size_t base, const TokStride &ts, int n, int N,
                                           float *sink)
{
    const int lane = threadIdx.x & 31;
    const int tok = min(n + kPrefetchTokens + (lane & 7), N - 1);
    const unsigned long long which = (lane & 16) ? ((lane & 8) ? rt.a : rt.c) : ((lane & 8) ? rt.b : rt.a);
    const void *src = reinterpret_cast<const T *>(which) + base + tok_off(ts, tok);
    if (lane >= 24 && lane < 28 && rt.f != 0) {   // the statistics of tokens n + kPrefetchTokens and 32 further on
        const unsigned long long arr = (lane & 2) ? rt.g : rt.f;
        src = reinterpret_cast<const float *>(arr) + (size_t)blockIdx.y * N + min(n + kPrefetchTokens + 32 * (lane & 1), N - 1);
    }
    __builtin_amdgcn_global_load_lds(src, sink, 4, 0, 0);
}

inline unsigned long long addr(const void *p) { return (unsigned long long)(uintptr_t)p; }

constexpr int kLatentBlock = 256;  // threads per block in the thread-per-latent kernels
constexpr int kTokenBlock = 256;   // threads per block in the thread-per-token kernels
constexpr int kGroup = 8;          // scores handled between two running-max updates

// ---------------------------------------------------------------------------------------
// Encode partials: thread = latent m, block = (chunk of tokens, b*h, block of latents).
// Online softmax over the chunk's tokens; writes (running max, sum, unnormalised O) per chunk.
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kLatentBlock) void encode_partial_kernel(
    const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v,
    float *__restrict__ m_part, float *__restrict__ l_part, float *__restrict__ o_part,
    TokStride ts, int H, int N, int M, int chunk_len, int chunks, float c2, RowTouch touch)
{
    const int m = blockIdx.z * kLatentBlock + threadIdx.x;
    if (m >= M) return;
    const int bh = blockIdx.y, h = bh % H, chunk = blockIdx.x;
    float qm[D];
    load_row<D>(q + (size_t)h * ts.sq + (size_t)m * D, qm);
#pragma unroll
    for (int j = 0; j < D; ++j) qm[j] *= c2;
    const T *kb = k + tok_base(ts, bh, H);
    const T *vb = v + tok_base(ts, bh, H);
    const int n0 = chunk * chunk_len;
    const int n1 = min(N, n0 + chunk_len);

    float mr = -INFINITY, l = 0.f, o[D];
#pragma unroll
    for (int j = 0; j < D; ++j) o[j] = 0.f;

    __shared__ float sink[kLatentBlock];
    int n = n0;
    for (; n + kGroup <= n1; n += kGroup) {
        touch_rows<T>(touch, tok_base(ts, bh, H), ts, n, N, sink);
        float s[kGroup];
        float gm = mr;
#pragma unroll
        for (int t = 0; t < kGroup; ++t) {
            float kr[D];
            load_row<D>(kb + tok_off(ts, (n + t)), kr);
            s[t] = dot<D>(qm, kr);
            gm = fmaxf(gm, s[t]);
        }
        const float al = fast_exp2(mr - gm);   // mr = -inf on the first group: exp2(-inf) = 0
        mr = gm;
        l *= al;
#pragma unroll
        for (int j = 0; j < D; ++j) o[j] *= al;
#pragma unroll
        for (int t = 0; t < kGroup; ++t) {
            const float p = fast_exp2(s[t] - mr);
            l += p;
            float vr[D];
            load_row<D>(vb + tok_off(ts, (n + t)), vr);
#pragma unroll
            for (int j = 0; j < D; ++j) o[j] = fmaf(p, vr[j], o[j]);
        }
    }
    for (; n < n1; ++n) {
        float kr[D], vr[D];
        load_row<D>(kb + tok_off(ts, n), kr);
        const float s = dot<D>(qm, kr);
        const float gm = fmaxf(mr, s);
        const float al = fast_exp2(mr - gm);
        mr = gm;
        const float p = fast_exp2(s - mr);
        l = l * al + p;
        load_row<D>(vb + tok_off(ts, n), vr);
#pragma unroll
        for (int j = 0; j < D; ++j) o[j] = fmaf(p, vr[j], o[j] * al);
    }
    const size_t slot = ((size_t)bh * chunks + chunk) * M + m;
    m_part[slot] = mr;
    l_part[slot] = l;
    store_row<D>(o_part + slot * D, o);
}

// Merge of the partial slots of one (b*h, m): a workgroup takes 16 latents; the 16 threads of a
// latent each fold the slots p = j, j+16, ... in order and a fixed xor-shuffle tree folds the 16
// results, so the association order depends on the slot count only (bit-reproducible).
// A slot with m = -inf is empty and contributes nothing.
template <int D>
__global__ __launch_bounds__(256) void encode_merge_kernel(
    const float *__restrict__ m_part, const float *__restrict__ l_part, const float *__restrict__ o_part,
    float *__restrict__ z, float *__restrict__ lse_enc, int BH, int M, int parts)
{
    const int j = threadIdx.x & 15;
    const int m = blockIdx.x * 16 + (threadIdx.x >> 4);
    const int bh = blockIdx.y;
    const bool live = m < M;
    const int mm = live ? m : M - 1;
    float gm = -INFINITY, l = 0.f, o[D];
#pragma unroll
    for (int i = 0; i < D; ++i) o[i] = 0.f;
    // four slots at a time: their loads are all issued before the first is folded (one memory latency per
    // batch instead of two per slot); the folds keep the slot order
    constexpr int kBatch = 4;
    for (int p0 = j; p0 < parts; p0 += 16 * kBatch) {
        float mp[kBatch], lp[kBatch], oc[kBatch][D];
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            const int p = p0 + 16 * b;
            const size_t slot = ((size_t)bh * parts + min(p, parts - 1)) * M + mm;
            mp[b] = p < parts ? m_part[slot] : -INFINITY;
            lp[b] = l_part[slot];
            load_row<D>(o_part + slot * D, oc[b]);
        }
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            if (mp[b] == -INFINITY) continue;          // an empty slot (or none): contributes nothing
            const float ng = fmaxf(gm, mp[b]);
            const float wa = fast_exp2(gm - ng);          // gm = -inf on the first live slot: weight 0
            const float wb = fast_exp2(mp[b] - ng);
            l = l * wa + lp[b] * wb;
#pragma unroll
            for (int i = 0; i < D; ++i) o[i] = o[i] * wa + oc[b][i] * wb;
            gm = ng;
        }
    }
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
        const float gm2 = __shfl_xor(gm, off);
        const float l2 = __shfl_xor(l, off);
        const float ng = fmaxf(gm, gm2);
        const float wa = (gm == -INFINITY) ? 0.f : fast_exp2(gm - ng);
        const float wb = (gm2 == -INFINITY) ? 0.f : fast_exp2(gm2 - ng);
        // both lanes of a pair must form the same sum: order the operands by lane parity
        const bool low = (j & off) == 0;
        l = low ? (l * wa + l2 * wb) : (l2 * wb + l * wa);
#pragma unroll
        for (int i = 0; i < D; ++i) {
            const float o2 = __shfl_xor(o[i], off);
            o[i] = low ? (o[i] * wa + o2 * wb) : (o2 * wb + o[i] * wa);
        }
        gm = ng;
    }
    if (!live || j != 0) return;
    const float inv = 1.f / l;
#pragma unroll
    for (int i = 0; i < D; ++i) o[i] *= inv;
    const size_t idx = (size_t)bh * M + m;
    store_row<D>(z + idx * D, o);
    lse_enc[idx] = (gm + log2f(l)) * kLn2;
}

// The same merge for few partial slots (at most kFewSlots: many (b,h) pairs of short sequences).  With
// 16 threads per latent striding over the slots most of them would idle and each would fetch whole rows
// from scattered slots; here the D / 2 threads of a latent own two columns each and walk over the slots
// in order, so a workgroup reads one contiguous piece per slot.  One maximum first (exact in any order),
// then one pass of weighted sums in slot order: the bits depend on the slot count only.
constexpr int kFewSlots = 8;   // (measured: with 16 and 32 slots in a row the slot-parallel kernels are the faster ones)
template <int D>
__global__ __launch_bounds__(256) void encode_merge_few_kernel(
    const float *__restrict__ m_part, const float *__restrict__ l_part, const float *__restrict__ o_part,
    float *__restrict__ z, float *__restrict__ lse_enc, int BH, int M, int parts)
{
    constexpr int L = D / 2, ROWS = 256 / L;
    const int j = threadIdx.x % L;
    const int m = blockIdx.x * ROWS + threadIdx.x / L;
    const int bh = blockIdx.y;
    if (m >= M) return;
    const size_t s0 = (size_t)bh * parts * M + m;   // slot p of this latent: s0 + p * M
    float gm = -INFINITY;
    for (int p = 0; p < parts; ++p) gm = fmaxf(gm, m_part[s0 + (size_t)p * M]);
    float l = 0.f, o0 = 0.f, o1 = 0.f;
    for (int p = 0; p < parts; ++p) {
        const size_t slot = s0 + (size_t)p * M;
        const float mp = m_part[slot];
        if (mp == -INFINITY) continue;              // an empty slot contributes nothing
        const float w = fast_exp2(mp - gm);
        const float2 oc = *reinterpret_cast<const float2 *>(o_part + slot * D + 2 * j);
        l = fmaf(l_part[slot], w, l);
        o0 = fmaf(oc.x, w, o0);
        o1 = fmaf(oc.y, w, o1);
    }
    const float inv = 1.f / l;
    const size_t idx = (size_t)bh * M + m;
    *reinterpret_cast<float2 *>(z + idx * D + 2 * j) = make_float2(o0 * inv, o1 * inv);
    if (j == 0) lse_enc[idx] = (gm + log2f(l)) * kLn2;
}

// ---------------------------------------------------------------------------------------
// Per-token pass over the latents.  MODE 0: decode, writes y.  MODE 1: backward statistics,
// writes lse_dec2[n] = log2 sum_m 2^S2[m][n] and delta[n] = <dY_n, Y_n>.
// ---------------------------------------------------------------------------------------
template <typename T, int D, int MODE>
__global__ __launch_bounds__(kTokenBlock) void token_pass_kernel(
    const T *__restrict__ q, const T *__restrict__ k, const float *__restrict__ z,
    T *__restrict__ y, const T *__restrict__ dy, float *__restrict__ lse_dec2, float *__restrict__ delta,
    TokStride ts, int H, int N, int M, float c2, int y_f32)
{
    // y_f32 (MODE 0, 16-bit T): y points to fp32 rows (flare_shape.y_f32)
    const int n = blockIdx.x * kTokenBlock + threadIdx.x;
    const int bh = blockIdx.y, h = bh % H;
    const bool valid = n < N;
    const size_t row = (size_t)bh * N + (valid ? n : N - 1);                     // index of the per-token scalars
    const size_t trow = tok_base(ts, bh, H) + tok_off(ts, (valid ? n : N - 1));  // first element of the token's row
    float kn[D];
    load_row<D>(k + trow, kn);
#pragma unroll
    for (int j = 0; j < D; ++j) kn[j] *= c2;
    const T *qh = q + (size_t)h * ts.sq;
    const float *zb = z + (size_t)bh * M * D;

    float mr = -INFINITY, l = 0.f, acc[D];
#pragma unroll
    for (int j = 0; j < D; ++j) acc[j] = 0.f;
    int m = 0;
    for (; m + kGroup <= M; m += kGroup) {
        float s[kGroup];
        float gm = mr;
#pragma unroll
        for (int t = 0; t < kGroup; ++t) {
            float qr[D];
            load_row<D>(qh + (size_t)(m + t) * D, qr);
            s[t] = dot<D>(kn, qr);
            gm = fmaxf(gm, s[t]);
        }
        const float al = fast_exp2(mr - gm);
        mr = gm;
        l *= al;
#pragma unroll
        for (int j = 0; j < D; ++j) acc[j] *= al;
#pragma unroll
        for (int t = 0; t < kGroup; ++t) {
            const float p = fast_exp2(s[t] - mr);
            l += p;
            float zr[D];
            load_row<D>(zb + (size_t)(m + t) * D, zr);
#pragma unroll
            for (int j = 0; j < D; ++j) acc[j] = fmaf(p, zr[j], acc[j]);
        }
    }
    for (; m < M; ++m) {
        float qr[D], zr[D];
        load_row<D>(qh + (size_t)m * D, qr);
        const float s = dot<D>(kn, qr);
        const float gm = fmaxf(mr, s);
        const float al = fast_exp2(mr - gm);
        mr = gm;
        const float p = fast_exp2(s - mr);
        l = l * al + p;
        load_row<D>(zb + (size_t)m * D, zr);
#pragma unroll
        for (int j = 0; j < D; ++j) acc[j] = fmaf(p, zr[j], acc[j] * al);
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int j = 0; j < D; ++j) acc[j] *= inv;
    if (!valid) return;
    if constexpr (MODE == 0) {
        if (sizeof(T) == 2 && y_f32) store_row<D>(reinterpret_cast<float *>(y) + trow, acc);
        else store_row<D>(y + trow, acc);
        if (lse_dec2) lse_dec2[row] = (mr + log2f(l)) * kLn2;   // optional saved statistic, natural log
    } else {
        float g[D];
        load_row<D>(dy + trow, g);
        lse_dec2[row] = mr + log2f(l);
        delta[row] = dot<D>(g, acc);
    }
}

// Token statistics of the backward from what the forward saved: delta[n] = <dY_n, Y_n> with the
// stored Y, lse_dec2[n] = lse_dec[n] * log2(e).  thread = one token row of one head, numbered in
// the memory order of the token tensors so that a wave reads consecutive rows; purely HBM-bound.
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_prep_kernel(
    const T *__restrict__ y, const T *__restrict__ dy, const float *__restrict__ lse_dec,
    float *__restrict__ lse_dec2, float *__restrict__ delta, bool head_fastest, int H, int N, size_t rows)
{
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= rows) return;
    const size_t trow = t * D;     // both layouts are dense: row t of the tensor as it lies in memory
    size_t row = t;                // index into the [B][H][N] statistics
    if (head_fastest) {            // t = (b*N + n)*H + h
        const size_t bn = t / H, h = t % H, b = bn / N, n = bn % N;
        row = (b * H + h) * N + n;
    }
    float a[D], g[D];
    load_row<D>(y + trow, a);
    load_row<D>(dy + trow, g);
    delta[row] = dot<D>(a, g);
    lse_dec2[row] = lse_dec[row] * kLog2e;
}

// The same from the forward's fp32 y (flare_shape.y_f32): delta[n] = <dY_n, Y_n> with an unrounded Y.
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_prep_y32_kernel(
    const float *__restrict__ y, const T *__restrict__ dy, float *__restrict__ delta, bool head_fastest, int H, int N,
    size_t rows)
{
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= rows) return;
    size_t row = t;
    if (head_fastest) {
        const size_t bn = t / H, h = t % H, b = bn / N, n = bn % N;
        row = (b * H + h) * N + n;
    }
    float a[D], g[D];
    load_row<D>(y + t * D, a);
    load_row<D>(dy + t * D, g);
    if constexpr (sizeof(T) == 2) {
        // The matrix-core kernels take dY as a bf16 operand (fp16 storage is rounded to bf16 when read), and
        // c - delta = <dY_n, Z_m - Y_n> only cancels if delta is formed from the same rounded values.
#pragma unroll
        for (int i = 0; i < D; ++i) {
            uint32_t u = __float_as_uint(g[i]);
            u += 0x7fffu + ((u >> 16) & 1u);
            g[i] = __uint_as_float(u & 0xffff0000u);
        }
    }
    delta[row] = dot<D>(a, g);
}

// ---------------------------------------------------------------------------------------
// dZ partials: thread = latent m; dZ[m] += R[n][m] dY[n] over the chunk's tokens.
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kLatentBlock) void dz_partial_kernel(
    const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ dy,
    const float *__restrict__ lse_dec2, float *__restrict__ dz_part,
    TokStride ts, int H, int N, int M, int chunk_len, int chunks, float c2, RowTouch touch)
{
    const int m = blockIdx.z * kLatentBlock + threadIdx.x;
    if (m >= M) return;
    const int bh = blockIdx.y, h = bh % H, chunk = blockIdx.x;
    float qm[D];
    load_row<D>(q + (size_t)h * ts.sq + (size_t)m * D, qm);
#pragma unroll
    for (int j = 0; j < D; ++j) qm[j] *= c2;
    const T *kb = k + tok_base(ts, bh, H);
    const T *gb = dy + tok_base(ts, bh, H);
    const float *lb = lse_dec2 + (size_t)bh * N;
    const int n0 = chunk * chunk_len;
    const int n1 = min(N, n0 + chunk_len);
    float acc[D];
#pragma unroll
    for (int j = 0; j < D; ++j) acc[j] = 0.f;
    __shared__ float sink[kLatentBlock];
    auto token = [&](int n) {
        float kr[D], g[D];
        load_row<D>(kb + tok_off(ts, n), kr);
        const float r = fast_exp2(dot<D>(qm, kr) - lb[n]);
        load_row<D>(gb + tok_off(ts, n), g);
#pragma unroll
        for (int j = 0; j < D; ++j) acc[j] = fmaf(r, g[j], acc[j]);
    };
    int n = n0;
    for (; n + kGroup <= n1; n += kGroup) {   // whole groups: the touch is unconditional, no branch inside the group
        touch_rows<T>(touch, tok_base(ts, bh, H), ts, n, N, sink);
#pragma unroll
        for (int t = 0; t < kGroup; ++t) token(n + t);
    }
    for (; n < n1; ++n) token(n);
    store_row<D>(dz_part + (((size_t)bh * chunks + chunk) * M + m) * D, acc);
}

// Fixed-order sum of partial slots, shared by dZ and dQ.  A workgroup takes 16 rows (latents); the
// 16 threads of a row each add the slots j, j+16, ... in order and a fixed xor-shuffle tree adds
// the 16 results, so the association order depends on the slot count only.
// Slot s of output row (outer, m) lives at  part[((s / inner) * stride_o + outer) * inner + s % inner][m]
// with stride_o = outer count:  dZ: outer = b*h, one group of `inner` slots;  dQ: outer = h, the
// slots of all batch items b (groups of `inner` partials each), i.e. the batch sum in b order.
template <int D>
__device__ __forceinline__ void sum_slots(const float *__restrict__ part, int outer, int n_outer, int groups,
                                          int inner, int M, int m, int j, float (&acc)[D])
{
#pragma unroll
    for (int i = 0; i < D; ++i) acc[i] = 0.f;
    const int total = groups * inner;
    // four slots at a time: their loads are all issued before the first is added; the sums keep the slot order
    constexpr int kBatch = 4;
    for (int s0 = j; s0 < total; s0 += 16 * kBatch) {
        float t[kBatch][D];
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            const int s = min(s0 + 16 * b, total - 1);
            const size_t slot = ((size_t)(s / inner) * n_outer + outer) * inner + (s % inner);
            load_row<D>(part + (slot * M + m) * D, t[b]);
        }
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            if (s0 + 16 * b < total) {
#pragma unroll
                for (int i = 0; i < D; ++i) acc[i] += t[b][i];
            }
        }
    }
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
        const bool low = (j & off) == 0;
#pragma unroll
        for (int i = 0; i < D; ++i) {
            const float o = __shfl_xor(acc[i], off);
            acc[i] = low ? (acc[i] + o) : (o + acc[i]);
        }
    }
}

// dZ[b*h][m] = sum of its partial slots; eps[m] = <dZ_m, Z_m>.
template <int D>
__global__ __launch_bounds__(256) void dz_merge_kernel(
    const float *__restrict__ dz_part, const float *__restrict__ z,
    float *__restrict__ dz, float *__restrict__ eps, int BH, int M, int parts, int round_bf16,
    const float *__restrict__ ld_range, const float *__restrict__ lse_enc, int *__restrict__ plan, int force_two)
{
    const int j = threadIdx.x & 15;
    const int m = blockIdx.x * 16 + (threadIdx.x >> 4);
    const int bh = blockIdx.y;
    // matrix-core path: which variant of the next kernels runs for this (b,h) (every workgroup works it out for
    // itself: the one-exponential variant wants dZ scaled, see bwd_one_exp_ok); one more workgroup records it
    __shared__ float plan_red[16];
    const bool one_exp = plan != nullptr && bwd_one_exp_ok(ld_range, lse_enc, bh, parts, M, force_two, plan_red);
    if (plan != nullptr && blockIdx.x == gridDim.x - 1) {
        if (threadIdx.x == 0) plan[bh] = one_exp ? 1 : 0;
        return;
    }
    const bool live = m < M;
    float acc[D], zr[D];
    sum_slots<D>(dz_part, bh, BH, 1, parts, M, live ? m : M - 1, j, acc);
    if (!live || j != 0) return;
    const size_t idx = (size_t)bh * M + m;
    if (one_exp) {
        const float em = exp2f(-lse_enc[idx] * 1.4426950408889634f);
#pragma unroll
        for (int i = 0; i < D; ++i) acc[i] *= em;
    }
    if (round_bf16) {
        // The matrix-core kernels take dZ as a bf16 operand.  Rounding it here, before eps is formed,
        // keeps a[m][n] = <dZ_m, V_n - Z_m> an exact expression in the rounded dZ (eps and the products
        // see the same values), instead of leaving <V_n, rounding error> uncancelled in every score.
#pragma unroll
        for (int i = 0; i < D; ++i) {
            uint32_t u = __float_as_uint(acc[i]);
            u += 0x7fffu + ((u >> 16) & 1u);
            acc[i] = __uint_as_float(u & 0xffff0000u);
        }
    }
    load_row<D>(z + idx * D, zr);
    store_row<D>(dz + idx * D, acc);
    eps[idx] = dot<D>(acc, zr);
}

// Few slots (at most kFewSlots in all): the D / 2 threads of a row own two columns each and add the slots in
// order (see encode_merge_few_kernel); same slot addressing as sum_slots.
template <int D>
__device__ __forceinline__ float2 sum_slots_few(const float *__restrict__ part, int outer, int n_outer, int groups,
                                                int inner, int M, int m, int j)
{
    float a0 = 0.f, a1 = 0.f;
    for (int g = 0; g < groups; ++g)
        for (int i = 0; i < inner; ++i) {
            const size_t slot = ((size_t)g * n_outer + outer) * inner + i;
            const float2 t = *reinterpret_cast<const float2 *>(part + (slot * M + m) * D + 2 * j);
            a0 += t.x;
            a1 += t.y;
        }
    return make_float2(a0, a1);
}

template <int D>
__global__ __launch_bounds__(256) void dz_merge_few_kernel(
    const float *__restrict__ dz_part, const float *__restrict__ z,
    float *__restrict__ dz, float *__restrict__ eps, int BH, int M, int parts, int round_bf16,
    const float *__restrict__ ld_range, const float *__restrict__ lse_enc, int *__restrict__ plan, int force_two)
{
    constexpr int L = D / 2, ROWS = 256 / L;
    const int j = threadIdx.x % L;
    const int m = blockIdx.x * ROWS + threadIdx.x / L;
    const int bh = blockIdx.y;
    __shared__ float plan_red[16];                   // as in dz_merge_kernel
    const bool one_exp = plan != nullptr && bwd_one_exp_ok(ld_range, lse_enc, bh, parts, M, force_two, plan_red);
    if (plan != nullptr && blockIdx.x == gridDim.x - 1) {
        if (threadIdx.x == 0) plan[bh] = one_exp ? 1 : 0;
        return;
    }
    const bool live = m < M;                         // no early exit: the row's lanes meet in the shuffles below
    float2 a = sum_slots_few<D>(dz_part, bh, BH, 1, parts, M, live ? m : M - 1, j);
    if (one_exp) {                                   // the one-exponential kernels take dZ scaled by 2^-lse_enc2[m]
        const float em = exp2f(-lse_enc[(size_t)bh * M + (live ? m : M - 1)] * 1.4426950408889634f);
        a.x *= em;
        a.y *= em;
    }
    if (round_bf16) {                                // as in dz_merge_kernel: round before eps is formed
        uint32_t u = __float_as_uint(a.x);
        u += 0x7fffu + ((u >> 16) & 1u);
        a.x = __uint_as_float(u & 0xffff0000u);
        u = __float_as_uint(a.y);
        u += 0x7fffu + ((u >> 16) & 1u);
        a.y = __uint_as_float(u & 0xffff0000u);
    }
    const size_t idx = (size_t)bh * M + (live ? m : M - 1);
    const float2 zr = *reinterpret_cast<const float2 *>(z + idx * D + 2 * j);
    float e = fmaf(a.y, zr.y, a.x * zr.x);
#pragma unroll
    for (int off = 1; off < L; off <<= 1) {          // fixed tree over the row's lanes (L is a power of two)
        const float o = __shfl_xor(e, off);
        e = ((j & off) == 0) ? (e + o) : (o + e);
    }
    if (!live) return;
    *reinterpret_cast<float2 *>(dz + idx * D + 2 * j) = a;
    if (j == 0) eps[idx] = e;
}

template <int D>
__global__ __launch_bounds__(256) void dq_reduce_few_kernel(
    const float *__restrict__ dq_part, float *__restrict__ dq, int B, int H, int M, int parts, float scale)
{
    constexpr int L = D / 2, ROWS = 256 / L;
    const int j = threadIdx.x % L;
    const int m = blockIdx.x * ROWS + threadIdx.x / L;
    const int h = blockIdx.y;
    if (m >= M) return;
    const float2 a = sum_slots_few<D>(dq_part, h, H, B, parts, M, m, j);
    *reinterpret_cast<float2 *>(dq + ((size_t)h * M + m) * D + 2 * j) = make_float2(a.x * scale, a.y * scale);
}

// ---------------------------------------------------------------------------------------
// dQ partials: thread = latent m;  dQ[m] += dS[m][n] k[n] over the chunk's tokens, with
// dS[m][n] = P[m][n](<dZ_m,V_n> - eps_m) + R[n][m](<dY_n,Z_m> - delta_n).
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kLatentBlock) void dq_partial_kernel(
    const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v, const T *__restrict__ dy,
    const float *__restrict__ z, const float *__restrict__ lse_enc, const float *__restrict__ dz,
    const float *__restrict__ eps, const float *__restrict__ lse_dec2, const float *__restrict__ delta,
    float *__restrict__ dq_part, TokStride ts, int H, int N, int M, int chunk_len, int chunks, float c2,
    RowTouch touch)
{
    const int m = blockIdx.z * kLatentBlock + threadIdx.x;
    if (m >= M) return;
    const int bh = blockIdx.y, h = bh % H, chunk = blockIdx.x;
    float qm[D], zm[D], dzm[D], acc[D];
    load_row<D>(q + (size_t)h * ts.sq + (size_t)m * D, qm);
    load_row<D>(z + ((size_t)bh * M + m) * D, zm);
    load_row<D>(dz + ((size_t)bh * M + m) * D, dzm);
#pragma unroll
    for (int j = 0; j < D; ++j) { qm[j] *= c2; acc[j] = 0.f; }
    const float le2 = lse_enc[(size_t)bh * M + m] * kLog2e;
    const float ep = eps[(size_t)bh * M + m];
    const T *kb = k + tok_base(ts, bh, H);
    const T *vb = v + tok_base(ts, bh, H);
    const T *gb = dy + tok_base(ts, bh, H);
    const float *lb = lse_dec2 + (size_t)bh * N;
    const float *db = delta + (size_t)bh * N;
    const int n0 = chunk * chunk_len;
    const int n1 = min(N, n0 + chunk_len);
    __shared__ float sink[kLatentBlock];
    auto token = [&](int n) {
        float kr[D], vr[D], g[D];
        load_row<D>(kb + tok_off(ts, n), kr);
        load_row<D>(vb + tok_off(ts, n), vr);
        load_row<D>(gb + tok_off(ts, n), g);
        const float s2 = dot<D>(qm, kr);
        const float p = fast_exp2(s2 - le2);
        const float r = fast_exp2(s2 - lb[n]);
        const float ds = p * (dot<D>(dzm, vr) - ep) + r * (dot<D>(zm, g) - db[n]);
#pragma unroll
        for (int j = 0; j < D; ++j) acc[j] = fmaf(ds, kr[j], acc[j]);
    };
    int n = n0;
    for (; n + kGroup <= n1; n += kGroup) {   // whole groups: the touch is unconditional, no branch inside the group
        touch_rows<T>(touch, tok_base(ts, bh, H), ts, n, N, sink);
#pragma unroll
        for (int t = 0; t < kGroup; ++t) token(n + t);
    }
    for (; n < n1; ++n) token(n);
    store_row<D>(dq_part + (((size_t)bh * chunks + chunk) * M + m) * D, acc);
}

// dq_lat[h][m] = scale * sum over batch items and partial slots (fixed order, see sum_slots).
template <int D>
__global__ __launch_bounds__(256) void dq_reduce_kernel(
    const float *__restrict__ dq_part, float *__restrict__ dq, int B, int H, int M, int parts, float scale)
{
    const int j = threadIdx.x & 15;
    const int m = blockIdx.x * 16 + (threadIdx.x >> 4);
    const int h = blockIdx.y;
    const bool live = m < M;
    float acc[D];
    sum_slots<D>(dq_part, h, H, B, parts, M, live ? m : M - 1, j, acc);
    if (!live || j != 0) return;
#pragma unroll
    for (int i = 0; i < D; ++i) acc[i] *= scale;
    store_row<D>(dq + ((size_t)h * M + m) * D, acc);
}

// ---------------------------------------------------------------------------------------
// dK, dV: thread = token n;  dK_n = scale * sum_m dS[m][n] q_m,  dV_n = sum_m P[m][n] dZ_m.
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kTokenBlock) void dkdv_kernel(
    const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v, const T *__restrict__ dy,
    const float *__restrict__ z, const float *__restrict__ lse_enc, const float *__restrict__ dz,
    const float *__restrict__ eps, const float *__restrict__ lse_dec2, const float *__restrict__ delta,
    T *__restrict__ dk, T *__restrict__ dv, TokStride ts, int H, int N, int M, float scale)
{
    const int n = blockIdx.x * kTokenBlock + threadIdx.x;
    const int bh = blockIdx.y, h = bh % H;
    const bool valid = n < N;
    const size_t row = (size_t)bh * N + (valid ? n : N - 1);
    const size_t trow = tok_base(ts, bh, H) + tok_off(ts, (valid ? n : N - 1));
    const float c2 = scale * kLog2e;
    float kn[D], vn[D], g[D], ak[D], av[D];
    load_row<D>(k + trow, kn);
    load_row<D>(v + trow, vn);
    load_row<D>(dy + trow, g);
#pragma unroll
    for (int j = 0; j < D; ++j) { kn[j] *= c2; ak[j] = 0.f; av[j] = 0.f; }
    const float ld2 = lse_dec2[row];
    const float dl = delta[row];
    const T *qh = q + (size_t)h * ts.sq;
    const float *zb = z + (size_t)bh * M * D;
    const float *dzb = dz + (size_t)bh * M * D;
    const float *leb = lse_enc + (size_t)bh * M;
    const float *epb = eps + (size_t)bh * M;
    for (int m = 0; m < M; ++m) {
        float qr[D], zr[D], dzr[D];
        load_row<D>(qh + (size_t)m * D, qr);
        load_row<D>(zb + (size_t)m * D, zr);
        load_row<D>(dzb + (size_t)m * D, dzr);
        const float s2 = dot<D>(kn, qr);
        const float p = fast_exp2(s2 - leb[m] * kLog2e);
        const float r = fast_exp2(s2 - ld2);
        const float ds = p * (dot<D>(dzr, vn) - epb[m]) + r * (dot<D>(zr, g) - dl);
#pragma unroll
        for (int j = 0; j < D; ++j) {
            ak[j] = fmaf(ds, qr[j], ak[j]);
            av[j] = fmaf(p, dzr[j], av[j]);
        }
    }
    if (!valid) return;
#pragma unroll
    for (int j = 0; j < D; ++j) ak[j] *= scale;
    store_row<D>(dk + trow, ak);
    store_row<D>(dv + trow, av);
}

// ---- workspace carving --------------------------------------------------------------------
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct BwdWs { float *lse_dec2, *delta, *part, *dz, *eps, *ld_range; int *plan; void *tok_part; float *acc32; };

// `slots` = partial slots per (b,h) the shared partial buffer must hold
size_t bwd_layout(const flare_shape &s, int slots, void *ws, BwdWs *out)
{
    const size_t BH = (size_t)s.B * s.H;
    size_t off = 0;
    char *base = static_cast<char *>(ws);
    if (out) out->lse_dec2 = reinterpret_cast<float *>(base + off);
    off += align256(BH * s.N * 4);
    if (out) out->delta = reinterpret_cast<float *>(base + off);
    off += align256(BH * s.N * 4);
    if (out) out->part = reinterpret_cast<float *>(base + off);
    off += align256(BH * slots * s.M * s.d * 4);
    if (out) out->dz = reinterpret_cast<float *>(base + off);
    off += align256(BH * s.M * s.d * 4);
    if (out) out->eps = reinterpret_cast<float *>(base + off);
    off += align256(BH * s.M * 4);
    if (out) out->ld_range = reinterpret_cast<float *>(base + off);
    off += align256(BH * slots * 2 * 4);
    if (out) out->plan = reinterpret_cast<int *>(base + off);
    off += align256(BH * 4);
    if (mfma_supported(s)) {   // only shapes with more than 256 latents on the matrix-core path use these
        if (out) out->tok_part = base + off;
        off += mfma_tok_part_bytes(s);
        if (out) out->acc32 = reinterpret_cast<float *>(base + off);
        off += mfma_dkdv_acc_bytes(s);
    } else if (out) {
        out->tok_part = nullptr;
        out->acc32 = nullptr;
    }
    return off;
}

inline int check_launch() { return hipGetLastError() == hipSuccess ? FLARE_OK : FLARE_ELAUNCH; }

inline int bwd_slots(const flare_shape &s, const ValuPlan &plan)
{
    int mf = 0;
    if (mfma_supported(s)) {
        mf = mfma_plan(s).parts;
        if (mfma_dq_parts(s) > mf) mf = mfma_dq_parts(s);
        if (mfma_dkdv_blocks(s) > mf) mf = mfma_dkdv_blocks(s);
    }
    return plan.bwd.chunks > mf ? plan.bwd.chunks : mf;
}

template <typename T, int D>
int encode_impl(const flare_shape &s, const T *q, const T *k, const T *v, float *z, float *lse_enc,
                float scale, void *ws, hipStream_t stream)
{
    const ValuPlan plan = valu_plan(s);
    float *m_part, *l_part, *o_part;
    valu_fwd_layout(s, plan.enc, ws, &m_part, &l_part, &o_part);
    const int BH = s.B * s.H;
    const int lat_blocks = (s.M + kLatentBlock - 1) / kLatentBlock;
    {
        LaunchTimer t(KID_ENCODE_PARTIAL, stream);
        encode_partial_kernel<T, D><<<dim3(plan.enc.chunks, BH, lat_blocks), kLatentBlock, 0, stream>>>(
            q, k, v, m_part, l_part, o_part, tok_stride(s), s.H, s.N, s.M, plan.enc.chunk_len, plan.enc.chunks, scale * kLog2e,
            RowTouch{addr(k), addr(v), addr(k), 0, 0});
    }
    if (check_launch() != FLARE_OK) return FLARE_ELAUNCH;
    return launch_encode_merge(s, m_part, l_part, o_part, z, lse_enc, plan.enc.chunks, stream);
}

template <typename T, int D>
int decode_impl(const flare_shape &s, const T *q, const T *k, const float *z, T *y, float *lse_dec, float scale,
                hipStream_t stream)
{
    LaunchTimer t(KID_DECODE, stream);
    token_pass_kernel<T, D, 0><<<dim3((s.N + kTokenBlock - 1) / kTokenBlock, s.B * s.H), kTokenBlock, 0, stream>>>(
        q, k, z, y, nullptr, lse_dec, nullptr, tok_stride(s), s.H, s.N, s.M, scale * kLog2e, s.y_f32);
    return check_launch();
}

template <typename T, int D>
int backward_impl(const flare_shape &s, const T *q, const T *k, const T *v, const T *y, const float *lse_dec,
                  const T *dy, const float *z, const float *lse_enc, float *dq, T *dk, T *dv, float scale, void *ws,
                  hipStream_t stream)
{
    const ValuPlan plan = valu_plan(s);
    const bool mf = mfma_supported(s);          // matrix-core kernels where they exist
    const int dz_parts = mf ? mfma_plan(s).parts : plan.bwd.chunks;
    BwdWs w;
    bwd_layout(s, bwd_slots(s, plan), ws, &w);
    const int BH = s.B * s.H;
    const float c2 = scale * kLog2e;
    const TokStride ts = tok_stride(s);
    const int lat_blocks = (s.M + kLatentBlock - 1) / kLatentBlock;
    const dim3 tok_grid((s.N + kTokenBlock - 1) / kTokenBlock, BH);
    const dim3 lat_grid(plan.bwd.chunks, BH, lat_blocks);
    // token statistics: from what the forward saved, or recomputed.  On the matrix-core path the
    // saved ones need no pass of their own: the dZ kernel forms delta while it streams dY, and every
    // kernel reads lse_dec itself, scaled to log2 units.
    // With bf16 storage (or bf16 softmax weights behind fp16 storage: the matrix-core path) and d < 16,
    // delta = <dY_n, Y_n> from the forward's y is too coarse (few terms, and c - delta cancels): such
    // shapes recompute the statistics even when y and lse_dec are given.
    // The same with at most one tile of tokens: every dot product and sum is short, nothing averages the
    // rounding of y out (dq_lat, dK 2.1-2.4e-2 from the saved y, 8e-3 recomputed), and the recomputation costs
    // nothing at that size.
    // (at most one tile of tokens: any 16-bit y, also fp16 on the fp32 kernels)
    // Likewise with fewer tokens than latents: a latent's gradient is then a sum over few tokens (300 tokens, 1000
    // latents, d = 32: dq_lat 1.9e-2 ... 2.1e-2 from the saved y, 9e-3 recomputed).
    const bool bf16_weights = s.dtype == FLARE_BF16 || (s.dtype == FLARE_F16 && mf);
    const bool coarse_y = s.dtype != FLARE_F32 && ((bf16_weights && s.d < 16) || s.N <= 32 || s.N < s.M) &&
                          !(s.y_f32 && mf);   // an fp32 y is not coarse (the fp32 kernels, which take the
                                              // 16-bit shapes of fewer than 16 tokens, never read it: they recompute)
    const bool saved = y && lse_dec && !coarse_y;
    const bool fused = saved && mf && mfma_dkdv_supported(s);   // every later kernel is a matrix-core one
    const float *ld = fused ? lse_dec : w.lse_dec2;
    const float ld_mul = fused ? kLog2e : 1.f;
    // delta from the fp32 y: at d <= 8 inside the dZ kernel like from a 16-bit y, else by a pass of its own
    const bool y32 = fused && s.y_f32 && s.d > 8;
    if (y32) {
        LaunchTimer t(KID_BWD_PREP, stream);
        const size_t rows = (size_t)BH * s.N;
        bwd_prep_y32_kernel<T, D><<<(unsigned)((rows + 255) / 256), 256, 0, stream>>>(
            reinterpret_cast<const float *>(y), dy, w.delta, s.layout == FLARE_BNHD, s.H, s.N, rows);
    } else if (fused) {
    } else if (saved) {
        LaunchTimer t(KID_BWD_PREP, stream);
        const size_t rows = (size_t)BH * s.N;
        bwd_prep_kernel<T, D><<<(unsigned)((rows + 255) / 256), 256, 0, stream>>>(
            y, dy, lse_dec, w.lse_dec2, w.delta, s.layout == FLARE_BNHD, s.H, s.N, rows);
    } else if (mf) {
        const int rc = mfma_token_stats(s, q, k, z, dy, w.lse_dec2, w.delta, scale, w.tok_part, stream);
        if (rc != FLARE_OK) return rc;
    } else {
        LaunchTimer t(KID_BWD_TOKEN_STATS, stream);
        token_pass_kernel<T, D, 1><<<tok_grid, kTokenBlock, 0, stream>>>(q, k, z, nullptr, dy, w.lse_dec2, w.delta,
                                                                         ts, s.H, s.N, s.M, c2, 0);
    }
    if (check_launch() != FLARE_OK) return FLARE_ELAUNCH;
    if (mf) {
        int rc = mfma_dz_partial(s, q, k, dy, ld, ld_mul, (fused && !y32) ? y : nullptr,
                                 (fused && !y32) ? w.delta : nullptr, w.ld_range, w.part, scale, stream);
        if (rc != FLARE_OK) return rc;
    } else {
        {
            LaunchTimer t(KID_BWD_DZ_PARTIAL, stream);
            dz_partial_kernel<T, D><<<lat_grid, kLatentBlock, 0, stream>>>(q, k, dy, w.lse_dec2, w.part, ts, s.H,
                                                                           s.N, s.M, plan.bwd.chunk_len, plan.bwd.chunks,
                                                                           c2, RowTouch{addr(k), addr(dy), addr(k), addr(w.lse_dec2), addr(w.lse_dec2)});
        }
        if (check_launch() != FLARE_OK) return FLARE_ELAUNCH;
    }
    constexpr int kFewRows = 256 / (D / 2);   // rows per workgroup of the few-slot merge kernels
    {
        LaunchTimer t(KID_BWD_DZ_MERGE, stream);
        if (dz_parts <= kFewSlots)
            dz_merge_few_kernel<D><<<dim3((s.M + kFewRows - 1) / kFewRows + (mf ? 1 : 0), BH), 256, 0, stream>>>(
                w.part, z, w.dz, w.eps, BH, s.M, dz_parts, mf ? 1 : 0, w.ld_range, lse_enc, mf ? w.plan : nullptr,
                (s.variant & FLARE_VARIANT_TWO_EXP) ? 1 : 0);
        else
            dz_merge_kernel<D><<<dim3((s.M + 15) / 16 + (mf ? 1 : 0), BH), 256, 0, stream>>>(
                w.part, z, w.dz, w.eps, BH, s.M, dz_parts, mf ? 1 : 0, w.ld_range, lse_enc, mf ? w.plan : nullptr,
                (s.variant & FLARE_VARIANT_TWO_EXP) ? 1 : 0);
    }
    if (check_launch() != FLARE_OK) return FLARE_ELAUNCH;
    int dq_parts = plan.bwd.chunks;
    const bool dq_fused = mf && mfma_dkdv_supported(s) && mfma_dq_fused(s);   // dQ comes out of the dK/dV kernel
    if (dq_fused) {
        dq_parts = mfma_dkdv_blocks(s);
    } else if (mf) {
        dq_parts = mfma_dq_parts(s);
        const int rc = mfma_dq_partial(s, q, k, v, dy, z, lse_enc, w.dz, w.eps, ld, w.delta, ld_mul, w.plan, w.part,
                                       scale, stream);   // each (b,h) slice by the variant its plan names
        if (rc != FLARE_OK) return rc;
    } else {
        LaunchTimer t(KID_BWD_DQ_PARTIAL, stream);
        dq_partial_kernel<T, D><<<lat_grid, kLatentBlock, 0, stream>>>(q, k, v, dy, z, lse_enc, w.dz, w.eps,
                                                                       w.lse_dec2, w.delta, w.part, ts, s.H, s.N, s.M,
                                                                       plan.bwd.chunk_len, plan.bwd.chunks, c2,
                                                                       RowTouch{addr(k), addr(v), addr(dy), addr(w.lse_dec2), addr(w.delta)});
    }
    if (check_launch() != FLARE_OK) return FLARE_ELAUNCH;
    auto reduce_dq = [&]() -> int {
        LaunchTimer t(KID_BWD_DQ_REDUCE, stream);
        // shared latents: one gradient for all heads, summed over (b, h) in that fixed order
        const int groups = s.shared_latents ? BH : s.B, outers = s.shared_latents ? 1 : s.H;
        if ((long long)groups * dq_parts <= kFewSlots)
            dq_reduce_few_kernel<D><<<dim3((s.M + kFewRows - 1) / kFewRows, outers), 256, 0, stream>>>(
                w.part, dq, groups, outers, s.M, dq_parts, scale);
        else
            dq_reduce_kernel<D><<<dim3((s.M + 15) / 16, outers), 256, 0, stream>>>(w.part, dq, groups, outers, s.M,
                                                                                 dq_parts, scale);
        return check_launch();
    };
    if (!dq_fused) {
        const int rc = reduce_dq();
        if (rc != FLARE_OK) return rc;
    }
    if (mf && mfma_dkdv_supported(s)) {
        const bool chunked = mfma_dkdv_acc_bytes(s) != 0;   // more than 256 latents: one pass per chunk
        for (int m0 = 0; m0 < s.M; m0 += 256) {   // each (b,h) slice by the variant its plan names
            const int rc = mfma_dkdv(s, q, k, v, dy, z, lse_enc, w.dz, w.eps, ld, w.delta, ld_mul, w.plan, dk, dv,
                                     chunked ? w.acc32 : nullptr, dq_fused ? w.part : nullptr, m0, scale, stream);
            if (rc != FLARE_OK) return rc;
        }
        return dq_fused ? reduce_dq() : FLARE_OK;
    }
    {
        LaunchTimer t(KID_BWD_DKDV, stream);
        dkdv_kernel<T, D><<<tok_grid, kTokenBlock, 0, stream>>>(q, k, v, dy, z, lse_enc, w.dz, w.eps, w.lse_dec2,
                                                                w.delta, dk, dv, ts, s.H, s.N, s.M, scale);
    }
    return check_launch();
}

// Dispatch on (dtype, d) to the template instances.
#define FLARE_DISPATCH(s, CALL)                                                   \
    do {                                                                          \
        if ((s).dtype == FLARE_F32) {                                             \
            typedef float T;                                                      \
            switch ((s).d) {                                                      \
                case 4: { constexpr int D = 4; return CALL; }                     \
                case 8: { constexpr int D = 8; return CALL; }                     \
                case 16: { constexpr int D = 16; return CALL; }                   \
                case 32: { constexpr int D = 32; return CALL; }                   \
            }                                                                     \
        } else if ((s).dtype == FLARE_F16) {                                      \
            typedef f16_t T;                                                      \
            switch ((s).d) {                                                      \
                case 4: { constexpr int D = 4; return CALL; }                     \
                case 8: { constexpr int D = 8; return CALL; }                     \
                case 16: { constexpr int D = 16; return CALL; }                   \
                case 32: { constexpr int D = 32; return CALL; }                   \
            }                                                                     \
        } else {                                                                  \
            typedef bf16_t T;                                                     \
            switch ((s).d) {                                                      \
                case 4: { constexpr int D = 4; return CALL; }                     \
                case 8: { constexpr int D = 8; return CALL; }                     \
                case 16: { constexpr int D = 16; return CALL; }                   \
                case 32: { constexpr int D = 32; return CALL; }                   \
            }                                                                     \
        }                                                                         \
        return FLARE_EUNSUPPORTED;                                                \
    } while (0)

}  // namespace

size_t valu_fwd_layout(const flare_shape &s, const Split &sp, void *ws, float **m_part, float **l_part,
                       float **o_part)
{
    const size_t slots = (size_t)s.B * s.H * sp.chunks * s.M;
    size_t off = 0;
    char *base = static_cast<char *>(ws);
    if (m_part) *m_part = reinterpret_cast<float *>(base + off);
    off += align256(slots * 4);
    if (l_part) *l_part = reinterpret_cast<float *>(base + off);
    off += align256(slots * 4);
    if (o_part) *o_part = reinterpret_cast<float *>(base + off);
    off += align256(slots * s.d * 4);
    return off;
}

int launch_encode_merge(const flare_shape &s, const float *m_part, const float *l_part, const float *o_part,
                        float *z, float *lse_enc, int parts, hipStream_t stream)
{
    const int BH = s.B * s.H;
    const dim3 blocks((s.M + 15) / 16, BH);
    LaunchTimer t(KID_ENCODE_MERGE, stream);
    if (parts <= kFewSlots) {
#define FLARE_EMF(DD)                                                                                          \
    encode_merge_few_kernel<DD><<<dim3((s.M + 256 / (DD / 2) - 1) / (256 / (DD / 2)), BH), 256, 0, stream>>>(   \
        m_part, l_part, o_part, z, lse_enc, BH, s.M, parts)
        switch (s.d) {
            case 4: FLARE_EMF(4); break;
            case 8: FLARE_EMF(8); break;
            case 16: FLARE_EMF(16); break;
            case 32: FLARE_EMF(32); break;
            default: return FLARE_EUNSUPPORTED;
        }
#undef FLARE_EMF
        return check_launch();
    }
    switch (s.d) {
        case 4: encode_merge_kernel<4><<<blocks, 256, 0, stream>>>(m_part, l_part, o_part, z, lse_enc, BH, s.M, parts); break;
        case 8: encode_merge_kernel<8><<<blocks, 256, 0, stream>>>(m_part, l_part, o_part, z, lse_enc, BH, s.M, parts); break;
        case 16: encode_merge_kernel<16><<<blocks, 256, 0, stream>>>(m_part, l_part, o_part, z, lse_enc, BH, s.M, parts); break;
        case 32: encode_merge_kernel<32><<<blocks, 256, 0, stream>>>(m_part, l_part, o_part, z, lse_enc, BH, s.M, parts); break;
        default: return FLARE_EUNSUPPORTED;
    }
    return check_launch();
}

ValuPlan valu_plan(const flare_shape &s)
{
    ValuPlan p;
    const int BH = s.B * s.H;
    // chunks of at least 64 tokens: short sequences with few heads still spread over the chip; and of at
    // most 8192: a thread adds its chunk's terms one after the other in fp32, and the rounding of such a
    // sum grows with the square root of its length (the partial results are then combined by a tree)
    p.enc = plan_split(s.N, BH, 64, 2048);
    constexpr int kMaxChunk = 8192;
    if (p.enc.chunk_len > kMaxChunk) {
        p.enc.chunk_len = kMaxChunk;
        p.enc.chunks = (s.N + kMaxChunk - 1) / kMaxChunk;
    }
    p.bwd = p.enc;
    p.fwd_bytes = valu_fwd_layout(s, p.enc, nullptr, nullptr, nullptr, nullptr);
    p.bwd_bytes = bwd_layout(s, bwd_slots(s, p), nullptr, nullptr);
    return p;
}

int valu_encode(const flare_shape &s, const void *q, const void *k, const void *v, float *z, float *lse_enc,
                float scale, void *ws, hipStream_t stream)
{
    FLARE_DISPATCH(s, (encode_impl<T, D>(s, (const T *)q, (const T *)k, (const T *)v, z, lse_enc, scale, ws, stream)));
}
int valu_decode(const flare_shape &s, const void *q, const void *k, const float *z, void *y, float *lse_dec,
                float scale, hipStream_t stream)
{
    FLARE_DISPATCH(s, (decode_impl<T, D>(s, (const T *)q, (const T *)k, z, (T *)y, lse_dec, scale, stream)));
}
int valu_backward(const flare_shape &s, const void *q, const void *k, const void *v, const void *y,
                  const float *lse_dec, const void *dy, const float *z, const float *lse_enc, float *dq, void *dk,
                  void *dv, float scale, void *ws, hipStream_t stream)
{
    FLARE_DISPATCH(s, (backward_impl<T, D>(s, (const T *)q, (const T *)k, (const T *)v, (const T *)y, lse_dec,
                                           (const T *)dy, z, lse_enc, dq, (T *)dk, (T *)dv, scale, ws, stream)));
}

}  // namespace flare
