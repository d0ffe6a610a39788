// libflare_rates.so: micro-benchmarks of the gfx950 rates the FLARE kernels are priced against
// (copy bandwidth, vector and matrix instruction issue, and how the two share a SIMD).
// Contract in include/flare_rates.h.  Not linked into the operator's library.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "flare_rates.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum Experiment {
    E_COPY = 0,
    E_EXP, E_FMA, E_CVT, E_MAX3, E_PERM, E_DOT2, E_ADD,
    E_MFMA32, E_MFMA16,
    E_SAME32_EXP, E_SAME32_FMA, E_SAME16_EXP, E_EXP_FMA,
    E_OTHER32, E_OTHER16,
    E_TILE,
    E_F64,
    E_COUNT
};
const char *const kNames[E_COUNT] = {
    "copy",
    "v_exp_f32", "v_fma_f32", "v_cvt_pk_bf16_f32", "v_max3_f32", "v_perm_b32", "v_dot2c_f32_bf16", "v_add_f32",
    "v_mfma_f32_32x32x16_bf16", "v_mfma_f32_16x16x32_bf16",
    "same wave: 1 mfma 32x32x16 + k v_exp_f32", "same wave: 1 mfma 32x32x16 + k v_fma_f32",
    "same wave: 1 mfma 16x16x32 + k v_exp_f32", "same wave: 1 v_exp_f32 + k v_fma_f32",
    "other wave: mfma 32x32x16 wave beside exp+pack waves (param 0 both, 1 matrix only, 2 vector only)",
    "other wave: mfma 16x16x32 wave beside exp+pack waves (param 0 both, 1 matrix only, 2 vector only)",
    "softmax tile: k score mfma -> 16 exp -> 8 pack -> 2 value mfma, next tile's scores issued first",
    "fp64: param % 8 = 0 v_fma_f64, 1 v_mul_f64, 2 v_add_f64, 3 v_rsq_f64, 4 v_rcp_f64; param < 8 one dependent chain "
    "per wave (latency), 8 <= param < 16 eight independent chains (issue rate), param >= 16 as param - 16 on eight "
    "workgroups only"};

constexpr size_t kScratch = (size_t)1 << 30;   // copy experiment: 512 MiB in, 512 MiB out
constexpr int kClockSlots = 4;                 // uint64 per launch: shader and real-time ticks, start and end

#define GROUP_MFMA(n) __builtin_amdgcn_sched_group_barrier(0x008, n, 0)
#define GROUP_TRANS(n) __builtin_amdgcn_sched_group_barrier(0x400, n, 0)
#define GROUP_VALU(n) __builtin_amdgcn_sched_group_barrier(0x002, n, 0)

__device__ __forceinline__ uint32_t cvt_pk(float a, float b)
{
    f32x2 v;
    v[0] = a;
    v[1] = b;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// first wave of workgroup 0 records the two counters around its own loop
struct Clocks {
    uint64_t *slot;
    __device__ Clocks(uint64_t *s) : slot((blockIdx.x == 0 && threadIdx.x == 0) ? s : nullptr)
    {
        if (slot) {
            slot[0] = __builtin_amdgcn_s_memtime();
            slot[1] = __builtin_amdgcn_s_memrealtime();
        }
    }
    __device__ ~Clocks()
    {
        if (slot) {
            slot[2] = __builtin_amdgcn_s_memtime();
            slot[3] = __builtin_amdgcn_s_memrealtime();
        }
    }
};

__global__ __launch_bounds__(256) void copy_kernel(const u32x4 *__restrict__ in, u32x4 *__restrict__ out, size_t n,
                                                   uint64_t *clk)
{
    Clocks c(clk);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) out[i] = in[i];
}

// ---- one vector instruction, 16 independent chains per wave ---------------------------------
template <int OP>
__global__ __launch_bounds__(1024) void vector_kernel(float *__restrict__ sink, int iters, uint64_t *clk)
{
    float x[16];
    uint32_t u[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        x[i] = -0.01f * (float)(threadIdx.x % 13) - 0.03f * (float)i;
        u[i] = 0x3f800000u + 977u * threadIdx.x + 131u * i;
    }
    const float ya = 0.999f - 1e-6f * (float)threadIdx.x, yb = -1e-3f;
    const uint32_t sel = 0x07020500u;
    const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
    {
        Clocks c(clk);
        for (int it = 0; it < iters; it += 8) {   // eight rounds per trip: the loop's own cost stays below 2 %
#pragma unroll
            for (int rep = 0; rep < 8; ++rep)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if constexpr (OP == E_EXP) x[i] = __builtin_amdgcn_exp2f(-__builtin_fabsf(x[i]));
                else if constexpr (OP == E_FMA) x[i] = __builtin_fmaf(x[i], ya, yb);
                else if constexpr (OP == E_CVT) u[i] = cvt_pk(__uint_as_float(u[i]), ya);
                else if constexpr (OP == E_MAX3) x[i] = __builtin_fmaxf(__builtin_fmaxf(x[i], x[(i + 5) & 15]), yb);
                else if constexpr (OP == E_PERM) u[i] = __builtin_amdgcn_perm(u[i], u[(i + 5) & 15], sel);
                else if constexpr (OP == E_DOT2)
                    x[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, u[i]), ones, x[i], false);
                else x[i] = x[i] + yb;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += x[i] + __uint_as_float(u[i]);
    if (s == 12345.678f) sink[0] = s;
}

template <int SHAPE>
struct Mfma;
template <>
struct Mfma<32> {
    typedef f32x16 Acc;
    static __device__ __forceinline__ Acc run(bf16x8 a, bf16x8 b, Acc c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static constexpr int kRegs = 16;
};
template <>
struct Mfma<16> {
    typedef f32x4 Acc;
    static __device__ __forceinline__ Acc run(bf16x8 a, bf16x8 b, Acc c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    static constexpr int kRegs = 4;
};

__device__ __forceinline__ void make_operands(bf16x8 &a, bf16x8 &b)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(0.01f * (float)((threadIdx.x + i) % 7));
        b[i] = (__bf16)(0.02f * (float)((threadIdx.x + 2 * i) % 5));
    }
}

// ---- matrix instructions alone (K = 0), or each followed by K vector instructions of the same wave ----
// VOP: E_EXP or E_FMA.  SHAPE 0: no matrix instruction, one v_exp_f32 followed by K v_fma_f32.
template <int SHAPE, int VOP, int K>
__global__ __launch_bounds__(1024) void same_wave_kernel(float *__restrict__ sink, int iters, uint64_t *clk)
{
    constexpr int S = SHAPE == 0 ? 16 : SHAPE;
    typedef typename Mfma<S>::Acc Acc;
    bf16x8 a, b;
    make_operands(a, b);
    Acc c[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < Mfma<S>::kRegs; ++i) c[j][i] = 0.f;
    float x[16], e[4];
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = -0.01f * (float)(threadIdx.x % 13) - 0.03f * (float)i;
#pragma unroll
    for (int i = 0; i < 4; ++i) e[i] = -0.5f * (float)i;
    const float ya = 0.999f - 1e-6f * (float)threadIdx.x, yb = -1e-3f;
    {
        Clocks cl(clk);
        for (int it = 0; it < iters; it += 4) {   // four rounds per trip
#pragma unroll
            for (int rep = 0; rep < 4; ++rep)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (SHAPE != 0) c[j] = Mfma<S>::run(a, b, c[j]);
                else e[j] = __builtin_amdgcn_exp2f(-__builtin_fabsf(e[j]));
#pragma unroll
                for (int i = 0; i < K; ++i) {
                    const int r = (j * K + i) & 15;
                    if constexpr (VOP == E_EXP && SHAPE != 0) x[r] = __builtin_amdgcn_exp2f(-__builtin_fabsf(x[r]));
                    else x[r] = __builtin_fmaf(x[r], ya, yb);
                }
                if constexpr (SHAPE != 0) GROUP_MFMA(1);
                else GROUP_TRANS(1);
                if constexpr (K > 0) {
                    if constexpr (VOP == E_EXP && SHAPE != 0) GROUP_TRANS(K);
                    else GROUP_VALU(K);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < Mfma<S>::kRegs; ++i) s += c[j][i];
#pragma unroll
    for (int i = 0; i < 16; ++i) s += x[i];
#pragma unroll
    for (int i = 0; i < 4; ++i) s += e[i];
    if (s == 12345.678f) sink[0] = s;
}

// ---- one matrix wave per SIMD beside vector waves ---------------------------------------------
// Waves 0-3 of the workgroup (one per SIMD) loop over four independent matrix instructions, na times;
// the other waves loop over 16 exponentials and 8 packs, nb times.
template <int SHAPE>
__global__ __launch_bounds__(1024) void other_wave_kernel(float *__restrict__ sink, int na, int nb, uint64_t *clk)
{
    typedef typename Mfma<SHAPE>::Acc Acc;
    const int wave = threadIdx.x >> 6;
    float s = 0.f;
    Clocks cl(clk);
    if (wave < 4) {
        bf16x8 a, b;
        make_operands(a, b);
        Acc c[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < Mfma<SHAPE>::kRegs; ++i) c[j][i] = 0.f;
        for (int it = 0; it < na; ++it) {
#pragma unroll
            for (int j = 0; j < 4; ++j) c[j] = Mfma<SHAPE>::run(a, b, c[j]);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < Mfma<SHAPE>::kRegs; ++i) s += c[j][i];
    } else {
        float x[16];
        uint32_t pk[8];
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = -0.01f * (float)(threadIdx.x % 13) - 0.03f * (float)i;
#pragma unroll
        for (int i = 0; i < 8; ++i) pk[i] = 0u;
        for (int it = 0; it < nb; ++it) {
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = __builtin_amdgcn_exp2f(-__builtin_fabsf(x[i]));
#pragma unroll
            for (int i = 0; i < 8; ++i) pk[i] ^= cvt_pk(x[2 * i], x[2 * i + 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) s += x[i];
#pragma unroll
        for (int i = 0; i < 8; ++i) s += (float)pk[i];
    }
    if (s == 12345.678f) sink[0] = s;
}

// ---- the dependent chain of one softmax tile, without memory ------------------------------------
// Per tile: NS score products into a fresh accumulator (for the NEXT tile, issued first), 16
// exponentials and 8 packs of the current tile's scores, two value products into the running sum.
template <int NS>
__global__ __launch_bounds__(1024) void tile_kernel(float *__restrict__ sink, int iters, uint64_t *clk)
{
    bf16x8 a, b;
    make_operands(a, b);
    f32x16 cur, nxt, o;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        cur[i] = -0.01f * (float)i;
        o[i] = 0.f;
    }
    // one tile: scores of the next tile into `to`, softmax work on `from`, value products into o
    auto tile = [&](f32x16 &from, f32x16 &to) {
#pragma unroll
        for (int i = 0; i < 16; ++i) to[i] = -1.f;
        asm volatile("" : "+v"(a), "+v"(b));   // the operands change from tile to tile as far as the compiler knows
#pragma unroll
        for (int j = 0; j < NS; ++j)
            to = __builtin_amdgcn_mfma_f32_32x32x16_bf16(j & 1 ? b : a, j & 1 ? a : b, to, 0, 0, 0);
        u32x4 w0, w1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            w0[i] = cvt_pk(__builtin_amdgcn_exp2f(from[2 * i]), __builtin_amdgcn_exp2f(from[2 * i + 1]));
            w1[i] = cvt_pk(__builtin_amdgcn_exp2f(from[8 + 2 * i]), __builtin_amdgcn_exp2f(from[8 + 2 * i + 1]));
        }
        o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, w0), o, 0, 0, 0);
        o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, w1), o, 0, 0, 0);
        GROUP_MFMA(NS);
        GROUP_TRANS(8);
        GROUP_VALU(4);
        GROUP_MFMA(1);
        GROUP_TRANS(8);
        GROUP_VALU(4);
        GROUP_MFMA(1);
        __builtin_amdgcn_sched_barrier(0);
    };
    {
        Clocks cl(clk);
        for (int it = 0; it < iters; it += 2) {
            tile(cur, nxt);
            tile(nxt, cur);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += o[i] + cur[i];
    if (s == 12345.678f) sink[0] = s;
}

// ---- fp64: NCH independent chains per wave of one instruction kind (NCH = 1: its dependent latency) ----
template <int OP, int NCH>
__global__ __launch_bounds__(1024) void f64_kernel(float *__restrict__ sink, int iters, uint64_t *clk)
{
    double x[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) x[i] = 1.0 + 1e-3 * (double)(threadIdx.x % 17) + 0.01 * (double)i;
    const double ya = 0.999 - 1e-6 * (double)threadIdx.x, yb = 1e-3;
    {
        Clocks c(clk);
        for (int it = 0; it < iters; it += 8) {
#pragma unroll
            for (int rep = 0; rep < 8; ++rep)
#pragma unroll
                for (int i = 0; i < NCH; ++i) {
                    if constexpr (OP == 0) x[i] = __builtin_fma(x[i], ya, yb);
                    else if constexpr (OP == 1) x[i] = x[i] * ya;
                    else if constexpr (OP == 2) x[i] = x[i] + yb;
                    else if constexpr (OP == 3) x[i] = __builtin_amdgcn_rsq(x[i]);
                    else x[i] = __builtin_amdgcn_rcp(x[i]);
                }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < NCH; ++i) s += x[i];
    if (s == 12345.678) sink[0] = (float)s;
}

int launch(int threads, int ex, int k, int iters, int cus, float *sink, uint64_t *clk, hipStream_t st, double *vec, double *mat)
{
    const double w = threads / 256;   // waves per SIMD
    *vec = 0.0;
    *mat = 0.0;
#define VEC(OP)                                                         \
    vector_kernel<OP><<<cus, threads, 0, st>>>(sink, iters, clk); \
    *vec = 16.0 * ((iters + 7) / 8 * 8) * w;                            \
    return 0
#define SAME(SHAPE, VOP)                                                                          \
    switch (k) {                                                                                  \
        case 0: same_wave_kernel<SHAPE, VOP, 0><<<cus, threads, 0, st>>>(sink, iters, clk); break;   \
        case 1: same_wave_kernel<SHAPE, VOP, 1><<<cus, threads, 0, st>>>(sink, iters, clk); break;   \
        case 2: same_wave_kernel<SHAPE, VOP, 2><<<cus, threads, 0, st>>>(sink, iters, clk); break;   \
        case 4: same_wave_kernel<SHAPE, VOP, 4><<<cus, threads, 0, st>>>(sink, iters, clk); break;   \
        case 8: same_wave_kernel<SHAPE, VOP, 8><<<cus, threads, 0, st>>>(sink, iters, clk); break;   \
        case 16: same_wave_kernel<SHAPE, VOP, 16><<<cus, threads, 0, st>>>(sink, iters, clk); break; \
        default: return -1;                                                                       \
    }                                                                                             \
    *vec = (4.0 * k + (SHAPE == 0 ? 4.0 : 0.0)) * ((iters + 3) / 4 * 4) * w;                      \
    *mat = SHAPE == 0 ? 0.0 : 4.0 * ((iters + 3) / 4 * 4) * w;                                    \
    return 0
    switch (ex) {
        case E_EXP: VEC(E_EXP);
        case E_FMA: VEC(E_FMA);
        case E_CVT: VEC(E_CVT);
        case E_MAX3: VEC(E_MAX3);
        case E_PERM: VEC(E_PERM);
        case E_DOT2: VEC(E_DOT2);
        case E_ADD: VEC(E_ADD);
        case E_MFMA32: k = 0; SAME(32, E_EXP);
        case E_MFMA16: k = 0; SAME(16, E_EXP);
        case E_SAME32_EXP: SAME(32, E_EXP);
        case E_SAME32_FMA: SAME(32, E_FMA);
        case E_SAME16_EXP: SAME(16, E_EXP);
        case E_EXP_FMA: SAME(0, E_FMA);
        case E_OTHER32:
        case E_OTHER16: {
            if (threads < 512 || k < 0 || k > 2) return -1;
            const int vw = threads / 256 - 1;                 // vector waves per SIMD
            const int na = (k == 2) ? 0 : iters * vw, nb = (k == 1) ? 0 : iters;
            if (ex == E_OTHER32) other_wave_kernel<32><<<cus, threads, 0, st>>>(sink, na, nb, clk);
            else other_wave_kernel<16><<<cus, threads, 0, st>>>(sink, na, nb, clk);
            *vec = 24.0 * nb * vw;
            *mat = 4.0 * na;
            return 0;
        }
        case E_TILE:
            switch (k) {
                case 1: tile_kernel<1><<<cus, threads, 0, st>>>(sink, iters, clk); break;
                case 2: tile_kernel<2><<<cus, threads, 0, st>>>(sink, iters, clk); break;
                case 3: tile_kernel<3><<<cus, threads, 0, st>>>(sink, iters, clk); break;
                default: return -1;
            }
            *vec = 24.0 * iters * w;
            *mat = (2.0 + k) * iters * w;
            return 0;
        case E_F64: {
            const int wgs = k >= 16 ? 8 : cus;     // param >= 16: eight workgroups only (a nearly idle chip)
            k %= 16;
#define F64(OP)                                                                              \
    if (k >= 8) f64_kernel<OP, 8><<<wgs, threads, 0, st>>>(sink, iters, clk);              \
    else f64_kernel<OP, 1><<<wgs, threads, 0, st>>>(sink, iters, clk);                     \
    break
            switch (k % 8) {
                case 0: F64(0);
                case 1: F64(1);
                case 2: F64(2);
                case 3: F64(3);
                case 4: F64(4);
                default: return -1;
            }
#undef F64
            *vec = (k >= 8 ? 8.0 : 1.0) * ((iters + 7) / 8 * 8) * w;
            return 0;
        }
        default: return -1;
    }
#undef VEC
#undef SAME
}

}  // namespace

extern "C" {

int flare_rates_count(void) { return E_COUNT; }
const char *flare_rates_name(int e) { return (e >= 0 && e < E_COUNT) ? kNames[e] : ""; }
size_t flare_rates_scratch_bytes(void) { return kScratch + 256; }

int flare_rates_run(int experiment, int waves_per_simd, int param, int iters, void *scratch, size_t scratch_bytes,
                    void *stream, flare_rates_result *out)
{
    if (!scratch || !out || scratch_bytes < kScratch + 256 || (reinterpret_cast<uintptr_t>(scratch) & 255u) != 0)
        return -1;
    if (experiment < 0 || experiment >= E_COUNT || waves_per_simd < 1 || waves_per_simd > 4 || iters < 1) return -1;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -5;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return -5;
    uint64_t *clk = reinterpret_cast<uint64_t *>(static_cast<char *>(scratch) + kScratch);
    float *sink = reinterpret_cast<float *>(clk + kClockSlots);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return -5;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return -5; }
    double vec = 0.0, mat = 0.0, bytes = 0.0;
    int rc = 0;
    for (int rep = 0; rep < 2 && rc == 0; ++rep) {   // the first launch warms up, the second is timed
        if (rep == 1 && hipEventRecord(e0, st) != hipSuccess) rc = -5;
        if (experiment == E_COPY) {
            const size_t n = kScratch / 2 / sizeof(u32x4);
            copy_kernel<<<cus * 8, 256, 0, st>>>(static_cast<const u32x4 *>(scratch),
                                                 static_cast<u32x4 *>(scratch) + n, n, clk);
            bytes = (double)kScratch;
        } else {
            rc = launch(256 * waves_per_simd, experiment, param, iters, cus, sink, clk, st, &vec, &mat);
        }
        if (rc == 0 && hipGetLastError() != hipSuccess) rc = -5;
    }
    if (rc == 0 && (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess)) rc = -5;
    float ms = 0.f;
    if (rc == 0 && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = -5;
    uint64_t t[kClockSlots] = {0, 0, 0, 0};
    if (rc == 0 && hipMemcpy(t, clk, sizeof(t), hipMemcpyDeviceToHost) != hipSuccess) rc = -5;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != 0) return rc;
    out->ms = ms;
    out->vector_ops = vec;
    out->matrix_ops = mat;
    out->bytes = bytes;
    out->shader_mhz = (t[3] > t[1]) ? 100.0 * (double)(t[2] - t[0]) / (double)(t[3] - t[1]) : 0.0;
    return 0;
}

}  // extern "C"
