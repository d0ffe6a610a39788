/*
 * flare_rates.h -- C ABI of libflare_rates.so: micro-benchmarks of the machine rates that the
 * roofline figures of the FLARE kernels are priced against (not part of the operator; the
 * operator's library does not link it).  Every experiment is one kernel, launched with one
 * workgroup per compute unit, timed with a pair of HIP events on the given stream.
 *
 * Experiments (flare_rates_count() of them, flare_rates_name(i) names one):
 *   - "copy": a plain device copy of `bytes`/2 bytes from the first to the second half of the
 *     scratch buffer (read + write bytes are reported);
 *   - one per vector instruction (v_exp_f32, v_fma_f32, v_cvt_pk_bf16_f32, v_max3_f32,
 *     v_perm_b32, v_dot2c_f32_bf16, v_add_f32): 16 independent chains per wave;
 *   - one per matrix instruction (32x32x16 and 16x16x32, bf16): four independent accumulators;
 *   - "same wave" mixes: every wave issues one matrix instruction followed by k vector
 *     instructions (k = param), all independent, pinned in that order;
 *   - "other wave" mixes: per SIMD one wave issues only matrix instructions and the other
 *     waves only vector instructions (16 exponentials + 8 packs per round).
 *
 * Conventions: `scratch` is a DEVICE pointer owned by the caller, 256-byte aligned, of at
 * least flare_rates_scratch_bytes() bytes; the call enqueues on `stream` (a hipStream_t passed
 * as void*), waits for its own stop event (it is a measurement) and allocates nothing but the
 * two events it destroys again.  Returns 0, or -1 for a bad argument, -5 for a HIP error.
 */
#ifndef FLARE_RATES_H
#define FLARE_RATES_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    double ms;            /* duration of the timed launch */
    double vector_ops;    /* vector instructions (wave64) issued per SIMD during the launch */
    double matrix_ops;    /* matrix instructions issued per SIMD during the launch */
    double bytes;         /* bytes moved (copy experiment), else 0 */
    double shader_mhz;    /* shader clock during the launch: shader-clock ticks per 100 MHz tick, times 100 */
} flare_rates_result;

int flare_rates_count(void);
const char *flare_rates_name(int experiment);
size_t flare_rates_scratch_bytes(void);

/*
 * Runs one experiment.  waves_per_simd in 1..4 (workgroups of 256 * waves_per_simd threads, one per
 * compute unit); param: the k of a "same wave" mix, else ignored; iters: loop trips per wave.
 */
int flare_rates_run(int experiment, int waves_per_simd, int param, int iters, void *scratch, size_t scratch_bytes,
                    void *stream, flare_rates_result *out);

#ifdef __cplusplus
}
#endif
#endif /* FLARE_RATES_H */
