/*
 * vla_bench.h — measurement support of the VLA policy library (include/vla.h): the practical ceilings of the
 * device and per-kernel-family timing.  Not part of the policy path; used by bench.py only.
 */
#ifndef VLA_BENCH_H
#define VLA_BENCH_H

#include "vla.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Practical ceilings of the device the context runs on, for reporting next to the vendor peaks (benchmark
 * support, not part of the policy path; unlike every other call it waits for its own kernels).  Needs loaded
 * weights on the 16-bit path.
 *   kind 0: an MFMA-only loop (8 independent 32x32x16 half-precision MFMAs per iteration and wave, two waves
 *           per SIMD, operands = real weight fragments held in registers) -> *value_out in TFLOP/s
 *   kind 1: a plain 16-byte-per-lane streaming read of all layer weights                -> *value_out in GB/s
 * Best of three timed runs after a warm-up. */
int vla_probe(vla_ctx* ctx, int32_t kind, double* value_out, void* hip_stream);

/* Timing hooks for the benchmark: duration of the launches of one kernel family, measured with
 * HIP events recorded on the launch stream around each launch.  vla_prof_enable(ctx, mask) clears
 * what was collected and then times the families whose bit (1 << index) is set in mask (0 = off).
 * vla_prof_read synchronises the recorded events (host-blocking) and reports, for family index i
 * (0 <= i < vla_prof_count()), its name, number of launches and total milliseconds.  Families are
 * named by the read-out itself: the four GEMMs (qkv, o, gate-up, down) and the attention of prefill
 * and of decode, rmsnorm, head_select, misc. */
int vla_prof_enable(vla_ctx* ctx, int32_t mask);
int vla_prof_count(void);
int vla_prof_read(vla_ctx* ctx, int32_t i, const char** name, int64_t* launches, double* total_ms);

#ifdef __cplusplus
}
#endif
#endif /* VLA_BENCH_H */
