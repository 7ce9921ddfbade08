/*
 * gmidrl_bench.h -- measurement interface of libgmidrl: the per-kernel launch timer and two probes that
 * bench.py and the scripts under benchmarks/ use.  NOT part of the hot path's boundary (gmidrl.h): nothing here
 * computes any step of the method.
 */
#ifndef GMIDRL_BENCH_H
#define GMIDRL_BENCH_H

#include "gmidrl.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Built-in timer for measurement runs (the paper's profile() step of Algorithm 2 measures a trial
 * run; here the unit is one kernel class = one kernel symbol).  class_mask bit c = 1: every launch of
 * kernel class c on this instance carries a pair of HIP events on the instance's stream that receive the
 * kernel's own begin and end timestamps, so a class total is execution time without launch gaps.
 * Enabling (or passing 0 to disable) synchronises the stream and clears earlier measurements.  Event
 * pairs are created on demand, so a profiled call may allocate host-side event objects. */
int gmi_profile_enable(gmi_t gmi, uint32_t class_mask);
/* Number of kernel classes, and the name of class cls (NULL if out of range). */
int gmi_profile_classes(void);
const char* gmi_profile_class_name(int cls);
/* Synchronises the stream and returns the summed duration (ms) and the number of bracketed
 * launches of class cls since profiling was enabled.  host: total_ms, launches. */
int gmi_profile_read(gmi_t gmi, int cls, double* total_ms, int64_t* launches);
/* Algorithmic work (flops; bytes of operands read and results written once) that the launchers stated
 * for the timed launches of class cls since gmi_profile_enable; 0 for classes whose launcher states
 * none (the linear-layer and weight-gradient classes state theirs).  host: flops, bytes. */
int gmi_profile_work(gmi_t gmi, int cls, double* flops, double* bytes);

/* Achievable-peak probes for measurement reports: what = 0 runs a pure bf16 matrix-core loop and
 * returns TFLOP/s, what = 1 runs a streaming copy over the two halves of `scratch` and returns GB/s
 * (bytes read + written).  Blocks until done.  scratch: dev, scratch_bytes long; result: host. */
int gmi_measure_peak(gmi_t gmi, int what, void* scratch, size_t scratch_bytes, double* result);

/* Micro-benchmark of one bf16 linear-layer product of the MLPs (Table 6 shapes) on synthetic operands
 * carved out of `scratch` (dev; zero or arbitrary finite contents): kind 0 = forward with bias + ELU,
 * 2 = input gradient, 3 = weight gradient.  rows x K -> F, K and F multiples of 32, n_nets (1 or 2)
 * problems per launch as in the real path.  us_per_launch (host) = average over reps launches. Blocks. */
int gmi_bench_linear(gmi_t gmi, int kind, int rows, int K, int F, int n_nets, int reps, void* scratch,
                     size_t scratch_bytes, double* us_per_launch);

/* gae_compute has two kernels for the recurrence over the horizon: the serial walk with one lane per env (0, the
 * default at every size) and a wavefront scan with lanes over time (1; horizons up to 64, else the serial walk
 * runs).  Forces one of them for every later call of the process; results agree within fp32 rounding. */
int gmi_bench_gae_variant(int variant);

#ifdef __cplusplus
}
#endif
#endif /* GMIDRL_BENCH_H */
