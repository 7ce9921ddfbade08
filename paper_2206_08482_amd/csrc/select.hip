// Profiling-based instance exploration (Algorithm 2 of the paper, "Workload-aware GMI Selection"): the
// search over (instances per GPU, environments per instance) with the saturation early stop.  Host code
// only; what a point costs is measured by the caller's profile() callback (a trial run of the hot path on
// CU-masked instances), exactly as the paper's profile() launches a trial run per point.
#include <math.h>

#include "internal.h"

namespace {

// Relative change and Sat are IEEE divisions: x/0 = +-inf, 0/0 = NaN; NaN never compares below alpha.
double ratio(double num, double den) { return num / den; }

double default_estimate(int gmi_per_gpu, int num_gpu, double top, void*) {
  // every instance of every GPU contributes its measured throughput
  return top * (double)gmi_per_gpu * (double)num_gpu;
}

}  // namespace

extern "C" int gmi_explore(gmi_profile_fn profile, void* profile_user, gmi_estimate_fn estimate, void* estimate_user,
                           int num_gpu, double alpha, const int32_t* gmi_per_gpu_values, int32_t n_gmi,
                           const int32_t* num_env_values, int32_t n_env, int32_t* num_env_out,
                           int32_t* gmi_per_gpu_out, double* projected_out) {
  if (!profile) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_explore: profile callback is NULL");
  if (!num_env_out || !gmi_per_gpu_out) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_explore: NULL output");
  if (num_gpu < 1) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_explore: num_gpu must be >= 1");
  if (n_gmi < 0 || n_env < 0 || (n_gmi > 0 && !gmi_per_gpu_values) || (n_env > 0 && !num_env_values))
    GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_explore: bad value lists");
  if (!estimate) estimate = default_estimate;
  bool have_best = false;
  int best_env = 0, best_gmi = 0;
  double max_top = -INFINITY;
  for (int a = 0; a < n_gmi; ++a) {
    const int gmi_per_gpu = gmi_per_gpu_values[a];
    double pre_top = 0.0, pre_mem = 0.0;
    for (int b = 0; b < n_env; ++b) {
      const int num_env = num_env_values[b];
      int runnable = 0;
      double top = 0.0, mem = 0.0;
      const int rc = profile(gmi_per_gpu, num_env, &runnable, &top, &mem, profile_user);
      if (rc != 0) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_explore: profile callback failed (%d) at GMIperGPU %d, num_env %d",
                            rc, gmi_per_gpu, num_env);
      if (!runnable) continue;
      if (pre_top == 0.0 && pre_mem == 0.0) {
        pre_top = top;
        pre_mem = mem;
        continue;
      }
      const double r_top = ratio(top - pre_top, pre_top);
      const double r_mem = ratio(mem - pre_mem, pre_mem);
      const double sat = ratio(r_top, r_mem);
      pre_top = top;
      pre_mem = mem;
      if (sat < alpha) break;
      const double acc_top = estimate(gmi_per_gpu, num_gpu, top, estimate_user);
      if (acc_top > max_top) {
        max_top = acc_top;
        best_env = num_env;
        best_gmi = gmi_per_gpu;
        have_best = true;
      }
    }
  }
  *num_env_out = have_best ? best_env : 0;
  *gmi_per_gpu_out = have_best ? best_gmi : 0;
  if (projected_out) *projected_out = have_best ? max_top : 0.0;
  return GMI_OK;
}

// ---------------------------------------------------------------------------------------------------------
// Layout-aware gradient reduction, host logic (Section 4.1 of the paper): which of the three strategies a
// layout of trainer instances calls for (Algorithm 1), which instance leads its GPU in the cross-GPU step of
// the hierarchical form, and the time models of Table 2.  On one GPU only the first answer ever occurs and
// this build performs that reduction in memory (ppo_update_group); the functions describe layouts this build
// does not run.
extern "C" int gmi_select_reduction(const int32_t* gmis_per_gpu, int32_t n_gpus, int32_t* strategy_out) {
  if (!strategy_out) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_select_reduction: NULL output");
  if (n_gpus < 0 || (n_gpus > 0 && !gmis_per_gpu)) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_select_reduction: bad layout");
  for (int p = 0; p < n_gpus; ++p)
    if (gmis_per_gpu[p] < 0) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_select_reduction: negative count for GPU %d", p);
  if (n_gpus <= 1) {                               // all instances on the same GPU
    *strategy_out = GMI_REDUCE_MULTI_PROCESS;
    return GMI_OK;
  }
  bool equal = true;                               // do all GPUs host the same number of instances?
  for (int p = 1; p < n_gpus; ++p) equal = equal && gmis_per_gpu[p] == gmis_per_gpu[0];
  if (!equal || gmis_per_gpu[0] > n_gpus) *strategy_out = GMI_REDUCE_HIERARCHICAL;
  else *strategy_out = GMI_REDUCE_MULTI_RING;
  return GMI_OK;
}

extern "C" int gmi_har_leaders(const int32_t* gmi_ids, const int32_t* gpu_start, int32_t n_gpus, int32_t t,
                               int32_t* leaders_out) {
  if (n_gpus < 0 || (n_gpus > 0 && (!gpu_start || !leaders_out)))
    GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_har_leaders: bad arguments");
  for (int p = 0; p < n_gpus; ++p) {
    const int b = gpu_start[p], e = gpu_start[p + 1];
    if (e < b || (e > b && !gmi_ids)) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_har_leaders: bad range for GPU %d", p);
    const int m = e - b;
    leaders_out[p] = -1;
    for (int i = b; i < e; ++i)
      if (gmi_ids[i] >= 0 && gmi_ids[i] % m == t) { leaders_out[p] = gmi_ids[i]; break; }
  }
  return GMI_OK;
}

extern "C" int gmi_reduction_time(int32_t strategy, int32_t g, int32_t t, double m_p, double b1, double b2,
                                  double* seconds_out) {
  if (!seconds_out) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_reduction_time: NULL output");
  if (g < 1 || t < 1) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_reduction_time: need g >= 1 GPUs and t >= 1 instances per GPU");
  const double gd = g, td = t;
  switch (strategy) {
    case GMI_REDUCE_MULTI_PROCESS: *seconds_out = 2.0 * (gd * td - 1.0) * m_p / (gd * td * b1); break;
    case GMI_REDUCE_MULTI_RING: *seconds_out = 2.0 * (gd - 1.0) * (td + 1.0) * m_p / (gd * b2); break;
    case GMI_REDUCE_HIERARCHICAL:
      *seconds_out = 2.0 * (gd - 1.0) * m_p / (gd * b2) + 2.0 * (td - 1.0) * m_p / (td * b1);
      break;
    default: GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_reduction_time: unknown strategy %d", strategy);
  }
  return GMI_OK;
}
