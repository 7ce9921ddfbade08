// Profiling-based instance exploration (Algorithm 2 of the paper, "Workload-aware GMI Selection"): the
// search over (instances per GPU, environments per instance) with the saturation early stop.  Host code
// only; what a point costs is measured by the caller's profile() callback (a trial run of the hot path on
// CU-masked instances), exactly as the paper's profile() launches a trial run per point.
#include <math.h>

#include "internal.h"

namespace {

// One measured operating point of an instance size.
struct Point {
  int envs;
  double rate, bytes;      // throughput and memory of ONE instance
  // a point with neither throughput nor memory cannot anchor a comparison (the listing's "trackers still 0")
  bool anchors() const { return rate != 0.0 || bytes != 0.0; }
};

// Throughput gained per memory spent when an instance grows from `from` to `to`, both as relative changes.
// IEEE divisions on purpose: x/0 = +-inf, 0/0 = NaN, and a NaN is never "below alpha".
double gain_per_memory(const Point& from, const Point& to) {
  const double gain = (to.rate - from.rate) / from.rate;
  const double cost = (to.bytes - from.bytes) / from.bytes;
  return gain / cost;
}

struct Candidate {
  int instances, envs;
  double system_rate;
};

double whole_system(int instances, int gpus, double rate, void*) {
  // every instance of every GPU contributes its measured throughput
  return rate * (double)instances * (double)gpus;
}

// Grows the environments of one instance size through env_grid until growth stops paying (gain per memory below
// alpha), measuring each size with the caller's trial run; every point that still paid becomes a candidate with
// its projected whole-system throughput.  The first measurable point only anchors the comparison.
int scan_instance_size(int instances, const int32_t* env_grid, int n_env, gmi_profile_fn trial, void* trial_user,
                       gmi_estimate_fn project, void* project_user, int gpus, double alpha,
                       std::vector<Candidate>* out) {
  Point last = {0, 0.0, 0.0};
  for (int i = 0; i < n_env; ++i) {
    Point now = {env_grid[i], 0.0, 0.0};
    int ran = 0;
    const int rc = trial(instances, now.envs, &ran, &now.rate, &now.bytes, trial_user);
    if (rc != 0) GMI_FAIL(GMI_ERR_INVALID_ARG, "gmi_explore: profile callback failed (%d) at GMIperGPU %d, num_env %d",
                          rc, instances, now.envs);
    if (!ran) continue;                                  // this size does not run at all (memory, hang): skip it
    const bool comparable = last.anchors();
    const double paid = comparable ? gain_per_memory(last, now) : 0.0;
    last = now;
    if (!comparable) continue;
    if (paid < alpha) break;                             // saturated
    out->push_back({instances, now.envs, project(instances, gpus, now.rate, project_user)});
  }
  return GMI_OK;
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
  std::vector<Candidate> candidates;
  for (int a = 0; a < n_gmi; ++a) {
    const int rc = scan_instance_size(gmi_per_gpu_values[a], num_env_values, n_env, profile, profile_user,
                                      estimate ? estimate : whole_system, estimate_user, num_gpu, alpha, &candidates);
    if (rc != GMI_OK) return rc;
  }
  // the candidate with the highest projected throughput; of equals the one measured first; a NaN never wins
  const Candidate* best = nullptr;
  for (const Candidate& c : candidates)
    if (best ? c.system_rate > best->system_rate : c.system_rate > -INFINITY) best = &c;
  *num_env_out = best ? best->envs : 0;
  *gmi_per_gpu_out = best ? best->instances : 0;
  if (projected_out) *projected_out = best ? best->system_rate : 0.0;
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
