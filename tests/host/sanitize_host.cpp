// Host-only exercise of the library's host logic (instance search, reduction choice, leader rule, time models,
// least-loaded routing, error paths that return before any device call) for a build with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host side.  No GPU is touched.  Exit code 0 = all checks passed.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/gmidrl.h"

static int fails = 0;
#define CHECK(c) do { if (!(c)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #c); ++fails; } } while (0)

struct Table { int calls = 0; };
// throughput grows with the env count and saturates; memory grows linearly
static int profile(int32_t k, int32_t n, int32_t* runnable, double* top, double* mem, void* user) {
  static_cast<Table*>(user)->calls++;
  *runnable = k <= 8;
  *top = 1000.0 * n / (n + 2048.0) / k;
  *mem = 1e6 * n + 5e7;
  return 0;
}

int main() {
  {
    Table t;
    const int32_t ks[] = {8, 4, 2, 1, 16}, ns[] = {128, 512, 2048, 8192};
    int32_t n_out = -1, k_out = -1;
    double proj = -1.0;
    const int rc = gmi_explore(profile, &t, nullptr, nullptr, 1, 0.05, ks, 5, ns, 4, &n_out, &k_out, &proj);
    CHECK(rc == GMI_OK);
    CHECK(t.calls > 0 && t.calls <= 20);
    CHECK(n_out > 0 && k_out > 0 && proj > 0.0);
    CHECK(gmi_explore(nullptr, &t, nullptr, nullptr, 1, 0.05, ks, 5, ns, 4, &n_out, &k_out, &proj) != GMI_OK);
    CHECK(std::strlen(gmi_last_error()) > 0);
    // an empty grid records no point: the documented answer is the pair (0, 0)
    CHECK(gmi_explore(profile, &t, nullptr, nullptr, 1, 0.05, ks, 0, ns, 4, &n_out, &k_out, &proj) == GMI_OK && n_out == 0 && k_out == 0);
  }
  {
    const int64_t load[] = {50, 20, 20, 70};
    int32_t best = -1;
    CHECK(gmi_route_least_loaded(load, 4, &best) == GMI_OK && best == 1);
    CHECK(gmi_route_least_loaded(load, 0, &best) != GMI_OK);
    CHECK(gmi_route_least_loaded(nullptr, 4, &best) != GMI_OK);
  }
  {
    // Algorithm 1's three exits, the leader rule and the time models (Table 2)
    int32_t strat = -1;
    const int32_t one[] = {4}, even[] = {2, 2, 2, 2}, uneven[] = {2, 3}, many[] = {4, 4};
    CHECK(gmi_select_reduction(one, 1, &strat) == GMI_OK && strat == GMI_REDUCE_MULTI_PROCESS);
    CHECK(gmi_select_reduction(even, 4, &strat) == GMI_OK && strat == GMI_REDUCE_MULTI_RING);
    CHECK(gmi_select_reduction(uneven, 2, &strat) == GMI_OK && strat == GMI_REDUCE_HIERARCHICAL);
    CHECK(gmi_select_reduction(many, 2, &strat) == GMI_OK && strat == GMI_REDUCE_HIERARCHICAL);
    CHECK(gmi_select_reduction(nullptr, 2, &strat) != GMI_OK);
    const int32_t ids[] = {0, 1, 2, 3, 4, 5}, start[] = {0, 3, 6};
    int32_t leaders[2] = {-2, -2};
    CHECK(gmi_har_leaders(ids, start, 2, 1, leaders) == GMI_OK && leaders[0] == 1 && leaders[1] == 4);
    double sec[3] = {0, 0, 0};
    for (int st = 0; st < 3; ++st) CHECK(gmi_reduction_time(st, 4, 2, 1e6, 1e9, 1e10, &sec[st]) == GMI_OK && sec[st] > 0.0);
    CHECK(gmi_reduction_time(7, 4, 2, 1e6, 1e9, 1e10, &sec[0]) != GMI_OK);
  }
  {
    // bad handles are reported before anything touches a device
    CHECK(gmi_sync(nullptr) == GMI_ERR_BAD_HANDLE);
    CHECK(gmi_destroy(nullptr) == GMI_ERR_BAD_HANDLE);
    CHECK(gmi_channels_drop(nullptr, 1) == GMI_ERR_BAD_HANDLE);
    CHECK(gmi_stream(nullptr) == nullptr);
  }
  std::printf(fails ? "host checks: %d failed\n" : "host checks passed\n", fails);
  return fails ? 1 : 0;
}
