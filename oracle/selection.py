"""Oracle for the profiling-based instance exploration (Algorithm 2, "Workload-aware GMI Selection").

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing in the product).  Plain Python, the algorithm's
steps in the paper's order and notation; `profile` and `estimate` are passed in, so the search itself is
a pure function of what they return.

Readings where the paper is silent:
  * Sat = R_top / R_mem is an IEEE division: x/0 = +-inf, 0/0 = NaN, and a NaN never satisfies "Sat < alpha"
    (so an unchanged memory footprint is never read as saturation by itself);
  * the tracking variables count as uninitialised exactly while both are 0 (the listing's test);
  * if no point is ever recorded the result is None.
"""
from __future__ import annotations

import math
from typing import Callable, Iterable, Optional, Sequence, Tuple

NUM_ENV_GRID = [128, 256, 512, 1024, 2048, 4096, 8192, 16384]      # "128, 256, 512, ..., 16384"
GMI_PER_GPU_RANGE = list(range(10, 0, -1))                         # "10 ... 1"


def _ratio(num: float, den: float) -> float:
    if den == 0.0:
        if num == 0.0 or math.isnan(num):
            return math.nan
        return math.inf if num > 0 else -math.inf
    return num / den


def explore(profile: Callable[[int, int], Tuple[bool, float, float]],
            estimate: Callable[[int, int, float], float], num_gpu: int, alpha: float,
            gmi_per_gpu_values: Iterable[int] = tuple(GMI_PER_GPU_RANGE),
            num_env_values: Sequence[int] = tuple(NUM_ENV_GRID)) -> Optional[Tuple[int, int]]:
    """Returns (num_env, GMIperGPU) of the best projected system throughput, or None.

    profile(GMIperGPU, num_env) -> (runnable, throughput, memory) of ONE instance;
    estimate(GMIperGPU, num_GPU, throughput) -> projected throughput of the whole system."""
    best_config = None
    max_top = -math.inf
    for gmi_per_gpu in gmi_per_gpu_values:
        pre_top = 0.0
        pre_mem = 0.0
        for num_env in num_env_values:
            runnable, top, mem = profile(gmi_per_gpu, num_env)
            if not runnable:                          # filter out non-runnable instances
                continue
            if pre_top == 0.0 and pre_mem == 0.0:     # initialise the tracking variables
                pre_top, pre_mem = top, mem
                continue
            r_top = _ratio(top - pre_top, pre_top)    # relative throughput gain
            r_mem = _ratio(mem - pre_mem, pre_mem)    # relative memory penalty
            sat = _ratio(r_top, r_mem)
            pre_top, pre_mem = top, mem
            if sat < alpha:                           # saturated: stop growing num_env for this size
                break
            acc_top = estimate(gmi_per_gpu, num_gpu, top)
            if acc_top > max_top:
                max_top = acc_top
                best_config = (num_env, gmi_per_gpu)
    return best_config
