"""Trial runs for the instance exploration (Algorithm 2 of the paper, Section 5.3): profile() of one
(instances per GPU, environments per instance) point on CU-masked instances of one GPU.

Each instance is a holistic one (simulator + agent + trainer on its own stream, the synchronized-training
template of Section 5.1) with an even share of the compute units; all instances of a point run their
iterations concurrently.  Throughput is per instance (samples/s), memory is the device memory one instance
adds.  No arithmetic of the method happens here; the search itself is `gmi_explore` in the library."""
from __future__ import annotations

import time
from typing import Callable, List, Sequence, Tuple

import torch

from . import GmiError, gmi_cu_count, gmi_create, gmi_destroy
from .instances import XCDS, cu_masks


def cus_per_instance(device_cus: int, gmi_per_gpu: int) -> int:
    """Even split of the device, rounded down to whole rows of one CU per die (masks must keep a CU on
    every die)."""
    return (device_cus // gmi_per_gpu) // XCDS * XCDS


class InstanceProfiler:
    """profile(gmi_per_gpu, num_env) -> (runnable, samples/s of one instance, bytes of one instance).

    build(num_env, cu_mask) returns a session object with rollout/gae/update-style stepping done by
    step(session, iteration) (asynchronous on the session's stream), .sync() and .close();
    samples(num_env) is the number of samples one iteration of one instance processes."""

    def __init__(self, build: Callable, step: Callable, samples: Callable[[int], int], iterations: int = 3,
                 warmup: int = 1, progress=None):
        self.build, self.step, self.samples = build, step, samples
        self.iterations, self.warmup = iterations, warmup
        self.progress = progress                     # optional callable(row dict) after every point
        probe = gmi_create()
        self.device_cus = gmi_cu_count(probe)
        gmi_destroy(probe)
        self.log: List[dict] = []

    def __call__(self, gmi_per_gpu: int, num_env: int) -> Tuple[bool, float, float]:
        cus = cus_per_instance(self.device_cus, gmi_per_gpu)
        row = {"gmi_per_gpu": gmi_per_gpu, "num_env": num_env, "cus_per_instance": cus}
        sessions = []
        try:
            if cus < XCDS:
                raise ValueError("fewer than one compute unit per die")
            masks = [None] if gmi_per_gpu == 1 and cus == self.device_cus else \
                cu_masks(self.device_cus, [cus] * gmi_per_gpu, "contiguous")
            torch.cuda.synchronize()
            torch.cuda.empty_cache()
            free0, _ = torch.cuda.mem_get_info()
            for m in masks:
                sessions.append(self.build(num_env, m))
            torch.cuda.synchronize()
            free1, _ = torch.cuda.mem_get_info()
            it = 0
            for _ in range(self.warmup):
                for s in sessions:
                    self.step(s, it)
                it += 1
            for s in sessions:
                s.sync()
            t0 = time.perf_counter()
            for _ in range(self.iterations):
                for s in sessions:
                    self.step(s, it)
                it += 1
            for s in sessions:
                s.sync()
            el = time.perf_counter() - t0
            top = self.iterations * self.samples(num_env) / el
            mem = (free0 - free1) / len(sessions)
            row.update(runnable=True, samples_per_s=top, bytes=mem, ms_per_iteration=el * 1e3 / self.iterations)
            return True, top, float(mem)
        except (GmiError, ValueError, AssertionError, torch.cuda.OutOfMemoryError) as e:
            row.update(runnable=False, reason=str(e)[:200])
            return False, 0.0, 0.0
        finally:
            for s in sessions:
                try:
                    s.close()
                except GmiError:
                    pass
            sessions.clear()
            self.log.append(row)
            if self.progress is not None:
                self.progress(row)
