#!/usr/bin/env python3
"""Bandwidth-bound kernels of the hot path on inputs scaled up until HBM, not launch latency, bounds them.

At the benchmark configurations GAE, Adam, the env step and the experience store move 1-30 MB per call,
which is below launch latency and inside the caches; this script runs the same kernels (through the same
C-ABI entry points) on inputs of ~0.5-2 GB and prints achieved GB/s against the 8 TB/s HBM peak and against
a plain copy kernel on the same device.  One JSON object on stdout.

    python benchmarks/kernels.py [--large-only | --copy-only]

--large-only: only the inputs of 0.5 GB and more; --copy-only: only the copy kernel (the calibration run for the
hardware counters FETCH_SIZE and WRITE_SIZE).
"""
from __future__ import annotations

import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def measure(copy_only=False, large_only=False):
    """Returns the report as a dict.  large_only: only the inputs of 0.5 GB and more (the HBM-roofline evidence)."""
    import numpy as np
    import torch

    import paper_2206_08482_amd as g
    from paper_2206_08482_amd.runner import RolloutBuffers

    dev = torch.device("cuda:0")
    h = g.gmi_create()
    names = [g.gmi_profile_class_name(c) for c in range(g.gmi_profile_classes())]
    out = {"hbm_peak_GBs": 8000.0}
    scratch = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    out["copy_kernel_GBs"] = g.gmi_measure_peak(h, 1, scratch)
    if copy_only:
        # calibration run for hardware counters: the copy kernel reads and writes 2^29 bytes per launch
        g.gmi_destroy(h)
        return out
    out["mfma_loop_TFLOPs"] = g.gmi_measure_peak(h, 0, scratch)
    del scratch

    def timed(cls, fn, reps=10):
        fn()
        g.gmi_profile_enable(h, 1 << names.index(cls))
        for _ in range(reps):
            fn()
        ms, _ = g.gmi_profile_read(h, names.index(cls))   # summed kernel time; a call may launch several
        g.gmi_profile_enable(h, 0)
        return ms / reps

    rows = []
    # GAE: T x N rewards, values, dones -> advantages, returns (25 B per sample + 4 B per env)
    for T, N in ((64, 1 << 20),) if large_only else ((16, 4096), (32, 4096), (16, 16384), (32, 16384), (64, 1 << 20)):
        rb = RolloutBuffers(T, N, 1, 1, dev)
        rb.rew.normal_(); rb.val.normal_()
        lastv = torch.zeros(N, device=dev)
        torch.cuda.synchronize()
        hb = g.gmi_buffer_bind(h, rb.desc(0, N))
        for norm, nbytes in ((False, T * N * 17.0 + 4.0 * N), (True, T * N * 25.0 + 4.0 * N)):
            for variant, vname in ((0, ""), (1, " (wavefront scan)")):      # the default serial walk, then the scan
                g.gmi_bench_gae_variant(variant)
                ms = timed("gae", lambda: g.gae_compute(h, hb, lastv, 0.99, 0.95, norm))
                rows.append({"kernel": "gae" + ("+normalize" if norm else "") + vname, "size": f"T={T} N={N}",
                             "bytes": nbytes, "us": ms * 1e3, "GBs": nbytes / ms / 1e6})
            g.gmi_bench_gae_variant(0)
        g.gmi_buffer_destroy(hb)
        del rb
    # Adam on caller arrays: 16 B read + 12 B written per parameter
    for n in (1 << 26,) if large_only else (114129, 1 << 26):
        p, m, v, gr = (torch.zeros(n, device=dev) for _ in range(4))
        gr.normal_()
        torch.cuda.synchronize()
        hp = g.ppo_hparams()
        ms = timed("adam", lambda: g.adam_update(h, p, m, v, gr, n, hp, 1))
        rows.append({"kernel": "adam (plain arrays)", "size": f"P={n}", "bytes": 28.0 * n, "us": ms * 1e3,
                     "GBs": 28.0 * n / ms / 1e6})
        del p, m, v, gr
    # env step and experience store
    for N, O, A in ((1 << 20, 60, 8), (1 << 19, 108, 21), (1 << 18, 211, 20)) if large_only else (
            (4096, 60, 8), (1 << 20, 60, 8), (1 << 19, 108, 21), (1 << 18, 211, 20)):
        am = torch.eye(O, device=dev) * 0.95
        bm = torch.zeros(O, A, device=dev)
        ep = torch.zeros(N, dtype=torch.int32, device=dev)
        s = torch.randn(N, O, device=dev); a = torch.randn(N, A, device=dev)
        nxt = torch.zeros(N, O, device=dev); rew = torch.zeros(N, device=dev)
        done = torch.zeros(N, dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        he = g.gmi_env_bind(h, g.env_desc(N, O, A, 0.01, 1.0, 0, (1 << 32) // 1000, 0), am, bm, ep)
        nbytes = N * (4.0 * (2 * O + A) + 9)
        flops = N * (2.0 * O * (O + A) + 3 * O + 2 * A)
        ms = timed("env_step", lambda: g.env_step(h, he, s, a, 3, nxt, rew, done))
        rows.append({"kernel": "env_step", "size": f"N={N} O={O} A={A}", "bytes": nbytes, "us": ms * 1e3,
                     "GBs": nbytes / ms / 1e6, "fp32_TFLOPs": flops / ms / 1e9})
        g.gmi_env_destroy(he)
        T = 2
        rb = RolloutBuffers(T, N, O, A, dev)
        torch.cuda.synchronize()
        hb = g.gmi_buffer_bind(h, rb.desc(0, N))
        cb = N * 2 * (4.0 * (O + A + 3) + 1)
        ms = timed("collect", lambda: g.collect_experience(h, hb, 1, s, a, rew, rew, rew, done))
        rows.append({"kernel": "collect_experience", "size": f"N={N} O={O} A={A}", "bytes": cb, "us": ms * 1e3,
                     "GBs": cb / ms / 1e6})
        g.gmi_buffer_destroy(hb)
        del rb, s, a, nxt
    for r in rows:
        r["frac_of_hbm_peak"] = r["GBs"] / 8000.0
        r["frac_of_copy_kernel"] = r["GBs"] / out["copy_kernel_GBs"]
    out["rows"] = rows
    g.gmi_destroy(h)
    return out


def main() -> int:
    print(json.dumps(measure(copy_only="--copy-only" in sys.argv, large_only="--large-only" in sys.argv)))
    return 0


if __name__ == "__main__":
    sys.exit(main())
