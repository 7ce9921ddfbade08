#!/usr/bin/env python3
"""The agent's action decision in bf16 (agent_act, the serving path of the benchmark configurations) and in fp8
(agent_act_fp8: E4M3 weights and activations) on the benchmark model shapes: microseconds per call at the
configurations' env counts and at 2^18 envs, and the relative L2 distance of the fp8 means from the bf16 ones.
Calls are queued back to back on one instance and timed on the host around a final synchronisation.  One JSON
object on stdout.

    python benchmarks/inference_precision.py [--reps R]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def measure(reps=50):
    import numpy as np
    import torch

    import paper_2206_08482_amd as g
    from workloads import synthetic as syn

    dev = torch.device("cuda:0")
    h = g.gmi_create()
    rows = []
    for name in ("C2", "C3", "C4"):
        cfg = syn.get_config(name)
        theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
        for n in (cfg.n_envs, 1 << 18):
            obs = torch.tensor(syn.make_initial_state(n, cfg.obs_dim, cfg.seed), device=dev)
            th = torch.tensor(theta, device=dev)
            desc = g.model_desc(cfg.obs_dim, cfg.act_dim, list(cfg.hidden), g.dtype_code("bf16"), n)
            shadow = torch.zeros(max(g.gmi_model_shadow_bytes(desc), 256), dtype=torch.uint8, device=dev)
            out = {k: (torch.zeros(n, cfg.act_dim, device=dev), torch.zeros(n, cfg.act_dim, device=dev),
                       torch.zeros(n, device=dev), torch.zeros(n, device=dev)) for k in ("bf16", "fp8")}
            torch.cuda.synchronize()
            model = g.gmi_model_bind(h, desc, th, shadow, None, None)
            g.gmi_model_refresh_shadow(h, model)
            w8 = g.gmi_fp8_bind(h, desc)
            g.gmi_fp8_refresh(h, w8, th)

            def call(kind):
                act, mu, logp, val = out[kind]
                if kind == "bf16":
                    g.agent_act(h, model, obs, n, cfg.seed, 0, 0, act, logp, val, mu)
                else:
                    g.agent_act_fp8(h, w8, obs, n, cfg.seed, 0, 0, act, logp, val, mu)

            us = {}
            for kind in ("bf16", "fp8"):
                for _ in range(3):
                    call(kind)
                g.gmi_sync(h)
                t0 = time.perf_counter()
                for _ in range(reps):
                    call(kind)
                g.gmi_sync(h)
                us[kind] = (time.perf_counter() - t0) / reps * 1e6
            mu16, mu8 = out["bf16"][1].cpu().numpy().astype(np.float64), out["fp8"][1].cpu().numpy().astype(np.float64)
            rows.append({"model": f"{name}: obs {cfg.obs_dim}, {list(cfg.hidden)}", "envs": n, "bf16_us": us["bf16"],
                         "fp8_us": us["fp8"], "fp8_speedup": us["bf16"] / us["fp8"],
                         "mu_rel_l2_fp8_vs_bf16": float(np.linalg.norm(mu8 - mu16) / np.linalg.norm(mu16))})
            g.gmi_fp8_destroy(w8)
            g.gmi_model_destroy(model)
            del obs, out
    g.gmi_destroy(h)
    return {"reps": reps, "rows": rows}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=50)
    args = ap.parse_args()
    print(json.dumps(measure(args.reps)))
    return 0


if __name__ == "__main__":
    sys.exit(main())
