#!/usr/bin/env python3
"""Asynchronous serving / training on the multi-instance configuration C5 (4 agent instances x 4096 envs + 1
trainer instance, each driven by its own host thread, experience through the channels): PPS (env steps per
second the agents serve) and TTOP (samples per second the trainer consumes) for a ring whose full state makes
the agents wait, and for one where they discard the oldest slab instead; with all instances unmasked and with the
agents on disjoint quarters of the device.  The lock-step lag-1 pipeline of benchmarks/channels.py is the
comparison point (there PPS = TTOP by construction).  Prints one JSON object.

    python benchmarks/async_rates.py [--updates K]
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def measure(config="C5", updates=8):
    import torch

    import paper_2206_08482_amd as g
    from paper_2206_08482_amd.async_schedule import AsyncPipeline
    from paper_2206_08482_amd.instances import cu_masks
    from workloads import synthetic as syn

    cfg = syn.get_config(config)
    n_ag = cfg.n_agents
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    thr = (1 << 32) // cfg.done_prob_inv if cfg.done_prob_inv else 0
    probe = g.gmi_create()
    n_cu = g.gmi_cu_count(probe)
    g.gmi_destroy(probe)
    quarters = cu_masks(n_cu, [n_cu // n_ag // 8 * 8] * n_ag, "contiguous")
    small = cu_masks(n_cu, [8 * n_cu // 256] * n_ag + [n_cu - n_ag * 8 * n_cu // 256], "contiguous")
    train_args = dict(gamma=cfg.gamma, lam=cfg.lam, epochs=cfg.epochs, minibatch=cfg.minibatch, clip=cfg.clip,
                      c_v=cfg.c_v, c_e=cfg.c_e, lr=cfg.lr)
    rows = []
    for label, on_full, a_masks, t_mask in (
            ("unmasked, agents wait when the ring is full", "block", None, None),
            ("unmasked, agents discard the oldest slab", "drop_oldest", None, None),
            ("agents on disjoint quarters, trainer unmasked, agents wait", "block", quarters, None),
            ("agents on disjoint quarters, trainer unmasked, agents discard", "drop_oldest", quarters, None),
            ("agents 8 CUs each, trainer the rest, agents wait", "block", small[:n_ag], small[n_ag])):
        # the synthetic dynamics are unstable over many rounds: fresh states per row, few rounds per row
        states = [syn.make_initial_state(cfg.n_envs, cfg.obs_dim, cfg.seed + 10 + i) for i in range(n_ag)]
        pipe = AsyncPipeline(n_agents=n_ag, n_envs=cfg.n_envs, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim,
                             hidden=cfg.hidden, horizon=cfg.horizon, dtype=cfg.dtype, theta=theta, a_mat=a_mat,
                             b_mat=b_mat, state0=states, noise_std=cfg.noise_std, reward_scale=cfg.reward_scale,
                             done_period=cfg.done_period, done_threshold=thr, seed=cfg.seed, minibatch=cfg.minibatch,
                             slabs_per_update=n_ag, capacity=2 * n_ag, on_full=on_full, agent_masks=a_masks,
                             trainer_mask=t_mask, reset_each_round=True)
        pipe.run(2, **train_args)           # warm-up
        r = pipe.run(updates, **train_args)
        lags = []
        for e in pipe.trace:
            if e[0] == "update":
                lags += [e[1] - s[2] for s in e[2]]      # updates made since the slab's parameters were current
        r.update({"layout": label, "on_full": on_full, "mean_staleness_updates": sum(lags) / max(len(lags), 1),
                  "max_staleness_updates": max(lags) if lags else 0})
        r["finite"] = bool(torch.isfinite(pipe.theta).all().item())
        rows.append(r)
        pipe.close()
    return {"workload": f"{cfg.name}: {n_ag} agent instances x {cfg.n_envs} envs, obs {cfg.obs_dim}, MLP "
                        f"{list(cfg.hidden)}, horizon {cfg.horizon}, {cfg.epochs} epochs, minibatch {cfg.minibatch}; "
                        f"{n_ag} slabs per update, ring of {2 * n_ag} slabs",
            "updates_timed": updates, "rows": rows}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--updates", type=int, default=8)
    ap.add_argument("--config", default="C5")
    args = ap.parse_args()
    print(json.dumps(measure(args.config, args.updates)))
    return 0


if __name__ == "__main__":
    sys.exit(main())
