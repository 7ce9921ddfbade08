#!/usr/bin/env python3
"""CU-split sweep for the multi-instance configuration C5: 4 agent instances (4096 envs each) + 1 trainer
instance on CU-masked streams of one MI355X, lag-1 pipelined schedule, against the same work on a single
unmasked stream with the synchronous schedule.  Prints one JSON object with a row per layout.

    python benchmarks/instances.py [--steps K] [--warmup W] [--config C5]
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


def sweep(config="C5", steps=6, warmup=2, full=True):
    """Times the layouts of the multi-instance configuration; returns the report as a dict.  full=False: the single
    stream, the three agent/trainer splits the configuration names (contiguous masks, both hand-offs) and the
    layout with the agents on disjoint quarters of the device and an unmasked trainer."""
    import torch

    import paper_2206_08482_amd as g
    from paper_2206_08482_amd.instances import InstancePipeline, cu_masks
    from workloads import synthetic as syn

    cfg = syn.get_config(config)
    n_ag = cfg.n_agents
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    states = [syn.make_initial_state(cfg.n_envs, cfg.obs_dim, cfg.seed + 10 + i) for i in range(n_ag)]
    thr = (1 << 32) // cfg.done_prob_inv if cfg.done_prob_inv else 0
    probe = g.gmi_create()
    n_cu = g.gmi_cu_count(probe)
    g.gmi_destroy(probe)
    train_args = dict(gamma=cfg.gamma, lam=cfg.lam, epochs=cfg.epochs, minibatch=cfg.minibatch, clip=cfg.clip,
                      c_v=cfg.c_v, c_e=cfg.c_e, lr=cfg.lr)

    def run(label, schedule, agent_masks, trainer_mask, single_stream, host_ordered=False):
        pipe = InstancePipeline(n_agents=n_ag, n_envs=cfg.n_envs, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim,
                                hidden=cfg.hidden, horizon=cfg.horizon, dtype=cfg.dtype, theta=theta, a_mat=a_mat,
                                b_mat=b_mat, state0=states, noise_std=cfg.noise_std, reward_scale=cfg.reward_scale,
                                done_period=cfg.done_period, done_threshold=thr, seed=cfg.seed,
                                minibatch=cfg.minibatch, agent_masks=agent_masks, trainer_mask=trainer_mask,
                                single_stream=single_stream, host_ordered=host_ordered)
        s0 = [torch.tensor(s, device="cuda:0") for s in states]
        torch.cuda.synchronize()

        def reset():      # fresh env states every iteration (the synthetic dynamics are unstable)
            for ag, s in zip(pipe.agents, s0):
                g.gmi_transfer(ag.gmi, ag.gmi, s, ag.obs[ag.cur], s.numel() * 4)

        k = 0
        if schedule == "pipelined":
            pipe.prologue_pipelined()
        step = pipe.iteration_sync if schedule == "sync" else pipe.iteration_pipelined
        for _ in range(warmup):
            reset(); step(k, **train_args); k += 1
        pipe.sync_all()
        t0 = time.perf_counter()
        for _ in range(steps):
            reset(); step(k, **train_args); k += 1
        pipe.sync_all()
        dt = (time.perf_counter() - t0) / steps
        ok = bool(torch.isfinite(pipe.theta).all().item())
        a_cus, t_cus = pipe.cu_counts()
        pipe.close()
        return {"layout": label, "schedule": schedule, "hand_off": "host" if host_ordered else "events", "agent_cus_each": a_cus[0], "trainer_cus": t_cus,
                "ms_per_iteration": dt * 1e3, "samples_per_s": cfg.batch / dt, "finite": ok}

    rows = [run("single unmasked stream", "sync", None, None, True)]
    if full:
        rows += [run("5 unmasked streams", "sync", None, None, False),
                 run("5 unmasked streams", "pipelined", None, None, False)]
    for agents_total, trainer in ((192, 64), (128, 128), (64, 192)) + (((32, 224),) if full else ()):
        a = agents_total * n_cu // 256
        t = n_cu - a
        for style in ("contiguous", "interleaved") if full else ("contiguous",):
            # the agents' share is split evenly over the agent instances
            masks = cu_masks(n_cu, [a // n_ag // 8 * 8] * n_ag + [t], style)
            for ho in (False, True):
                rows.append(run(f"agents {a}/{n_ag} + trainer {t} CUs, {style}", "pipelined", masks[:n_ag], masks[n_ag],
                                False, ho))
            if full:      # the agents share one CU set
                shared = cu_masks(n_cu, [a, t], style)
                rows.append(run(f"agents share {a} + trainer {t} CUs, {style}", "pipelined", [shared[0]] * n_ag, shared[1], False))
    # the agents on disjoint CU sets that together cover the device, the trainer on all of it: with the synchronous
    # schedule the two stages never run at the same time, so the trainer needs no mask of its own
    for style in ("contiguous", "interleaved") if full else ("contiguous",):
        for parts in (n_ag, 2) if full else (n_ag,):
            masks = cu_masks(n_cu, [n_cu // parts // 8 * 8] * parts, style)
            masks = [masks[i % parts] for i in range(n_ag)]
            for schedule, ho in (("sync", False), ("sync", True), ("pipelined", True)) if full else (("sync", True),):
                rows.append(run(f"agents on {parts} disjoint sets of {n_cu // parts} CUs, trainer unmasked, {style}", schedule,
                                masks, None, False, ho))
    if full:
        rows.append(run("5 unmasked streams", "sync", None, None, False, True))
    base = rows[0]["samples_per_s"]
    for r in rows:
        r["vs_single_stream"] = r["samples_per_s"] / base
    best = max(rows[1:], key=lambda r: r["samples_per_s"])
    return {"workload": f"{cfg.name}: {n_ag} agent instances x {cfg.n_envs} envs, obs {cfg.obs_dim}, MLP "
                        f"{list(cfg.hidden)}, horizon {cfg.horizon}, {cfg.epochs} epochs, minibatch {cfg.minibatch}",
            "device_cus": n_cu, "steps": steps, "warmup": warmup, "rows": rows,
            "best": best["layout"] + " / " + best["schedule"] + " / " + best["hand_off"],
            "best_vs_single_stream": best["vs_single_stream"]}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=6)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="C5")
    ap.add_argument("--headline", action="store_true", help="only the layouts bench.py reports")
    args = ap.parse_args()
    print(json.dumps(sweep(args.config, args.steps, args.warmup, full=not args.headline)))
    return 0


if __name__ == "__main__":
    sys.exit(main())
