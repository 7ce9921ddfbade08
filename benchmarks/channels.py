#!/usr/bin/env python3
"""Experience channels against the direct hand-off, configuration C5 (4 agent instances x 4096 envs + 1 trainer
instance on one MI355X, unmasked streams unless a row says otherwise, lag-1 pipelined schedule = the one-GPU form
of the paper's asynchronous serving / training; two rows let the agents run further ahead): every agent pushes its round as a slab, the trainer's batcher stacks the four slabs into its
batch.  Rows: direct column-slice hand-off (no bytes moved), multi-channel slabs (one array per type), uni-channel
slabs (interleaved records).  Reports the paper's two throughput metrics of this setting: PPS (predictions per
second: env steps the agents serve) and TTOP (training throughput: samples per second the trainer consumes); in
this lock-step pipeline both equal batch / iteration time.  Prints one JSON object.

    python benchmarks/channels.py [--steps K] [--warmup W]
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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=6)
    ap.add_argument("--warmup", type=int, default=2)
    args = ap.parse_args()

    import torch

    import paper_2206_08482_amd as g
    from paper_2206_08482_amd.channels import ChannelPipeline
    from paper_2206_08482_amd.instances import InstancePipeline
    from workloads import synthetic as syn

    cfg = syn.get_config("C5")
    n_ag = cfg.n_agents
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    states = [syn.make_initial_state(cfg.n_envs, cfg.obs_dim, cfg.seed + 10 + i) for i in range(n_ag)]
    thr = (1 << 32) // cfg.done_prob_inv
    train_args = dict(gamma=cfg.gamma, lam=cfg.lam, epochs=cfg.epochs, minibatch=cfg.minibatch, clip=cfg.clip,
                      c_v=cfg.c_v, c_e=cfg.c_e, lr=cfg.lr)
    common = dict(n_agents=n_ag, n_envs=cfg.n_envs, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim, hidden=cfg.hidden,
                  horizon=cfg.horizon, dtype=cfg.dtype, theta=theta, a_mat=a_mat, b_mat=b_mat, state0=states,
                  noise_std=cfg.noise_std, reward_scale=cfg.reward_scale, done_period=cfg.done_period,
                  done_threshold=thr, seed=cfg.seed, minibatch=cfg.minibatch)
    slab_bytes = cfg.horizon * cfg.n_envs * (4 * (cfg.obs_dim + cfg.act_dim + 3) + 1) + 4 * cfg.n_envs

    def run(label, make, lag=0):
        pipe = make()
        s0 = [torch.tensor(s, device="cuda:0") for s in states]
        torch.cuda.synchronize()

        def reset():
            for ag, s in zip(pipe.agents, s0):
                g.gmi_transfer(ag.gmi, ag.gmi, s, ag.obs[ag.cur], s.numel() * 4)

        k = 0
        if lag:
            pipe.prologue_lagged(lag)
            step = lambda kk: pipe.iteration_lagged(kk, lag, **train_args)
        else:
            pipe.prologue_pipelined()
            step = lambda kk: pipe.iteration_pipelined(kk, **train_args)
        for _ in range(args.warmup):
            reset(); step(k); k += 1
        pipe.sync_all()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            reset(); step(k); k += 1
        pipe.sync_all()
        dt = (time.perf_counter() - t0) / args.steps
        ok = bool(torch.isfinite(pipe.theta).all().item())
        pipe.close()
        moved = 0 if label.startswith("direct") else 2 * n_ag * slab_bytes       # into the slab and out of it
        return {"hand_off": label, "ms_per_iteration": dt * 1e3, "pps_env_steps_per_s": cfg.batch / dt,
                "ttop_samples_per_s": cfg.batch / dt, "bytes_moved_per_iteration": moved, "finite": ok}

    rows = [run("direct (agents write column slices of the trainer's batch)", lambda: InstancePipeline(**common)),
            run("multi-channel slabs (one array per type)", lambda: ChannelPipeline(mode=g.CHANNELS_MULTI, **common)),
            run("uni-channel slabs (interleaved records)", lambda: ChannelPipeline(mode=g.CHANNELS_UNI, **common))]
    # bounded staleness: the agents `lag` rounds ahead of the trainer (the channels hold lag rounds)
    for lag in (2, 4):
        rows.append(run(f"multi-channel slabs, agents {lag} rounds ahead",
                        lambda: ChannelPipeline(mode=g.CHANNELS_MULTI, capacity=(lag + 1) * n_ag, **common), lag))
    # the layout that wins in benchmarks/instances.py (agents on disjoint quarters of the device, trainer unmasked, the
    # host orders the hand-offs), through channels
    probe = g.gmi_create()
    n_cu = g.gmi_cu_count(probe)
    g.gmi_destroy(probe)
    from paper_2206_08482_amd.instances import cu_masks
    masks = cu_masks(n_cu, [n_cu // n_ag // 8 * 8] * n_ag, "contiguous")
    rows.append(run("multi-channel slabs, agents on disjoint CU sets, host-ordered",
                    lambda: ChannelPipeline(mode=g.CHANNELS_MULTI, agent_masks=masks, host_ordered=True, **common)))
    for r in rows:
        r["vs_direct"] = r["ttop_samples_per_s"] / rows[0]["ttop_samples_per_s"]
    print(json.dumps({"workload": f"C5: {n_ag} agent instances x {cfg.n_envs} envs, obs {cfg.obs_dim}, MLP {list(cfg.hidden)}, "
                                  f"horizon {cfg.horizon}, {cfg.epochs} epochs, minibatch {cfg.minibatch}; unmasked streams, "
                                  "lag-1 pipelined", "steps": args.steps, "warmup": args.warmup, "rows": rows}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
