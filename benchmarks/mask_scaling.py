#!/usr/bin/env python3
"""What a CU mask costs each stage of the multi-instance configuration C5 when the stage runs alone: the
trainer's update of the whole batch (4 x 4096 envs x horizon) per kernel class on 256 / 224 / 192 / 128 CUs,
and one agent instance's collection (4096 envs) on 256 / 64 / 32 / 16 / 8 CUs.  From these two tables the
best any agents + masked-trainer split can reach follows by arithmetic (printed as `bound_ms`): the trainer's
time on its share, or the agents' on theirs, whichever is longer, against collection + training on one
unmasked stream.  Prints one JSON object.

    python benchmarks/mask_scaling.py [--steps K]
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


def measure(config="C5", steps=5):
    import torch

    import paper_2206_08482_amd as g
    from paper_2206_08482_amd.instances import cu_masks
    from paper_2206_08482_amd.runner import PPOSession
    from workloads import synthetic as syn

    cfg = syn.get_config(config)
    n_ag = cfg.n_agents
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    thr = (1 << 32) // cfg.done_prob_inv if cfg.done_prob_inv else 0
    probe = g.gmi_create()
    n_cu = g.gmi_cu_count(probe)
    g.gmi_destroy(probe)
    n_cls = g.gmi_profile_classes()
    names = [g.gmi_profile_class_name(c) for c in range(n_cls)]
    hp = dict(epochs=cfg.epochs, minibatch=cfg.minibatch, clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, lr=cfg.lr)

    def session(n_envs, cus):
        mask = None if cus >= n_cu else cu_masks(n_cu, [cus], "contiguous")[0]
        state0 = syn.make_initial_state(n_envs, cfg.obs_dim, cfg.seed + 10)
        ses = PPOSession(n_envs=n_envs, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim, hidden=cfg.hidden,
                         horizon=cfg.horizon, dtype=cfg.dtype, theta=theta, a_mat=a_mat, b_mat=b_mat, state0=state0,
                         noise_std=cfg.noise_std, reward_scale=cfg.reward_scale, done_period=cfg.done_period,
                         done_threshold=thr, seed=cfg.seed, minibatch=cfg.minibatch, cu_mask=mask)
        s0 = torch.tensor(state0, device="cuda:0")
        torch.cuda.synchronize()
        return ses, s0

    def reset(ses, s0):
        g.gmi_transfer(ses.gmi, ses.gmi, s0, ses.obs[ses.cur], s0.numel() * 4)

    trainer_rows = []
    for cus in (256, 224, 192, 128):
        c = cus * n_cu // 256
        ses, s0 = session(n_ag * cfg.n_envs, c)
        ses.rollout(0); ses.gae(cfg.gamma, cfg.lam); ses.sync()
        for k in range(2):
            ses.update(k, **hp)
        ses.sync()
        t0 = time.perf_counter()
        for k in range(steps):
            ses.update(2 + k, **hp)
        ses.sync()
        wall = (time.perf_counter() - t0) / steps * 1e3
        g.gmi_profile_enable(ses.gmi, (1 << n_cls) - 1)
        ses.update(2 + steps, **hp)
        ses.sync()
        per = {}
        for ci, nm in enumerate(names):
            ms, launches = g.gmi_profile_read(ses.gmi, ci)
            if launches:
                per[nm] = {"ms": ms, "launches": launches}
        g.gmi_profile_enable(ses.gmi, 0)
        trainer_rows.append({"cus": c, "update_ms": wall, "per_class": per})
        ses.close()

    agent_rows = []
    for cus in (256, 64, 32, 16, 8):
        c = cus * n_cu // 256
        ses, s0 = session(cfg.n_envs, c)
        for k in range(2):
            reset(ses, s0); ses.rollout(k)
        ses.sync()
        t0 = time.perf_counter()
        for k in range(steps):
            reset(ses, s0); ses.rollout(2 + k)
        ses.sync()
        agent_rows.append({"cus": c, "collect_ms": (time.perf_counter() - t0) / steps * 1e3})
        ses.close()

    t_full = trainer_rows[0]["update_ms"]
    a_full = agent_rows[0]["collect_ms"]
    single = n_ag * a_full + t_full
    agent_ms = {r["cus"]: r["collect_ms"] for r in agent_rows}
    bounds = []
    for tr in trainer_rows[1:]:
        each = (n_cu - tr["cus"]) // n_ag // 8 * 8
        if each in agent_ms:
            b = max(tr["update_ms"], agent_ms[each])
            bounds.append({"trainer_cus": tr["cus"], "agent_cus_each": each, "bound_ms": b,
                           "single_stream_ms": single, "best_possible_vs_single": single / b})
    return {"workload": f"{cfg.name}: trainer batch {n_ag * cfg.n_envs} envs x {cfg.horizon}, agents {cfg.n_envs} envs each",
            "device_cus": n_cu, "steps": steps, "trainer_alone": trainer_rows, "agent_alone": agent_rows,
            "single_stream_collect_plus_update_ms": single, "bounds": bounds}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--config", default="C5")
    args = ap.parse_args()
    print(json.dumps(measure(args.config, args.steps)))
    return 0


if __name__ == "__main__":
    sys.exit(main())
