#!/usr/bin/env python3
"""Holistic instances with synchronized training on one MI355X (the paper's TCG_EX layout, Section 5.1, with
the gradient reduction of Section 4.1 as an in-memory mean): k CU-masked instances, each simulating
n_total / k environments and training a replica of one model on its own experience, against one unmasked
instance doing the same total work.  The union minibatch has the same size in every row, so all rows take
the same number of Adam steps on the same number of samples.  Prints one JSON object.

    python benchmarks/group.py [--config C2] [--envs 16384] [--steps K] [--warmup W]
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
    ap.add_argument("--config", default="C2")
    ap.add_argument("--envs", type=int, default=16384, help="environments in total, over all instances")
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    args = ap.parse_args()

    import torch

    import paper_2206_08482_amd as g
    from paper_2206_08482_amd.instances import cu_masks
    from paper_2206_08482_amd.runner import PPOSession
    from workloads import synthetic as syn

    cfg = syn.get_config(args.config)
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    thr = (1 << 32) // cfg.done_prob_inv if cfg.done_prob_inv else 0
    probe = g.gmi_create()
    n_cu = g.gmi_cu_count(probe)
    g.gmi_destroy(probe)
    hp = dict(clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, lr=cfg.lr)
    batch = args.envs * cfg.horizon

    def run(k: int, masked: bool, synchronized: bool):
        n = args.envs // k
        mb = cfg.minibatch // k
        masks = cu_masks(n_cu, [n_cu // k // 8 * 8] * k, "contiguous") if masked else [None] * k
        states = [syn.make_initial_state(n, cfg.obs_dim, cfg.seed + i) for i in range(k)]
        ses = []
        for i in range(k):
            ses.append(PPOSession(
                n_envs=n, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim, hidden=cfg.hidden, horizon=cfg.horizon,
                dtype=cfg.dtype, theta=theta, a_mat=a_mat, b_mat=b_mat, state0=states[i], noise_std=cfg.noise_std,
                reward_scale=cfg.reward_scale, done_period=cfg.done_period, done_threshold=thr, seed=cfg.seed,
                minibatch=mb, cu_mask=masks[i], env_offset=i * n,
                replica_of=ses[0] if (i and synchronized) else None))
        s0 = [torch.tensor(s, device="cuda:0") for s in states]
        torch.cuda.synchronize()

        def step(it: int) -> None:
            for s, x in zip(ses, s0):       # fresh env states (the synthetic dynamics are unstable)
                g.gmi_transfer(s.gmi, s.gmi, x, s.obs[s.cur], x.numel() * 4)
                s.rollout(it)
                s.gae(cfg.gamma, cfg.lam, True)
            if synchronized and k > 1:
                PPOSession.update_group(ses, it, epochs=cfg.epochs, minibatch=mb, **hp)
            else:
                for s in ses:
                    s.update(it, epochs=cfg.epochs, minibatch=mb, **hp)

        it = 0
        for _ in range(args.warmup):
            step(it); it += 1
        for s in ses:
            s.sync()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(it); it += 1
        for s in ses:
            s.sync()
        dt = (time.perf_counter() - t0) / args.steps
        ok = all(bool(torch.isfinite(s.theta).all().item()) for s in ses)
        cus = g.gmi_cu_count(ses[0].gmi)
        for s in reversed(ses):
            s.close()
        return {"instances": k, "envs_per_instance": n, "minibatch_per_instance": mb, "cus_per_instance": cus,
                "masked": masked, "training": "synchronized (in-memory gradient mean)" if synchronized and k > 1
                else ("independent replicas" if k > 1 else "single instance"),
                "ms_per_iteration": dt * 1e3, "samples_per_s": batch / dt, "finite": ok}

    rows = [run(1, False, False)]
    for k in (2, 4):
        rows.append(run(k, True, True))
        rows.append(run(k, True, False))
        rows.append(run(k, False, True))
    base = rows[0]["samples_per_s"]
    for r in rows:
        r["vs_single_instance"] = r["samples_per_s"] / base
    print(json.dumps({"workload": f"{cfg.name}-shaped: {args.envs} envs in total, obs {cfg.obs_dim}, MLP "
                                  f"{list(cfg.hidden)}, horizon {cfg.horizon}, {cfg.epochs} epochs, union minibatch "
                                  f"{cfg.minibatch}", "device_cus": n_cu, "steps": args.steps, "warmup": args.warmup,
                      "rows": rows}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
