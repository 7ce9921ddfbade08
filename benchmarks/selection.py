#!/usr/bin/env python3
"""Instance exploration (Algorithm 2 of the paper) on one MI355X for a C2-shaped workload.

profile() runs real PPO iterations (fresh reset, T-step rollout, GAE, E epochs of two minibatches) on
`GMIperGPU` CU-masked holistic instances with `num_env` environments each; the library's `gmi_explore`
walks GMIperGPU = 10 .. 1 and num_env = 128 .. 16384 with the saturation early stop and returns the pair
with the best projected throughput.  One JSON object on stdout.

    python benchmarks/selection.py [--config C2] [--alpha 0.1] [--iterations 3]
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="C2")
    ap.add_argument("--alpha", type=float, default=0.1)
    ap.add_argument("--iterations", type=int, default=3)
    ap.add_argument("--num-gpu", type=int, default=1)
    args = ap.parse_args()

    import torch

    import paper_2206_08482_amd as g
    from paper_2206_08482_amd.runner import PPOSession
    from paper_2206_08482_amd.selection import InstanceProfiler
    from workloads import synthetic as syn

    cfg = syn.get_config(args.config)
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    thr = (1 << 32) // cfg.done_prob_inv if cfg.done_prob_inv else 0
    hp = dict(clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2,
              adam_eps=cfg.adam_eps)
    states = {}

    def build(num_env, cu_mask):
        if num_env not in states:
            states[num_env] = syn.make_initial_state(num_env, cfg.obs_dim, cfg.seed)
        ses = PPOSession(n_envs=num_env, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim, hidden=cfg.hidden,
                         horizon=cfg.horizon, dtype=cfg.dtype, theta=theta, a_mat=a_mat, b_mat=b_mat,
                         state0=states[num_env], noise_std=cfg.noise_std, reward_scale=cfg.reward_scale,
                         done_period=cfg.done_period, done_threshold=thr, seed=cfg.seed,
                         minibatch=cfg.horizon * num_env // 2, cu_mask=cu_mask)
        ses.s0 = torch.tensor(states[num_env], device="cuda:0")
        ses.ep0 = torch.zeros(num_env, dtype=torch.int32, device="cuda:0")
        return ses

    def step(ses, it):
        g.gmi_transfer(ses.gmi, ses.gmi, ses.s0, ses.obs[ses.cur], ses.s0.numel() * 4)
        g.gmi_transfer(ses.gmi, ses.gmi, ses.ep0, ses.episode_step, ses.ep0.numel() * 4)
        ses.rollout(it)
        ses.gae(cfg.gamma, cfg.lam, True)
        ses.update(it, epochs=cfg.epochs, minibatch=cfg.horizon * ses.N // 2, **hp)

    prof = InstanceProfiler(build, step, lambda n: cfg.horizon * n, iterations=args.iterations,
                            progress=lambda row: print(json.dumps(row), file=sys.stderr, flush=True))
    ks = list(range(10, 0, -1))
    ns = [128 << i for i in range(8)]
    res = g.gmi_explore(prof, args.num_gpu, args.alpha, ks, ns)
    out = {
        "workload": f"{cfg.name}-shaped: obs {cfg.obs_dim}, act {cfg.act_dim}, MLP {list(cfg.hidden)}, horizon "
                    f"{cfg.horizon}, {cfg.epochs} epochs of 2 minibatches, holistic instances",
        "alpha": args.alpha, "num_gpu": args.num_gpu, "device_cus": prof.device_cus,
        "chosen": None if res is None else {"num_env": res[0], "gmi_per_gpu": res[1],
                                            "projected_samples_per_s": res[2]},
        "points_profiled": len(prof.log), "points_in_grid": len(ks) * len(ns),
        "rows": prof.log,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
