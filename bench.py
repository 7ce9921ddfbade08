#!/usr/bin/env python3
"""Benchmark of the PPO agent/trainer hot path on one MI355X.

A "step" is one whole PPO iteration over one batch of synthetic experience: T rounds of
[agent_act -> env_step -> collect_experience], the bootstrap value, gae_compute, and ppo_update
(E epochs of shuffled minibatches: forward, loss, backward, Adam).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C4] [--no-cpu-baseline] [--no-extras]

The default run also reports, as extra keys of the same line, the step times of the other single-instance
workloads, the agent/trainer CU-split sweep of the multi-instance configuration (benchmarks/instances.py), its
asynchronous serving / training rates (benchmarks/async_rates.py), the bandwidth-bound kernels on scaled inputs
(benchmarks/kernels.py) and the fp8 agents against the bf16 ones (benchmarks/inference_precision.py).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_FP32_TFLOPS = 157.3       # vector fp32

# HBM bytes per launch (fetch + write) of the kernels that dominate the bench workloads, from the
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in profiles/hbm_traffic_C2_C4.md (counter values
# scaled by what the same counters read for a copy kernel of known size).  Keyed by (workload, class).
MEASURED_TRAFFIC = {
    ("C2", "chain_train"): 209.18e6, ("C2", "wgrad"): 163.62e6, ("C2", "fused_rollout"): 36.40e6,
    ("C4", "chain_train"): 669.47e6, ("C4", "wgrad"): 689.71e6, ("C4", "adam"): 104.91e6,
}


def mac_per_sample(cfg, first_layer=True):
    """Multiply-accumulates of one forward of both nets for one sample (unpadded)."""
    total = 0
    for out_dim in (cfg.act_dim, 1):
        prev = cfg.obs_dim
        for li, h in enumerate(list(cfg.hidden) + [out_dim]):
            if first_layer or li > 0:
                total += prev * h
            prev = h
    return total


def pad32(x):
    return (x + 31) // 32 * 32


def layer_bytes_per_sample(cfg, es, first_layer=True):
    """Activation bytes one sample moves through the per-layer kernels of both nets: each layer reads its
    (padded) input row and writes its (padded) output row; the fp32 heads write 4 bytes per output."""
    total = 0
    for out_dim in (cfg.act_dim, 1):
        prev = cfg.obs_dim
        dims = list(cfg.hidden) + [out_dim]
        for li, h in enumerate(dims):
            if first_layer or li > 0:
                total += pad32(prev) * es + (4 * h if li == len(dims) - 1 else pad32(h) * es)
            prev = h
    return total


def class_work(cfg, n_params, launched):
    """Algorithmic work per *step* of the kernel classes whose launchers do not state it themselves
    (the linear-layer and weight-gradient classes report theirs through gmi_profile_work): HBM bytes and,
    for the fused kernels, flops; plus the whole step's matrix-product flops.
    `launched` maps class name -> launches seen in the profiled step."""
    N, T, B, MB, E = cfg.n_envs, cfg.horizon, cfg.batch, cfg.minibatch, cfg.epochs
    O, A, L = cfg.obs_dim, cfg.act_dim, len(cfg.hidden)
    mac = mac_per_sample(cfg)
    mac_dgrad = mac_per_sample(cfg, first_layer=False)        # no input gradient for the first layer
    mac_value = sum(a * b for a, b in zip([O] + list(cfg.hidden), list(cfg.hidden) + [1]))
    n_upd = E * (B // MB)
    es = 2 if cfg.dtype == "bf16" else 4
    w_bytes = n_params * es
    act_b = layer_bytes_per_sample(cfg, es)
    rollout_flops = 2.0 * (T * N * mac + N * mac_value)
    per_layer_rollout = not (launched.get("fused_agent") or launched.get("fused_rollout"))
    exp_bytes = T * N * (4.0 * (O + A + 3) + 1)               # one step's experience slot, all envs
    return {
        "gather": dict(bytes=(T + 1) * N * O * (4 + es) * (1 if per_layer_rollout else 0)
                       + n_upd * MB * (O * (4 + es) + 8.0 * (A + 3) + 4),
                       launches=(T + 1 if per_layer_rollout else 0) + n_upd),
        "loss": dict(bytes=n_upd * MB * (4.0 * (2 * A + 5) + es * (A + 1)), launches=n_upd),
        "adam": dict(bytes=n_upd * n_params * (16.0 + 12.0 + (3 * es if cfg.dtype == "bf16" else 0)), launches=n_upd),
        "env_step": dict(bytes=T * N * (4.0 * (2 * O + A) + 8 + 1), launches=T),
        "sample": dict(bytes=T * N * 4.0 * (2 * A + 1), launches=T),
        "collect": dict(bytes=2 * exp_bytes, launches=T),
        "gae": dict(bytes=B * (9.0 + 8.0 + 8.0) + 4.0 * N, launches=1),
        "permutation": dict(bytes=E * B * 4.0, launches=E),
        # fused kernels: all layers of both nets for a tile of rows in one launch
        "fused_agent": dict(flops=rollout_flops, bytes=T * N * 4.0 * (O + 2 * A + 2) + (T + 1) * w_bytes,
                            launches=T + 1),
        "fused_rollout": dict(flops=rollout_flops, bytes=exp_bytes + 8.0 * N * O + w_bytes, launches=1),
    }, 2.0 * (T * N * mac + N * mac_value + n_upd * MB * (2 * mac + mac_dgrad))


def cpu_baseline(cfg, budget_s=12.0):
    """The numpy oracle, as it stands, on the host cores: whole iterations of the same workload -- of a slice of
    its environments where one iteration of all of them would take minutes (the sample is stated in the result)."""
    import dataclasses

    import numpy as np

    from oracle import ppo as oppo
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from gpu_util import oracle_pieces
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    # about 2e11 matrix-product flops per iteration keep one iteration within the budget on a host like the GPU machine's
    _, flops_iter = class_work(cfg, 0, {})
    n_envs = cfg.n_envs
    while flops_iter * n_envs / cfg.n_envs > 1.2e12 and n_envs * cfg.horizon > cfg.minibatch and n_envs % 2 == 0:
        n_envs //= 2
    sub = dataclasses.replace(cfg, n_envs=n_envs) if n_envs != cfg.n_envs else cfg
    shape, theta, env, state0, hp = oracle_pieces(sub)
    z = np.zeros_like(theta)
    n_it, t0 = 0, time.perf_counter()
    m, v, k = z, z, 0
    while True:
        out = oppo.ppo_iteration(theta, m, v, k, shape, env, state0, np.zeros(sub.n_envs, np.uint32), sub.horizon,
                                 hp, sub.gamma, sub.lam, sub.seed, n_it)
        theta, m, v, k = out["theta"], out["m"], out["v"], out["k"]
        n_it += 1
        el = time.perf_counter() - t0
        if el >= budget_s or el * (n_it + 1) / n_it > 2.5 * budget_s:
            break
    what = (f"{n_it} whole iteration(s) of {cfg.name}" if sub is cfg else
            f"{n_it} whole iteration(s) of {cfg.name} on {sub.n_envs} of its {cfg.n_envs} environments (same horizon, "
            f"epochs and minibatch size)")
    return {"value": n_it * sub.batch / el, "unit": "samples/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{what} ({sub.batch} samples each, fresh reset) in {el:.1f} s, numpy fp32 with its BLAS threads"}


# kernel classes whose work is matrix products (judged against the matrix-core roof)
def is_matrix_class(name):
    return name in ("chain_train", "wgrad", "fused_agent", "fused_rollout") or name.startswith("linear_")


def run_workload(g, torch, syn, PPOSession, name, steps, warmup, fusion=None, detail=True):
    """Times `steps` whole PPO iterations of workload `name` on one unmasked instance.  detail: also the per-class
    kernel times of the last warm-up step and the launch timer on the dominant class during the timed steps."""
    cfg = syn.get_config(name)
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    state0 = syn.make_initial_state(cfg.n_envs, cfg.obs_dim, cfg.seed)
    thr = (1 << 32) // cfg.done_prob_inv if cfg.done_prob_inv else 0
    ses = PPOSession(n_envs=cfg.n_envs, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim, hidden=cfg.hidden,
                     horizon=cfg.horizon, dtype=cfg.dtype, theta=theta, a_mat=a_mat, b_mat=b_mat, state0=state0,
                     noise_std=cfg.noise_std, reward_scale=cfg.reward_scale, done_period=cfg.done_period,
                     done_threshold=thr, seed=cfg.seed, minibatch=cfg.minibatch)
    if fusion is not None:
        g.gmi_set_fusion(ses.gmi, fusion)
        ses.fused_rollout = ses.fused_rollout and fusion >= 1
    s0 = torch.tensor(state0, device="cuda:0")
    ep0 = torch.zeros(cfg.n_envs, dtype=torch.int32, device="cuda:0")
    torch.cuda.synchronize()
    hp = dict(clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2,
              adam_eps=cfg.adam_eps)

    def step(it: int) -> None:
        # fresh reset of the environments (the synthetic dynamics are unstable over long horizons):
        # two small device-to-device copies on the instance's own stream, inside the timed region
        g.gmi_transfer(ses.gmi, ses.gmi, s0, ses.obs[ses.cur], s0.numel() * 4)
        g.gmi_transfer(ses.gmi, ses.gmi, ep0, ses.episode_step, ep0.numel() * 4)
        ses.rollout(it)
        ses.gae(cfg.gamma, cfg.lam, True)
        ses.update(it, epochs=cfg.epochs, minibatch=cfg.minibatch, **hp)

    n_cls = g.gmi_profile_classes()
    names = [g.gmi_profile_class_name(c) for c in range(n_cls)]
    it = 0
    res = {"cfg": cfg, "n_params": int(ses.theta.numel())}
    for _ in range(max(warmup - 1, 0)):
        step(it); it += 1
    if detail:
        # last warm-up step with every class timed: finds the kernel class that dominates the step
        g.gmi_profile_enable(ses.gmi, (1 << n_cls) - 1)
    step(it); it += 1
    if detail:
        per_class = {names[c]: g.gmi_profile_read(ses.gmi, c) for c in range(n_cls)}
        dominant = max(per_class, key=lambda k: per_class[k][0])
        g.gmi_profile_enable(ses.gmi, 1 << names.index(dominant))
        res.update(per_class=per_class, dominant=dominant)

    ses.sync(); torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(it); it += 1
    ses.sync(); torch.cuda.synchronize()
    t1 = time.perf_counter()
    if detail:
        res["dom_ms"], res["dom_launches"] = g.gmi_profile_read(ses.gmi, names.index(dominant))
        res["dom_flops"], res["dom_bytes"] = g.gmi_profile_work(ses.gmi, names.index(dominant))
        g.gmi_profile_enable(ses.gmi, 0)
    assert torch.isfinite(ses.theta).all().item(), "parameters are not finite after the timed steps"
    res["seconds"] = t1 - t0

    # rollout alone (env-steps/s), untimed part of the report
    ses.sync()
    r0 = time.perf_counter()
    for _ in range(max(1, steps // 2)):
        g.gmi_transfer(ses.gmi, ses.gmi, s0, ses.obs[ses.cur], s0.numel() * 4)
        ses.rollout(it); it += 1
    ses.sync()
    res["env_steps_per_s"] = max(1, steps // 2) * cfg.batch / (time.perf_counter() - r0)
    ses.close()
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C4",
                    help="C4 (default): the largest single-instance workload, the one the matrix-core target is set on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the other workloads, the instance-split sweep, the asynchronous rates, the scaled bandwidth "
                         "kernels and the fp8 agents")
    ap.add_argument("--fusion", type=int, default=None,
                    help="fusion level of the instance (0 per-layer kernels only, 1 fused agent/rollout and trainer "
                         "kernels); default: the library's")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (its instances are CU-masked streams of one device); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import torch

    import paper_2206_08482_amd as g
    from paper_2206_08482_amd.runner import PPOSession
    from workloads import synthetic as syn
    sys.path.insert(0, os.path.join(ROOT, "tests"))

    if syn.get_config(args.config).n_agents != 1:
        print("bench.py: the multi-instance configuration is measured by benchmarks/instances.py (its summary is in "
              "the default run's c5_split_sweep)", file=sys.stderr)
        return 2
    r = run_workload(g, torch, syn, PPOSession, args.config, args.steps, args.warmup, args.fusion)
    cfg, per_class, dominant = r["cfg"], r["per_class"], r["dominant"]
    dom_ms, dom_launches, dom_flops, dom_bytes = r["dom_ms"], r["dom_launches"], r["dom_flops"], r["dom_bytes"]

    ms_per_step = r["seconds"] * 1e3 / args.steps
    value = args.steps * cfg.batch / r["seconds"]
    work, flops_step = class_work(cfg, r["n_params"], {k: v[1] for k, v in per_class.items()})
    avg_ms = dom_ms / max(dom_launches, 1)
    if dom_flops > 0 or dom_bytes > 0:          # stated by the launcher for exactly the timed launches
        flops_per_launch, bytes_per_launch = dom_flops / dom_launches, dom_bytes / dom_launches
    else:
        w = work.get(dominant, {"launches": 1})       # a class without stated work (only ever dominant under a profiler)
        flops_per_launch = w.get("flops", 0.0) / max(w["launches"], 1)
        bytes_per_launch = w.get("bytes", 0.0) / max(w["launches"], 1)
    # the roof: a kernel made of matrix products is judged against the matrix cores (unpadded 2 * MAC flops of its
    # launch / its time / the dense peak of its operand type), every other kernel against HBM
    peak_flops = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_TFLOPS
    traffic = MEASURED_TRAFFIC.get((cfg.name, dominant))
    if is_matrix_class(dominant) and flops_per_launch > 0:
        roof = {"bound": "mfma", "achieved": flops_per_launch / (avg_ms * 1e-3) / 1e12, "peak": peak_flops,
                "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": bytes_per_launch / (avg_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = traffic
    roof["kernel"] = dominant
    roof["avg_launch_us"] = avg_ms * 1e3
    roof["launches_timed"] = dom_launches
    roof["algorithmic_flops_per_launch"] = flops_per_launch
    # the HBM view of the same launches: the bytes the launcher calls algorithmic for its present design, and the
    # measured traffic, each over the kernel's time and the 8 TB/s peak
    roof["algorithmic_bytes_per_launch"] = bytes_per_launch
    roof["hbm_frac_algorithmic"] = bytes_per_launch / (avg_ms * 1e-3) / 1e9 / PEAK_HBM_GBS
    roof["hbm_frac_measured"] = traffic / (avg_ms * 1e-3) / 1e9 / PEAK_HBM_GBS if traffic else None

    total_ms = sum(v[0] for v in per_class.values())
    breakdown = {k: {"ms_per_step": round(v[0], 4), "launches": v[1]} for k, v in per_class.items() if v[1]}
    whole_tflops = flops_step / (ms_per_step * 1e-3) / 1e12
    out = {
        "metric": "PPO samples/sec (rollout+update) on 1 MI355X",
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_envs} envs, obs {cfg.obs_dim}, act {cfg.act_dim}, MLP "
                               f"{list(cfg.hidden)} ELU x2 nets, horizon {cfg.horizon}, {cfg.epochs} epochs, "
                               f"minibatch {cfg.minibatch}, linear-Gaussian env, one unmasked instance",
                   "samples_per_step": cfg.batch},
        "roofline": roof,
        "env_steps_per_s": r["env_steps_per_s"],
        "mlp_gemm_tflops_whole_step": whole_tflops,
        "mfma_frac_whole_step": whole_tflops / peak_flops,
        "kernel_ms_in_profiled_step": breakdown,
        "kernel_ms_sum": total_ms,
        "paper_context": "GMI-DRL reports up to 2.81x over Isaac Gym+NCCL on DGX-A100 (different hardware, env, baseline)",
    }
    if not args.no_extras:
        # the other single-instance workloads (fewer steps), the instance-split sweep of the multi-instance
        # configuration, its asynchronous rates, the bandwidth-bound kernels on inputs large enough for HBM to bound
        # them, and the fp8 agents against the bf16 ones.  A failure in one of them is recorded under its key and
        # does not cost the line.
        def extra(key, fn):
            try:
                out[key] = fn()
            except Exception as e:      # noqa: BLE001
                out[key] = {"error": f"{type(e).__name__}: {e}"}

        def others():
            res = {}
            for name in ("C2", "C3", "C4"):
                if name == cfg.name:
                    continue
                n = max(5, args.steps // 2)
                o = run_workload(g, torch, syn, PPOSession, name, n, 2, args.fusion, detail=False)
                res[name] = {"ms_per_step": o["seconds"] * 1e3 / n, "samples_per_s": n * o["cfg"].batch / o["seconds"],
                             "env_steps_per_s": o["env_steps_per_s"]}
            return res

        def split_sweep():
            from benchmarks import instances as binst
            sw = binst.sweep("C5", steps=4, warmup=2, full=False)
            return {"workload": sw["workload"], "single_stream_ms": sw["rows"][0]["ms_per_iteration"],
                    "best": sw["best"], "best_vs_single_stream": sw["best_vs_single_stream"],
                    "rows": [{k: (round(v, 4) if isinstance(v, float) else v) for k, v in row.items()
                              if k in ("layout", "schedule", "hand_off", "ms_per_iteration", "vs_single_stream")}
                             for row in sw["rows"]]}

        def async_rates():
            from benchmarks import async_rates as basy
            r = basy.measure("C5", updates=4)
            return {"workload": r["workload"],
                    "rows": [{"layout": row["layout"], "pps_env_steps_per_s": round(row["pps_env_steps_per_s"]),
                              "ttop_samples_per_s": round(row["ttop_samples_per_s"]),
                              "slabs_discarded": row["slabs_discarded"],
                              "mean_staleness_updates": round(row["mean_staleness_updates"], 2)} for row in r["rows"]]}

        def scaled_kernels():
            from benchmarks import kernels as bker
            bk = bker.measure(large_only=True)
            return {"copy_kernel_GBs": bk["copy_kernel_GBs"],
                    "rows": [{"kernel": row["kernel"], "size": row["size"], "GBs": round(row["GBs"], 1),
                              "frac_of_hbm_peak": round(row["frac_of_hbm_peak"], 4),
                              **({"fp32_TFLOPs": round(row["fp32_TFLOPs"], 2)} if "fp32_TFLOPs" in row else {})}
                             for row in bk["rows"]]}

        def fp8_agents():
            from benchmarks import inference_precision as binf
            r = binf.measure(reps=20)
            return [{"model": row["model"], "envs": row["envs"], "bf16_us": round(row["bf16_us"], 1),
                     "fp8_us": round(row["fp8_us"], 1), "fp8_speedup": round(row["fp8_speedup"], 2)} for row in r["rows"]]

        extra("other_workloads", others)
        extra("c5_split_sweep", split_sweep)
        extra("c5_async_rates", async_rates)
        extra("bandwidth_kernels_scaled", scaled_kernels)
        extra("fp8_agents_vs_bf16", fp8_agents)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
