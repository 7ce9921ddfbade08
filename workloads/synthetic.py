"""Synthetic PPO workloads: sizes of the benchmark configurations and seeded input generators.

The paper evaluates on physics-simulator tasks (Table 6: Ant 60:256:128:64:8, Humanoid,
ShadowHand, ...).  Those simulators are not available, so the workloads here keep the tasks'
*shapes* (observation/action sizes, MLP widths, number of environments, horizon) and replace the
physics by a seeded linear-Gaussian environment.  Everything here is plain numpy random draws
(PCG64 via ``numpy.random.default_rng``); none of it is part of the method under test.

Flat parameter vector layout (the same for every consumer, stated here once):

    policy net : for each layer l = 0..L   (L hidden layers + linear head)
                     W_l  [out_l, in_l] row-major, then b_l [out_l]
    value net  : same, head has out = 1
    log_std    : [A]

with in_0 = O, out_l = hidden[l] for l < L, head out = A (policy) or 1 (value).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Tuple

import numpy as np


@dataclass(frozen=True)
class PPOConfig:
    name: str
    n_envs: int              # environments per agent instance
    obs_dim: int
    act_dim: int
    hidden: Tuple[int, ...]
    horizon: int
    epochs: int
    minibatch: int
    dtype: str               # "f32" or "bf16" (bf16 weights/activations, fp32 master + accumulate)
    done_period: int = 0     # >0: done when (episode_step + 1) % period == 0
    done_prob_inv: int = 0   # >0: done with probability 1/done_prob_inv per step
    reward_scale: float = 1.0
    noise_std: float = 0.01
    gamma: float = 0.99
    lam: float = 0.95
    clip: float = 0.2
    c_v: float = 0.5
    c_e: float = 0.0
    lr: float = 3e-4
    beta1: float = 0.9
    beta2: float = 0.999
    adam_eps: float = 1e-8
    n_agents: int = 1        # agent instances feeding one trainer
    seed: int = 0

    @property
    def batch(self) -> int:
        return self.n_envs * self.n_agents * self.horizon


CONFIGS: Dict[str, PPOConfig] = {
    "C1": PPOConfig("C1", 64, 8, 2, (32, 32), 16, 1, 256, "f32", done_period=16),
    "C2": PPOConfig("C2", 4096, 60, 8, (256, 128, 64), 16, 4, 32768, "bf16", done_prob_inv=1000),
    "C3": PPOConfig("C3", 4096, 108, 21, (400, 200, 100), 32, 5, 32768, "bf16", done_prob_inv=1000),
    "C4": PPOConfig("C4", 16384, 211, 20, (512, 512, 256, 128), 16, 5, 32768, "bf16",
                    done_prob_inv=1000, reward_scale=0.01),
    "C5": PPOConfig("C5", 4096, 108, 21, (400, 200, 100), 32, 5, 65536, "bf16",
                    done_prob_inv=1000, n_agents=4),
    # The policy models of the paper's Table 6 under their own layer orders (its Ant model is C2's), on the same
    # synthetic env family: 4096 envs, horizon 16, 4 epochs, minibatch 32768 as for C2.
    "AY": PPOConfig("AY", 4096, 48, 12, (256, 128, 64), 16, 4, 32768, "bf16", done_prob_inv=1000),
    "BB": PPOConfig("BB", 4096, 24, 3, (256, 128, 64), 16, 4, 32768, "bf16", done_prob_inv=1000),
    "FC": PPOConfig("FC", 4096, 23, 9, (256, 128, 64), 16, 4, 32768, "bf16", done_prob_inv=1000),
    "HM": PPOConfig("HM", 4096, 108, 21, (200, 400, 100), 16, 4, 32768, "bf16", done_prob_inv=1000),
    "SH": PPOConfig("SH", 8192, 211, 20, (512, 512, 512, 256), 16, 4, 32768, "bf16", done_prob_inv=1000,
                    reward_scale=0.01),
}


def get_config(name: str, **overrides) -> PPOConfig:
    cfg = CONFIGS[name]
    return replace(cfg, **overrides) if overrides else cfg


def layer_dims(obs_dim: int, out_dim: int, hidden) -> List[Tuple[int, int]]:
    """(in, out) of every linear layer of one MLP, head included."""
    dims = []
    prev = obs_dim
    for h in hidden:
        dims.append((prev, h))
        prev = h
    dims.append((prev, out_dim))
    return dims


def param_count(obs_dim: int, act_dim: int, hidden) -> int:
    n = 0
    for out_dim in (act_dim, 1):
        for i, o in layer_dims(obs_dim, out_dim, hidden):
            n += i * o + o
    return n + act_dim


def make_model_params(obs_dim: int, act_dim: int, hidden, seed: int,
                      policy_head_scale: float = 0.01, log_std_init: float = 0.0) -> np.ndarray:
    """Flat fp32 parameter vector: W ~ N(0, 1/fan_in), small random biases, policy head scaled."""
    rng = np.random.default_rng([seed, 101])
    parts = []
    for out_dim, head_scale in ((act_dim, policy_head_scale), (1, 1.0)):
        dims = layer_dims(obs_dim, out_dim, hidden)
        for li, (i, o) in enumerate(dims):
            w = rng.standard_normal((o, i)) / np.sqrt(i)
            b = 0.01 * rng.standard_normal(o)
            if li == len(dims) - 1:
                w = w * head_scale
                b = b * head_scale
            parts.append(w.reshape(-1))
            parts.append(b)
    parts.append(np.full(act_dim, log_std_init))
    return np.concatenate(parts).astype(np.float32)


def make_env_matrices(obs_dim: int, act_dim: int, seed: int):
    """A = 0.95 I + 0.01 G  [O,O];  B = 0.1 G'  [O,A]   (G, G' standard normal)."""
    rng = np.random.default_rng([seed, 202])
    a_mat = 0.95 * np.eye(obs_dim) + 0.01 * rng.standard_normal((obs_dim, obs_dim))
    b_mat = 0.1 * rng.standard_normal((obs_dim, act_dim))
    return a_mat.astype(np.float32), b_mat.astype(np.float32)


def make_initial_state(n_envs: int, obs_dim: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng([seed, 303])
    return rng.standard_normal((n_envs, obs_dim)).astype(np.float32)


def make_rollout_batch(T: int, N: int, obs_dim: int, act_dim: int, seed: int,
                       done_prob: float = 0.05) -> dict:
    """A random, already-filled rollout buffer (time-major), for tests of GAE and the update that
    do not want to run a rollout first."""
    rng = np.random.default_rng([seed, 404])
    return {
        "obs": rng.standard_normal((T, N, obs_dim)).astype(np.float32),
        "act": rng.standard_normal((T, N, act_dim)).astype(np.float32),
        "logp": (-0.5 * act_dim * np.log(2 * np.pi)
                 - 0.5 * rng.chisquare(act_dim, (T, N))).astype(np.float32),
        "val": rng.standard_normal((T, N)).astype(np.float32),
        "rew": rng.standard_normal((T, N)).astype(np.float32),
        "done": (rng.random((T, N)) < done_prob).astype(np.uint8),
        "last_val": rng.standard_normal(N).astype(np.float32),
    }
