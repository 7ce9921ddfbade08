"""Host-side orchestration of one PPO iteration through the C ABI (allocation with PyTorch, calls in
the order of the paper's synchronized-training stages, Section 5.1: experience collection, then
model training).  No arithmetic of the method happens here."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np
import torch

from . import (DTYPE_BF16, DTYPE_F32, agent_act, agent_value, buffer_desc, collect_experience, env_desc,
               env_step, gae_compute, gmi_buffer_bind, gmi_buffer_destroy, gmi_create, gmi_destroy,
               gmi_env_bind, gmi_env_destroy, gmi_model_bind, gmi_model_destroy, gmi_model_refresh_shadow,
               gmi_model_shadow_bytes, gmi_stream, gmi_sync, gmi_wait_stream, model_desc, ppo_hparams, ppo_update,
               rollout_collect, GmiError, ERR_UNSUPPORTED, ppo_update_group)


def dtype_code(name: str) -> int:
    return {"f32": DTYPE_F32, "bf16": DTYPE_BF16}[name]


class RolloutBuffers:
    """Time-major experience arrays [T, ld, ...] on the device."""

    def __init__(self, T: int, ld: int, O: int, A: int, device):
        f = dict(dtype=torch.float32, device=device)
        self.obs = torch.zeros(T, ld, O, **f)
        self.act = torch.zeros(T, ld, A, **f)
        self.logp = torch.zeros(T, ld, **f)
        self.val = torch.zeros(T, ld, **f)
        self.rew = torch.zeros(T, ld, **f)
        self.done = torch.zeros(T, ld, dtype=torch.uint8, device=device)
        self.adv = torch.zeros(T, ld, **f)
        self.ret = torch.zeros(T, ld, **f)
        self.T, self.ld, self.O, self.A = T, ld, O, A

    def desc(self, col0: int, n_envs: int):
        """Descriptor of the column slice [col0, col0 + n_envs)."""
        def off(t, width=1):
            return t.data_ptr() + col0 * width * t.element_size()
        return buffer_desc(self.T, n_envs, self.ld, self.O, self.A, off(self.obs, self.O), off(self.act, self.A),
                           off(self.logp), off(self.val), off(self.rew), off(self.done), off(self.adv),
                           off(self.ret))

    def to_numpy(self) -> dict:
        return {k: getattr(self, k).cpu().numpy() for k in
                ("obs", "act", "logp", "val", "rew", "done", "adv", "ret")}


class PPOSession:
    """One holistic instance (environment + agent + trainer on the same stream)."""

    def __init__(self, *, n_envs: int, obs_dim: int, act_dim: int, hidden: Sequence[int], horizon: int,
                 dtype: str, theta: np.ndarray, a_mat: np.ndarray, b_mat: np.ndarray, state0: np.ndarray,
                 noise_std: float, reward_scale: float, done_period: int, done_threshold: int, seed: int,
                 minibatch: int, cu_mask: Optional[Sequence[int]] = None, gmi: Optional[int] = None,
                 fused_rollout: bool = True, env_offset: int = 0, replica_of: Optional["PPOSession"] = None):
        """env_offset: index of this session's env 0 in the Philox counters (distinct per instance when several
        instances simulate disjoint env shards).  replica_of: bind the model to that session's parameter,
        Adam and shadow arrays (a replica trained in lockstep through ``update_group``) instead of own ones."""
        dev = torch.device("cuda:0")
        self.dev = dev
        self.N, self.O, self.A, self.T = n_envs, obs_dim, act_dim, horizon
        self.seed = seed
        self.own_gmi = gmi is None
        self.gmi = gmi_create(cu_mask) if gmi is None else gmi
        self.stream = torch.cuda.ExternalStream(gmi_stream(self.gmi), device=dev)
        f = dict(dtype=torch.float32, device=dev)
        self.env_offset = env_offset
        if replica_of is None:
            self.theta = torch.tensor(theta, **f)
            self.adam_m = torch.zeros_like(self.theta)
            self.adam_v = torch.zeros_like(self.theta)
        else:
            self.theta, self.adam_m, self.adam_v = replica_of.theta, replica_of.adam_m, replica_of.adam_v
        self.adam_steps = 0
        rows = max(n_envs, minibatch)
        self.mdesc = model_desc(obs_dim, act_dim, list(hidden), dtype_code(dtype), rows)
        nshadow = gmi_model_shadow_bytes(self.mdesc)
        if replica_of is None:
            self.shadow = torch.zeros(max(nshadow, 256), dtype=torch.uint8, device=dev) if nshadow else None
        else:
            self.shadow = replica_of.shadow
        # torch filled the arrays above on its own stream; the library works on the instance's stream
        gmi_wait_stream(self.gmi)
        self.model = gmi_model_bind(self.gmi, self.mdesc, self.theta, self.shadow, self.adam_m, self.adam_v)
        if replica_of is None:
            gmi_model_refresh_shadow(self.gmi, self.model)
        self.a_mat = torch.tensor(a_mat, **f)
        self.b_mat = torch.tensor(b_mat, **f)
        self.episode_step = torch.zeros(n_envs, dtype=torch.int32, device=dev)
        self.edesc = env_desc(n_envs, obs_dim, act_dim, noise_std, reward_scale, done_period, done_threshold, seed,
                              env_offset)
        self.env = gmi_env_bind(self.gmi, self.edesc, self.a_mat, self.b_mat, self.episode_step)
        self.buf = RolloutBuffers(horizon, n_envs, obs_dim, act_dim, dev)
        self.bdesc = self.buf.desc(0, n_envs)
        self.buffer = gmi_buffer_bind(self.gmi, self.bdesc)
        self.obs = [torch.tensor(state0, **f), torch.zeros(n_envs, obs_dim, **f)]
        self.cur = 0
        self.act = torch.zeros(n_envs, act_dim, **f)
        self.logp = torch.zeros(n_envs, **f)
        self.value = torch.zeros(n_envs, **f)
        self.reward = torch.zeros(n_envs, **f)
        self.done = torch.zeros(n_envs, dtype=torch.uint8, device=dev)
        self.last_value = torch.zeros(n_envs, **f)
        self.fused_rollout = fused_rollout and dtype == "bf16"
        gmi_wait_stream(self.gmi)      # the fills above (torch's stream) come before anything queued on the instance

    # -- stage (i): experience collection
    def rollout(self, iteration: int) -> None:
        g = self.gmi
        if self.fused_rollout:
            try:
                rollout_collect(g, self.model, self.env, self.buffer, self.obs[self.cur], self.seed,
                                iteration * self.T, self.env_offset, self.last_value)
                return
            except GmiError as e:
                if e.code != ERR_UNSUPPORTED:
                    raise
                self.fused_rollout = False      # this model does not fit the one-launch kernel
        for t in range(self.T):
            step = iteration * self.T + t
            obs, nxt = self.obs[self.cur], self.obs[1 - self.cur]
            agent_act(g, self.model, obs, self.N, self.seed, step, self.env_offset, self.act, self.logp, self.value)
            env_step(g, self.env, obs, self.act, step, nxt, self.reward, self.done)
            collect_experience(g, self.buffer, t, obs, self.act, self.logp, self.value, self.reward, self.done)
            self.cur = 1 - self.cur
        agent_value(g, self.model, self.obs[self.cur], self.N, self.last_value)

    def gae(self, gamma: float, lam: float, normalize: bool = True) -> None:
        gae_compute(self.gmi, self.buffer, self.last_value, gamma, lam, normalize)

    # -- stage (ii): model training
    def update(self, iteration: int, *, epochs: int, minibatch: int, stats=None, **hp) -> None:
        h = ppo_hparams(epochs=epochs, minibatch=minibatch, seed=self.seed, iteration=iteration,
                        adam_step0=self.adam_steps, **hp)
        ppo_update(self.gmi, self.model, self.buffer, h, stats)
        self.adam_steps += epochs * (self.T * self.N // minibatch)

    @staticmethod
    def update_group(sessions: Sequence["PPOSession"], iteration: int, *, epochs: int, minibatch: int, stats=None,
                     **hp) -> None:
        """Stage (ii) for replicas trained in lockstep (sessions[1:] built with replica_of=sessions[0]):
        one synchronized update over all sessions' buffers, gradients averaged in memory."""
        lead = sessions[0]
        h = ppo_hparams(epochs=epochs, minibatch=minibatch, seed=lead.seed, iteration=iteration,
                        adam_step0=lead.adam_steps, **hp)
        ppo_update_group([s.gmi for s in sessions], [s.model for s in sessions], [s.buffer for s in sessions], h, stats)
        steps = epochs * (lead.T * lead.N // minibatch)
        for s in sessions:
            s.adam_steps += steps

    def sync(self) -> None:
        gmi_sync(self.gmi)

    def state(self) -> torch.Tensor:
        return self.obs[self.cur]

    def close(self) -> None:
        gmi_sync(self.gmi)
        gmi_buffer_destroy(self.buffer)
        gmi_env_destroy(self.env)
        gmi_model_destroy(self.model)
        if self.own_gmi:
            gmi_destroy(self.gmi)
