"""Several agent instances feeding one trainer instance on one GPU.

This is the dedicated-trainer layout of the paper's Section 5.1 (serving instances with environment +
agent, a separate trainer instance, experience gathered to the trainer, parameters pushed back), built
from CU-masked streams that share one address space: each agent instance fills its own column slice of
the trainer's experience buffer, so the experience hand-off is an ordering-only `gmi_transfer`; the
parameter hand-off is one device-to-device copy of the bf16 shadow plus orderings.

Two schedules, both deterministic:
  * ``sync``      collect D_k with theta_k on the agent instances, hand over, train theta_{k+1}, publish.
  * ``pipelined`` (lag 1) while the trainer computes theta_{k+1} from D_k the agents already collect
                  D_{k+1} with theta_k (double-buffered experience and weights); log-probs are recorded
                  at collection, so the clipped ratio stays well defined.  This is the one-GPU form of the
                  paper's decoupled serving / training.
No arithmetic of the method happens here.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import (agent_act, agent_value, collect_experience, dtype_code, env_desc, env_step, gae_compute,
               gmi_buffer_bind, gmi_buffer_destroy, gmi_create, gmi_cu_count, gmi_destroy, gmi_env_bind,
               gmi_env_destroy, gmi_model_bind, gmi_model_destroy, gmi_model_refresh_shadow,
               gmi_model_shadow_bytes, gmi_sync, gmi_transfer, model_desc, ppo_hparams, ppo_update, rollout_collect,
               GmiError, ERR_UNSUPPORTED)
from .runner import RolloutBuffers


XCDS = 8   # accelerator complex dies of an MI355X; CU-mask bit i addresses a CU of die i % 8


def cu_masks(n_cu: int, counts: Sequence[int], style: str = "contiguous") -> List[List[int]]:
    """Disjoint CU masks with counts[i] CUs each (sum <= n_cu) as lists of uint32 words.

    On this device mask bit i selects compute unit i // 8 of die i % 8, and the runtime refuses a
    mask that leaves any die without a compute unit (measured: such a stream cannot be created).  An
    instance therefore always spans all eight dies; masks are built from "rows" of 8 consecutive bits
    (the same CU index on every die), so counts must be multiples of 8.
    contiguous: instance i takes the next counts[i] / 8 rows; interleaved: rows are dealt out
    round-robin in proportion to the counts, so every instance's CUs are spread over the CU index range
    of each die."""
    if n_cu % XCDS or sum(counts) > n_cu:
        raise ValueError(f"{sum(counts)} compute units asked for, the device has {n_cu}")
    if not all(c % XCDS == 0 and c > 0 for c in counts):
        raise ValueError("CU counts must be positive multiples of 8 (the same number on every die)")
    if style not in ("contiguous", "interleaved"):
        raise ValueError(f"unknown style {style!r}")
    words = (n_cu + 31) // 32
    n_rows = n_cu // XCDS
    rows = [c // XCDS for c in counts]
    owner = [-1] * n_rows
    if style == "contiguous":
        r = 0
        for i, k in enumerate(rows):
            for _ in range(k):
                owner[r] = i
                r += 1
    else:
        remaining = list(rows)
        total = sum(rows)
        credit = [0.0] * len(rows)
        for r in range(total):
            for i in range(len(rows)):
                credit[i] += rows[i] / total
            best = max((i for i in range(len(rows)) if remaining[i] > 0), key=lambda i: credit[i])
            owner[r] = best
            credit[best] -= 1.0
            remaining[best] -= 1
    masks = [[0] * words for _ in counts]
    for r, i in enumerate(owner):
        if i >= 0:
            for b in range(r * XCDS, (r + 1) * XCDS):
                masks[i][b // 32] |= 1 << (b % 32)
    return masks


class _Agent:
    pass


class InstancePipeline:
    def __init__(self, *, n_agents: int, n_envs: int, obs_dim: int, act_dim: int, hidden: Sequence[int],
                 horizon: int, dtype: str, theta: np.ndarray, a_mat: np.ndarray, b_mat: np.ndarray,
                 state0: Sequence[np.ndarray], noise_std: float, reward_scale: float, done_period: int,
                 done_threshold: int, seed: int, minibatch: int,
                 agent_masks: Optional[Sequence[Optional[Sequence[int]]]] = None,
                 trainer_mask: Optional[Sequence[int]] = None, single_stream: bool = False,
                 fused_rollout: bool = True, host_ordered: bool = False):
        dev = torch.device("cuda:0")
        f = dict(dtype=torch.float32, device=dev)
        self.n_agents, self.N, self.O, self.A, self.T = n_agents, n_envs, obs_dim, act_dim, horizon
        self.Ntot = n_agents * n_envs
        self.seed = seed
        self.single_stream = single_stream
        # host_ordered: the host waits for a stage to finish before it hands the next one to another instance, so no
        # instance's queue ever holds work that waits for an event.  Measured on MI355X: while a CU-masked queue
        # holds such a waiting packet, kernels of every other queue run ~1.6x slower.
        self.host_ordered = host_ordered and not single_stream
        self.fused_rollout = fused_rollout and dtype == "bf16"      # one launch per agent and horizon where it fits
        self.trainer = gmi_create(trainer_mask)
        self.theta = torch.tensor(theta, **f)
        self.adam_m = torch.zeros_like(self.theta)
        self.adam_v = torch.zeros_like(self.theta)
        self.adam_steps = 0
        code = dtype_code(dtype)
        t_desc = model_desc(obs_dim, act_dim, list(hidden), code, minibatch)
        a_desc = model_desc(obs_dim, act_dim, list(hidden), code, n_envs)
        nsh = gmi_model_shadow_bytes(t_desc)
        self.shadow_bytes = nsh
        # shadow[0]: written by the trainer; shadow[1]: the published copy the agents read
        self.shadow = [torch.zeros(max(nsh, 256), dtype=torch.uint8, device=dev) for _ in range(2)] if nsh else [None, None]
        self.theta_pub = torch.tensor(theta, **f)       # fp32 path: the published parameters
        torch.cuda.synchronize()    # torch filled the arrays on its own stream; the library works on the instances' streams
        self.t_model = gmi_model_bind(self.trainer, t_desc, self.theta, self.shadow[0], self.adam_m, self.adam_v)
        gmi_model_refresh_shadow(self.trainer, self.t_model)
        # two experience buffers (the pipelined schedule trains on one while the other fills)
        self.bufs = [RolloutBuffers(horizon, self.Ntot, obs_dim, act_dim, dev) for _ in range(2)]
        self.t_buffer = [gmi_buffer_bind(self.trainer, b.desc(0, self.Ntot)) for b in self.bufs]
        self.last_value = [torch.zeros(self.Ntot, **f) for _ in range(2)]
        self.a_mat = torch.tensor(a_mat, **f)
        self.b_mat = torch.tensor(b_mat, **f)
        self.agents: List[_Agent] = []
        for i in range(n_agents):
            ag = _Agent()
            if single_stream:
                ag.gmi = self.trainer
            else:
                ag.gmi = gmi_create(agent_masks[i] if agent_masks else None)
            pub_params = self.theta_pub if code == 0 else self.theta
            ag.model = gmi_model_bind(ag.gmi, a_desc, pub_params, self.shadow[1], None, None)
            ag.episode_step = torch.zeros(n_envs, dtype=torch.int32, device=dev)
            ag.seed = seed + i
            ag.env = gmi_env_bind(ag.gmi, env_desc(n_envs, obs_dim, act_dim, noise_std, reward_scale, done_period,
                                                   done_threshold, ag.seed), self.a_mat, self.b_mat, ag.episode_step)
            ag.buffer = [gmi_buffer_bind(ag.gmi, b.desc(i * n_envs, n_envs)) for b in self.bufs]
            ag.obs = [torch.tensor(state0[i], **f), torch.zeros(n_envs, obs_dim, **f)]
            ag.cur = 0
            ag.act = torch.zeros(n_envs, act_dim, **f)
            ag.logp = torch.zeros(n_envs, **f)
            ag.value = torch.zeros(n_envs, **f)
            ag.reward = torch.zeros(n_envs, **f)
            ag.done = torch.zeros(n_envs, dtype=torch.uint8, device=dev)
            self.agents.append(ag)
        torch.cuda.synchronize()
        self.publish()
        self.sync_all()

    # ------------------------------------------------------------------ pieces
    def publish(self) -> None:
        """trainer -> agents: copy the freshly written shadow (or fp32 parameters) to the published copy,
        then let every agent instance wait for it."""
        first = self.trainer if self.host_ordered else self.agents[0].gmi
        if self.shadow_bytes:
            gmi_transfer(self.trainer, first, self.shadow[0], self.shadow[1], self.shadow_bytes)
        else:
            gmi_transfer(self.trainer, first, self.theta, self.theta_pub, self.theta.numel() * 4)
        if self.host_ordered:
            gmi_sync(self.trainer)
            return
        for ag in self.agents[1:]:
            gmi_transfer(self.trainer, ag.gmi, None, None, 0)

    def collect(self, iteration: int, slot: int) -> None:
        """Stage (i) on every agent instance: T rounds of act -> step -> store, then the bootstrap value,
        into experience buffer `slot`; ends with the ordering-only hand-off to the trainer."""
        T = self.T
        if self.fused_rollout:
            try:
                for i, ag in enumerate(self.agents):
                    lv = self.last_value[slot].data_ptr() + i * self.N * 4
                    rollout_collect(ag.gmi, ag.model, ag.env, ag.buffer[slot], ag.obs[ag.cur], ag.seed, iteration * T,
                                    0, lv)
                    self._hand_to_trainer(ag)
                self._agents_done()
                return
            except GmiError as e:
                if e.code != ERR_UNSUPPORTED:
                    raise
                self.fused_rollout = False      # refused before anything ran: the per-step calls below
        for t in range(T):
            step = iteration * T + t
            for ag in self.agents:                      # round-robin so the streams fill evenly
                obs, nxt = ag.obs[ag.cur], ag.obs[1 - ag.cur]
                agent_act(ag.gmi, ag.model, obs, self.N, ag.seed, step, 0, ag.act, ag.logp, ag.value)
                env_step(ag.gmi, ag.env, obs, ag.act, step, nxt, ag.reward, ag.done)
                collect_experience(ag.gmi, ag.buffer[slot], t, obs, ag.act, ag.logp, ag.value, ag.reward, ag.done)
                ag.cur = 1 - ag.cur
        for i, ag in enumerate(self.agents):
            lv = self.last_value[slot].data_ptr() + i * self.N * 4
            agent_value(ag.gmi, ag.model, ag.obs[ag.cur], self.N, lv)
            self._hand_to_trainer(ag)
        self._agents_done()

    def _hand_to_trainer(self, ag) -> None:
        if not self.host_ordered:
            gmi_transfer(ag.gmi, self.trainer, None, None, 0)       # ordering only: the trainer's stream waits

    def _agents_done(self) -> None:
        if self.host_ordered:
            for ag in self.agents:
                gmi_sync(ag.gmi)

    def train(self, iteration: int, slot: int, *, gamma: float, lam: float, epochs: int, minibatch: int,
              stats=None, **hp) -> None:
        """Stage (ii) on the trainer instance: GAE over the concatenated buffer, then the update."""
        gae_compute(self.trainer, self.t_buffer[slot], self.last_value[slot], gamma, lam, True)
        h = ppo_hparams(epochs=epochs, minibatch=minibatch, seed=self.seed, iteration=iteration,
                        adam_step0=self.adam_steps, **hp)
        ppo_update(self.trainer, self.t_model, self.t_buffer[slot], h, stats)
        self.adam_steps += epochs * (self.T * self.Ntot // minibatch)

    # ------------------------------------------------------------------ schedules
    def iteration_sync(self, k: int, **train_args) -> None:
        self.collect(k, 0)
        self.train(k, 0, **train_args)
        self.publish()

    def prologue_pipelined(self, **train_args) -> None:
        """Fills buffer 0 with D_0 collected under theta_0."""
        self.collect(0, 0)

    def iteration_pipelined(self, k: int, **train_args) -> None:
        """Trainer: theta_{k+1} from D_k (slot k%2).  Agents, concurrently: D_{k+1} with theta_k into the other slot."""
        self.train(k, k % 2, **train_args)
        self.collect(k + 1, (k + 1) % 2)
        self.publish()      # queued on the trainer after its update and after the agents' hand-off

    def sync_all(self) -> None:
        for ag in self.agents:
            gmi_sync(ag.gmi)
        gmi_sync(self.trainer)

    def cu_counts(self):
        return [gmi_cu_count(ag.gmi) for ag in self.agents], gmi_cu_count(self.trainer)

    def close(self) -> None:
        self.sync_all()
        for ag in self.agents:
            for b in ag.buffer:
                gmi_buffer_destroy(b)
            gmi_env_destroy(ag.env)
            gmi_model_destroy(ag.model)
            if not self.single_stream:
                gmi_destroy(ag.gmi)
        for b in self.t_buffer:
            gmi_buffer_destroy(b)
        gmi_model_destroy(self.t_model)
        gmi_destroy(self.trainer)
