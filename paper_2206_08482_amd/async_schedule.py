"""Asynchronous serving and training on one GPU (Section 5.2 of the paper: agents and trainers decoupled by the
experience channels, each running at its own rate; throughput reported as PPS, predictions per second served by
the agents, and TTOP, samples per second consumed by the trainer).

Every agent instance and the trainer instance is driven by a host thread of its own.  An agent loops: take the
newest published parameters into its own copy, collect one round into its own buffer, push the slab into the
channels.  The trainer loops: wait until `slabs_per_update` slabs are waiting, pop them (oldest first, stacked in
arrival order), GAE, update, publish.  Nothing fixes how many rounds the agents collect per update: the rates
follow from how fast each side runs.  When the ring is full an agent either waits (`on_full="block"`: in the long
run PPS = TTOP) or discards the oldest waiting slab (`on_full="drop_oldest"`: the agents never wait and the trainer
always finds the freshest experience; PPS and TTOP then differ by the share of slabs discarded).

The run is not deterministic, but it is replayable: `trace` records, in the order the ring saw them, every push
(agent, that agent's round, the parameter version the round was collected with), every discard, and every update
(the slabs it consumed).  Replaying the trace step by step reproduces the parameters (tests do so with the oracle).
No arithmetic of the method happens here."""
from __future__ import annotations

import threading
import time
from collections import deque
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import (CHANNELS_MULTI, agent_act, agent_act_fp8, agent_value, collect_experience, dtype_code,
               env_desc, env_step, gae_compute, gmi_buffer_bind, gmi_buffer_destroy, gmi_channels_create,
               gmi_channels_destroy, gmi_channels_drop, gmi_channels_pop, gmi_channels_push, gmi_create, gmi_destroy,
               gmi_env_bind, gmi_env_destroy, gmi_fp8_bind, gmi_fp8_destroy, gmi_fp8_refresh, gmi_model_bind, gmi_model_destroy, gmi_model_refresh_shadow,
               gmi_model_shadow_bytes, gmi_sync, gmi_transfer, model_desc, ppo_hparams, ppo_update, rollout_collect)
from .runner import RolloutBuffers


class _Agent:
    pass


class AsyncPipeline:
    def __init__(self, *, n_agents: int, n_envs: int, obs_dim: int, act_dim: int, hidden: Sequence[int],
                 horizon: int, dtype: str, theta: np.ndarray, a_mat: np.ndarray, b_mat: np.ndarray,
                 state0: Sequence[np.ndarray], noise_std: float, reward_scale: float, done_period: int,
                 done_threshold: int, seed: int, minibatch: int, slabs_per_update: Optional[int] = None,
                 capacity: Optional[int] = None, on_full: str = "block", mode: int = CHANNELS_MULTI,
                 agent_masks: Optional[Sequence[Optional[Sequence[int]]]] = None,
                 trainer_mask: Optional[Sequence[int]] = None, reset_each_round: bool = False,
                 agent_precision: str = "model"):
        """reset_each_round: every round starts from the agent's initial state (for timing runs: the synthetic
        dynamics are not stable over hundreds of steps).  agent_precision: "model" = the agents serve in the
        trainer's arithmetic; "fp8" = they serve through agent_act_fp8 (E4M3 weights re-quantised from every
        parameter version they take; the trainer is unchanged)."""
        if agent_precision not in ("model", "fp8"):
            raise ValueError(f"unknown agent_precision {agent_precision!r}")
        if on_full not in ("block", "drop_oldest"):
            raise ValueError(f"unknown on_full {on_full!r}")
        dev = torch.device("cuda:0")
        f = dict(dtype=torch.float32, device=dev)
        self.n_agents, self.N, self.O, self.A, self.T = n_agents, n_envs, obs_dim, act_dim, horizon
        self.S = n_agents if slabs_per_update is None else slabs_per_update
        if not 1 <= self.S <= 8:
            raise ValueError("1 <= slabs_per_update <= 8")
        self.Ntot = self.S * n_envs
        self.capacity = max(2 * self.S, n_agents + self.S) if capacity is None else capacity
        if self.capacity < self.S:
            raise ValueError("the ring must hold at least one update's slabs")
        self.on_full = on_full
        self.seed = seed
        code = dtype_code(dtype)
        self.f32 = code == 0
        self.fp8 = agent_precision == "fp8"
        self.fused_rollout = not self.f32 and not self.fp8
        self.trainer = gmi_create(trainer_mask)
        self.theta = torch.tensor(theta, **f)
        self.adam_m = torch.zeros_like(self.theta)
        self.adam_v = torch.zeros_like(self.theta)
        self.adam_steps = 0
        t_desc = model_desc(obs_dim, act_dim, list(hidden), code, minibatch)
        a_desc = model_desc(obs_dim, act_dim, list(hidden), code, n_envs)
        nsh = gmi_model_shadow_bytes(t_desc)
        pub_shadow = bool(nsh) and not self.fp8     # fp8 agents quantise from the fp32 parameters themselves
        self.pub_bytes = nsh if pub_shadow else self.theta.numel() * 4

        def weights():      # one copy of what an agent reads: the bf16 shadow, or the fp32 parameters
            if pub_shadow:
                return torch.zeros(max(nsh, 256), dtype=torch.uint8, device=dev)
            return torch.tensor(theta, **f)

        self.t_shadow = torch.zeros(max(nsh, 256), dtype=torch.uint8, device=dev) if nsh else None
        self.pub_shadow = pub_shadow
        self.pub = [weights(), weights()]       # version v is published in slot v % 2
        self.channels = gmi_channels_create(horizon, n_envs, obs_dim, act_dim, self.capacity, mode)
        self.batch = RolloutBuffers(horizon, self.Ntot, obs_dim, act_dim, dev)
        self.last_value = torch.zeros(self.Ntot, **f)
        self.a_mat = torch.tensor(a_mat, **f)
        self.b_mat = torch.tensor(b_mat, **f)
        torch.cuda.synchronize()    # torch filled the arrays on its own stream; the library works on the instances' streams
        self.t_model = gmi_model_bind(self.trainer, t_desc, self.theta, self.t_shadow, self.adam_m, self.adam_v)
        self.t_buffer = gmi_buffer_bind(self.trainer, self.batch.desc(0, self.Ntot))
        if nsh:
            gmi_model_refresh_shadow(self.trainer, self.t_model)
        self.agents: List[_Agent] = []
        for i in range(n_agents):
            ag = _Agent()
            ag.index = i
            ag.gmi = gmi_create(agent_masks[i] if agent_masks else None)
            ag.weights = weights()
            torch.cuda.synchronize()
            ag.model = ag.fp8 = None
            if self.fp8:
                ag.fp8 = gmi_fp8_bind(ag.gmi, a_desc)
            elif nsh:
                ag.model = gmi_model_bind(ag.gmi, a_desc, self.theta, ag.weights, None, None)
            else:
                ag.model = gmi_model_bind(ag.gmi, a_desc, ag.weights, None, None, None)
            ag.episode_step = torch.zeros(n_envs, dtype=torch.int32, device=dev)
            ag.seed = seed + i
            ag.env = gmi_env_bind(ag.gmi, env_desc(n_envs, obs_dim, act_dim, noise_std, reward_scale, done_period,
                                                   done_threshold, ag.seed), self.a_mat, self.b_mat, ag.episode_step)
            ag.rb = RolloutBuffers(horizon, n_envs, obs_dim, act_dim, dev)
            ag.obs = [torch.tensor(state0[i], **f), torch.zeros(n_envs, obs_dim, **f)]
            ag.state0 = torch.tensor(state0[i], **f) if reset_each_round else None
            ag.cur = 0
            ag.act = torch.zeros(n_envs, act_dim, **f)
            ag.logp = torch.zeros(n_envs, **f)
            ag.value = torch.zeros(n_envs, **f)
            ag.reward = torch.zeros(n_envs, **f)
            ag.done = torch.zeros(n_envs, dtype=torch.uint8, device=dev)
            ag.last = torch.zeros(n_envs, **f)
            torch.cuda.synchronize()
            ag.buffer = gmi_buffer_bind(ag.gmi, ag.rb.desc(0, n_envs))
            ag.rounds = 0
            self.agents.append(ag)
        # host state shared by the threads
        self.ring = threading.Condition()       # guards the channel calls, `waiting` and `trace`
        self.waiting = deque()                  # (agent, round, version) of the slabs in the ring, oldest first
        self.params = threading.Condition()     # guards `version` and `readers`
        self.version = 0
        self.readers = [0, 0]
        self.stop = False
        self.updates_total = 0                  # updates made so far = the newest parameter version
        self.trace: List[tuple] = []
        self.errors: List[BaseException] = []
        self._publish(0)
        gmi_sync(self.trainer)

    # ------------------------------------------------------------------ parameters
    def _publish(self, version: int) -> None:
        """The trainer's current weights into slot version % 2 (on the trainer's stream)."""
        slot = version % 2
        with self.params:       # agents that chose this slot two versions ago have finished copying from it
            while self.readers[slot]:
                self.params.wait()
        src = self.t_shadow if self.pub_shadow else self.theta
        gmi_transfer(self.trainer, self.trainer, src, self.pub[slot], self.pub_bytes)

    def _take_newest(self, ag) -> int:
        with self.params:
            v = self.version
            self.readers[v % 2] += 1
        try:
            gmi_transfer(ag.gmi, ag.gmi, self.pub[v % 2], ag.weights, self.pub_bytes)
            if ag.fp8 is not None:
                gmi_fp8_refresh(ag.gmi, ag.fp8, ag.weights)
            gmi_sync(ag.gmi)
        finally:
            with self.params:
                self.readers[v % 2] -= 1
                self.params.notify_all()
        return v

    # ------------------------------------------------------------------ the two loops
    def _collect(self, ag, r: int) -> None:
        T = self.T
        if ag.state0 is not None:
            gmi_transfer(ag.gmi, ag.gmi, ag.state0, ag.obs[ag.cur], ag.state0.numel() * 4)
        if self.fused_rollout:
            rollout_collect(ag.gmi, ag.model, ag.env, ag.buffer, ag.obs[ag.cur], ag.seed, r * T, 0, ag.last)
            return
        for t in range(T):
            step = r * T + t
            obs, nxt = ag.obs[ag.cur], ag.obs[1 - ag.cur]
            if ag.fp8 is not None:
                agent_act_fp8(ag.gmi, ag.fp8, obs, self.N, ag.seed, step, 0, ag.act, ag.logp, ag.value)
            else:
                agent_act(ag.gmi, ag.model, obs, self.N, ag.seed, step, 0, ag.act, ag.logp, ag.value)
            env_step(ag.gmi, ag.env, obs, ag.act, step, nxt, ag.reward, ag.done)
            collect_experience(ag.gmi, ag.buffer, t, obs, ag.act, ag.logp, ag.value, ag.reward, ag.done)
            ag.cur = 1 - ag.cur
        if ag.fp8 is not None:      # the bootstrap value: the value output of one more decision (its action is unused)
            agent_act_fp8(ag.gmi, ag.fp8, ag.obs[ag.cur], self.N, ag.seed, (r + 1) * T, 0, ag.act, ag.logp, ag.last)
        else:
            agent_value(ag.gmi, ag.model, ag.obs[ag.cur], self.N, ag.last)

    def _agent_loop(self, ag, max_rounds: Optional[int]) -> None:
        try:
            while not self.stop and (max_rounds is None or ag.rounds < max_rounds):
                r = ag.rounds
                v = self._take_newest(ag)
                self._collect(ag, r)
                gmi_sync(ag.gmi)        # the round is served: it counts towards PPS from here on
                ag.rounds = r + 1
                with self.ring:
                    while len(self.waiting) >= self.capacity and not self.stop:
                        if self.on_full == "drop_oldest":
                            gmi_channels_drop(self.channels, 1)
                            self.trace.append(("drop", self.waiting.popleft()))
                        else:
                            self.ring.wait(0.05)
                    if self.stop and len(self.waiting) >= self.capacity:
                        return
                    gmi_channels_push(ag.gmi, self.channels, ag.buffer, ag.last)
                    self.waiting.append((ag.index, r, v))
                    self.trace.append(("push", (ag.index, r, v)))
                    self.ring.notify_all()
                gmi_sync(ag.gmi)        # the slab is in the ring; the agent's buffer is free for the next round
        except BaseException as e:      # noqa: BLE001 -- reported by run()
            self.errors.append(e)
            self.stop = True
            with self.ring:
                self.ring.notify_all()

    def _trainer_loop(self, updates: int, train_args: dict) -> None:
        try:
            gamma, lam = train_args["gamma"], train_args["lam"]
            hp = {k: v for k, v in train_args.items() if k not in ("gamma", "lam")}
            for k in range(self.updates_total, self.updates_total + updates):
                with self.ring:
                    while len(self.waiting) < self.S and not self.stop:
                        self.ring.wait(0.05)
                    if len(self.waiting) < self.S:
                        return
                    gmi_channels_pop(self.trainer, self.channels, self.S, 0, self.N, self.t_buffer, 0, self.last_value)
                    took = [self.waiting.popleft() for _ in range(self.S)]
                    self.trace.append(("update", k, tuple(took)))
                    self.ring.notify_all()
                gae_compute(self.trainer, self.t_buffer, self.last_value, gamma, lam, True)
                h = ppo_hparams(seed=self.seed, iteration=k, adam_step0=self.adam_steps, **hp)
                ppo_update(self.trainer, self.t_model, self.t_buffer, h, None)
                self.adam_steps += hp["epochs"] * (self.T * self.Ntot // hp["minibatch"])
                self._publish(k + 1)
                gmi_sync(self.trainer)
                with self.params:
                    self.version = k + 1
                self.updates_total = k + 1
                self.updates_done += 1
        except BaseException as e:      # noqa: BLE001
            self.errors.append(e)
        finally:
            self.stop = True
            with self.ring:
                self.ring.notify_all()

    def run(self, updates: int, *, max_rounds: Optional[int] = None, **train_args) -> dict:
        """Runs until the trainer has made `updates` updates (or, with max_rounds, until no agent may collect any
        more and the ring cannot feed another update).  Returns the rates over the wall time of the run."""
        self.stop = False
        self.updates_done = 0
        threads = [threading.Thread(target=self._agent_loop, args=(ag, max_rounds)) for ag in self.agents]
        trainer = threading.Thread(target=self._trainer_loop, args=(updates, train_args))
        rounds0 = sum(ag.rounds for ag in self.agents)
        trace0 = len(self.trace)
        t0 = time.perf_counter()
        for th in threads + [trainer]:
            th.start()
        if max_rounds is not None:      # the agents end by themselves; then nothing can feed the trainer any more
            for th in threads:
                th.join()
            with self.ring:
                while len(self.waiting) >= self.S and not self.stop:
                    self.ring.wait(0.05)
            self.stop = True
            with self.ring:
                self.ring.notify_all()
        trainer.join()
        dt_train = time.perf_counter() - t0
        for th in threads:
            th.join()
        dt = time.perf_counter() - t0
        self.sync_all()
        if self.errors:
            raise self.errors[0]
        rounds = sum(ag.rounds for ag in self.agents) - rounds0
        per_slab = self.T * self.N
        dropped = sum(1 for e in self.trace[trace0:] if e[0] == "drop")
        return {"seconds": dt, "updates": self.updates_done, "rounds_collected": rounds, "slabs_discarded": dropped,
                "pps_env_steps_per_s": rounds * per_slab / dt,
                "ttop_samples_per_s": self.updates_done * self.S * per_slab / dt_train}

    def sync_all(self) -> None:
        for ag in self.agents:
            gmi_sync(ag.gmi)
        gmi_sync(self.trainer)

    def close(self) -> None:
        self.sync_all()
        for ag in self.agents:
            gmi_buffer_destroy(ag.buffer)
            gmi_env_destroy(ag.env)
            if ag.model is not None:
                gmi_model_destroy(ag.model)
            if ag.fp8 is not None:
                gmi_fp8_destroy(ag.fp8)
            gmi_destroy(ag.gmi)
        gmi_buffer_destroy(self.t_buffer)
        gmi_channels_destroy(self.channels)
        gmi_model_destroy(self.t_model)
        gmi_destroy(self.trainer)
