"""Agent instances feeding a trainer instance through experience channels (Section 4.2 of the paper) instead of
writing straight into the trainer's batch: every agent instance collects into a buffer of its own and pushes it
as a slab; the trainer pops the slabs of a round, stacked side by side, into its batch.  Same two schedules as
`instances.InstancePipeline` (whose direct hand-off moves no bytes and is the comparison point), plus the
bounded-staleness schedule that the queue makes possible: the agents run `lag` rounds ahead of the trainer, round
k + lag being collected with the parameters after k updates while the trainer works on round k.  This is the
one-GPU, replayable form of the paper's asynchronous serving / training (Section 5.2: agents and trainers
decoupled by the channels); lag = 1 is the pipelined schedule.  No arithmetic of the method happens here."""
from __future__ import annotations

from typing import Optional, Sequence

import torch

from . import (CHANNELS_MULTI, gae_compute, gmi_buffer_bind, gmi_buffer_destroy, gmi_channels_create,
               gmi_channels_destroy, gmi_channels_pop, gmi_channels_push, ppo_hparams, ppo_update,
               rollout_collect)
from .instances import InstancePipeline
from .runner import RolloutBuffers


class ChannelPipeline(InstancePipeline):
    def __init__(self, *, mode: int = CHANNELS_MULTI, capacity: Optional[int] = None, **kw):
        super().__init__(**kw)
        if not self.fused_rollout:
            raise ValueError("ChannelPipeline collects with rollout_collect (bf16 models)")
        dev = torch.device("cuda:0")
        cap = 2 * self.n_agents if capacity is None else capacity
        self.capacity = cap
        self.channels = gmi_channels_create(self.T, self.N, self.O, self.A, cap, mode)
        self.own = []                         # every agent's own experience buffer and bootstrap values
        for ag in self.agents:
            rb = RolloutBuffers(self.T, self.N, self.O, self.A, dev)
            lv = torch.zeros(self.N, dtype=torch.float32, device=dev)
            torch.cuda.synchronize()
            self.own.append((rb, gmi_buffer_bind(ag.gmi, rb.desc(0, self.N)), lv))

    def collect(self, iteration: int, slot: int) -> None:
        """Stage (i) on every agent instance into its own buffer, then the push of the slab."""
        for ag, (rb, handle, lv) in zip(self.agents, self.own):
            rollout_collect(ag.gmi, ag.model, ag.env, handle, ag.obs[ag.cur], ag.seed, iteration * self.T, 0, lv)
            gmi_channels_push(ag.gmi, self.channels, handle, lv)
            # the published weights these agents read may only be replaced after this round's collection
            self._hand_to_trainer(ag)
        self._agents_done()

    def train(self, iteration: int, slot: int, *, gamma: float, lam: float, epochs: int, minibatch: int,
              stats=None, **hp) -> None:
        """The trainer's batcher stacks the round's slabs into its batch; then GAE and the update."""
        gmi_channels_pop(self.trainer, self.channels, self.n_agents, 0, self.N, self.t_buffer[slot], 0,
                         self.last_value[slot])
        gae_compute(self.trainer, self.t_buffer[slot], self.last_value[slot], gamma, lam, True)
        h = ppo_hparams(epochs=epochs, minibatch=minibatch, seed=self.seed, iteration=iteration,
                        adam_step0=self.adam_steps, **hp)
        ppo_update(self.trainer, self.t_model, self.t_buffer[slot], h, stats)
        self.adam_steps += epochs * (self.T * self.Ntot // minibatch)

    # ------------------------------------------------------------------ bounded staleness
    def prologue_lagged(self, lag: int) -> None:
        """Rounds 0 .. lag-1, all collected with theta_0, queued in the channels."""
        if lag < 1 or (lag + 1) * self.n_agents > self.capacity:
            raise ValueError(f"lag {lag} needs channels of capacity >= {(max(lag, 1) + 1) * self.n_agents} slabs "
                             f"(have {self.capacity})")
        for r in range(lag):
            self.collect(r, 0)

    def iteration_lagged(self, k: int, lag: int, **train_args) -> None:
        """Trainer: theta_{k+1} from round k, the oldest in the channels.  Agents, concurrently: round k + lag with
        the published theta_k.  Then theta_{k+1} is published (after the agents' hand-off)."""
        self.train(k, k % 2, **train_args)
        self.collect(k + lag, 0)
        self.publish()

    def close(self) -> None:
        self.sync_all()
        for _, handle, _ in self.own:
            gmi_buffer_destroy(handle)
        gmi_channels_destroy(self.channels)
        super().close()
