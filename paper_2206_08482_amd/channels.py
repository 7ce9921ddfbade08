"""Agent instances feeding a trainer instance through experience channels (Section 4.2 of the paper) instead of
writing straight into the trainer's batch: every agent instance collects into a buffer of its own and pushes it
as a slab; the trainer pops the slabs of a round, stacked side by side, into its batch.  Same two schedules as
`instances.InstancePipeline` (whose direct hand-off moves no bytes and is the comparison point); the lag-1
pipelined one is the one-GPU form of the paper's asynchronous serving / training.  No arithmetic of the method
happens here."""
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

    def close(self) -> None:
        self.sync_all()
        for _, handle, _ in self.own:
            gmi_buffer_destroy(handle)
        gmi_channels_destroy(self.channels)
        super().close()
