"""Oracle for the channel-based experience sharing (Section 4.2) reduced to one GPU.

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing in the product).  Plain numpy.

What the paper describes: every agent's *dispenser* sorts its experience by type into channels (state, action,
reward, ...); the *compressor* joins several tensors of one channel into one larger movement; the *migrator*
routes channels to a trainer (the one with the least work when there are several); the trainer's *batcher*
slices (smaller batch) or stacks (larger batch) what arrives into its training batch.

The model here: a channel set is a FIFO of *slabs*.  A slab is one agent's experience of one collection round,
held as one array per type: obs [T, n, O], act [T, n, A], logp / val / rew [T, n] (float32), done [T, n] (uint8),
and the bootstrap values last_val [n].  push() appends a slab (fails when `capacity` slabs are waiting);
pop(k, env0, take) removes the k oldest slabs and returns, per type, the columns [env0, env0 + take) of each
(slicing) placed side by side in arrival order along the env axis (stacking).  Nothing is computed: every
output element is a copy of one input element, so parity is bit-exact.

Readings where the paper is silent: the FIFO order (oldest first) and the stacking order (arrival order along
the env axis) are this build's choice; "least workload" is the smallest number of samples handed to a trainer so
far, ties to the lowest trainer index; the uni-channel comparison of the paper's Table 8 moves the same slab as
ONE array of interleaved records, one record per (t, env): [obs | act | logp | val | rew | done as float], which
`pack_records` / `unpack_records` define.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

TYPES = ("obs", "act", "logp", "val", "rew", "done")


class ChannelError(RuntimeError):
    pass


class Channels:
    def __init__(self, horizon: int, n_envs: int, obs_dim: int, act_dim: int, capacity: int):
        self.T, self.n, self.O, self.A, self.capacity = horizon, n_envs, obs_dim, act_dim, capacity
        self.fifo: List[Dict[str, np.ndarray]] = []
        self.pushed = 0
        self.popped = 0

    def push(self, buf: Dict[str, np.ndarray], last_val: np.ndarray) -> None:
        """Dispenser + compressor: one slab, one array per type."""
        if len(self.fifo) >= self.capacity:
            raise ChannelError("channels full")
        slab = {}
        for k in TYPES:
            a = np.asarray(buf[k])
            want = (self.T, self.n) + ((self.O,) if k == "obs" else (self.A,) if k == "act" else ())
            if a.shape != want:
                raise ChannelError(f"{k}: shape {a.shape}, expected {want}")
            slab[k] = a.copy()
        lv = np.asarray(last_val)
        if lv.shape != (self.n,):
            raise ChannelError("last_val shape")
        slab["last_val"] = lv.copy()
        self.fifo.append(slab)
        self.pushed += 1

    def pop(self, k: int, env0: int = 0, take: int = None) -> Dict[str, np.ndarray]:
        """Migrator + batcher: the k oldest slabs, columns [env0, env0 + take) of each, stacked along envs."""
        take = self.n - env0 if take is None else take
        if k < 1 or k > len(self.fifo):
            raise ChannelError("not enough slabs")
        if env0 < 0 or take < 1 or env0 + take > self.n:
            raise ChannelError("bad slice")
        slabs, self.fifo = self.fifo[:k], self.fifo[k:]
        self.popped += k
        out = {key: np.concatenate([s[key][:, env0:env0 + take] for s in slabs], axis=1) for key in TYPES}
        out["last_val"] = np.concatenate([s["last_val"][env0:env0 + take] for s in slabs])
        return out

    def drop(self, k: int) -> None:
        """Discards the k oldest waiting slabs unread (an agent that must not wait for the trainer makes room this
        way: the asynchronous setting of Section 5.2).  They count as pushed, never as popped."""
        if k < 0 or k > len(self.fifo):
            raise ChannelError("not enough slabs")
        self.fifo = self.fifo[k:]

    def filled(self) -> int:
        return len(self.fifo)


def pack_records(buf: Dict[str, np.ndarray]) -> np.ndarray:
    """Uni-channel form of a slab: [T, n, O + A + 4] float32 records obs | act | logp | val | rew | done."""
    done = buf["done"].astype(np.float32)
    return np.concatenate([buf["obs"], buf["act"], buf["logp"][..., None], buf["val"][..., None],
                           buf["rew"][..., None], done[..., None]], axis=2).astype(np.float32)


def unpack_records(rec: np.ndarray, obs_dim: int, act_dim: int) -> Dict[str, np.ndarray]:
    O, A = obs_dim, act_dim
    return {"obs": rec[..., :O].copy(), "act": rec[..., O:O + A].copy(), "logp": rec[..., O + A].copy(),
            "val": rec[..., O + A + 1].copy(), "rew": rec[..., O + A + 2].copy(),
            "done": rec[..., O + A + 3].astype(np.uint8)}


def route_least_loaded(samples_so_far: Sequence[int]) -> int:
    """Migrator's choice among several trainers: the one that has received the fewest samples, lowest index on ties."""
    best = 0
    for i, s in enumerate(samples_so_far):
        if s < samples_so_far[best]:
            best = i
    return best
