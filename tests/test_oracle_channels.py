"""Pins of the channel oracle (Section 4.2 on one GPU): FIFO order, slicing and stacking as plain array
identities, capacity, the record form of the uni-channel comparison, least-loaded routing."""
import numpy as np
import pytest

from oracle import channels as och
from workloads import synthetic as syn


def slab(T, n, O, A, seed):
    b = syn.make_rollout_batch(T, n, O, A, seed=seed, done_prob=0.2)
    return b, b["last_val"]


def test_fifo_order_and_stacking_is_concatenation():
    ch = och.Channels(4, 6, 5, 3, capacity=4)
    slabs = [slab(4, 6, 5, 3, s) for s in range(3)]
    for b, lv in slabs:
        ch.push(b, lv)
    assert ch.filled() == 3
    out = ch.pop(2)
    for k in och.TYPES:
        assert out[k].shape[1] == 12
        assert np.array_equal(out[k][:, :6], slabs[0][0][k]) and np.array_equal(out[k][:, 6:], slabs[1][0][k])
    assert np.array_equal(out["last_val"], np.concatenate([slabs[0][1], slabs[1][1]]))
    assert ch.filled() == 1
    rest = ch.pop(1)
    assert np.array_equal(rest["obs"], slabs[2][0]["obs"])
    assert (ch.pushed, ch.popped) == (3, 3)


def test_drop_discards_the_oldest_and_keeps_the_order_of_the_rest():
    ch = och.Channels(4, 6, 5, 3, capacity=3)
    slabs = [slab(4, 6, 5, 3, s) for s in range(5)]
    for b, lv in slabs[:3]:
        ch.push(b, lv)
    ch.drop(1)                                   # slab 0 is gone, room for one more
    ch.push(*slabs[3])
    out = ch.pop(3)
    for j, src in enumerate((1, 2, 3)):
        assert np.array_equal(out["obs"][:, 6 * j:6 * (j + 1)], slabs[src][0]["obs"])
    assert (ch.pushed, ch.popped, ch.filled()) == (4, 3, 0)
    ch.drop(0)
    with pytest.raises(och.ChannelError):
        ch.drop(1)


def test_slices_of_one_slab_tile_it_exactly():
    """Popping the same slab content as two halves (pushed twice) gives back the two column halves: slicing
    followed by stacking is the identity."""
    b, lv = slab(3, 8, 4, 2, 7)
    ch = och.Channels(3, 8, 4, 2, capacity=2)
    ch.push(b, lv); ch.push(b, lv)
    left = ch.pop(1, 0, 4)
    right = ch.pop(1, 4, 4)
    for k in och.TYPES:
        assert np.array_equal(np.concatenate([left[k], right[k]], axis=1), b[k])
    assert np.array_equal(np.concatenate([left["last_val"], right["last_val"]]), lv)


def test_capacity_underflow_and_bad_arguments():
    ch = och.Channels(2, 4, 3, 2, capacity=2)
    b, lv = slab(2, 4, 3, 2, 1)
    ch.push(b, lv); ch.push(b, lv)
    with pytest.raises(och.ChannelError):
        ch.push(b, lv)                                  # full
    with pytest.raises(och.ChannelError):
        ch.pop(3)                                       # more than waiting
    with pytest.raises(och.ChannelError):
        ch.pop(1, 2, 3)                                 # slice past the slab
    ch.pop(2)
    with pytest.raises(och.ChannelError):
        ch.pop(1)                                       # empty
    bad = dict(b); bad["obs"] = b["obs"][:, :3]
    with pytest.raises(och.ChannelError):
        ch.push(bad, lv)
    ch.push(b, lv)                                      # room again after the pop: the ring wraps
    assert ch.filled() == 1


def test_copies_are_independent_of_the_source():
    ch = och.Channels(2, 4, 3, 2, capacity=1)
    b, lv = slab(2, 4, 3, 2, 3)
    keep = b["rew"].copy()
    ch.push(b, lv)
    b["rew"][:] = 0                                     # the agent reuses its buffer at once
    assert np.array_equal(ch.pop(1)["rew"], keep)


def test_records_round_trip_and_layout():
    b, _ = slab(3, 5, 4, 2, 9)
    rec = och.pack_records(b)
    assert rec.shape == (3, 5, 4 + 2 + 4) and rec.dtype == np.float32
    assert rec[1, 2, 0] == b["obs"][1, 2, 0] and rec[1, 2, 4] == b["act"][1, 2, 0]
    assert rec[2, 4, 6] == b["logp"][2, 4] and rec[2, 4, 7] == b["val"][2, 4] and rec[2, 4, 8] == b["rew"][2, 4]
    assert rec[0, 3, 9] == float(b["done"][0, 3])
    back = och.unpack_records(rec, 4, 2)
    for k in och.TYPES:
        assert np.array_equal(back[k], b[k]) and back[k].dtype == b[k].dtype


def test_least_loaded_routing():
    assert och.route_least_loaded([0, 0, 0]) == 0
    assert och.route_least_loaded([5, 3, 3]) == 1
    assert och.route_least_loaded([5, 3, 2]) == 2
    # feeding equal slabs one by one visits the trainers round-robin
    load, order = [0, 0, 0], []
    for _ in range(6):
        i = och.route_least_loaded(load); order.append(i); load[i] += 10
    assert order == [0, 1, 2, 0, 1, 2]
