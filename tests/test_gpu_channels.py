"""GPU parity of the experience channels (push = dispenser + compressor, pop = migrator + batcher) against the
oracle: every value is a copy, so all comparisons are bit-exact."""
import numpy as np
import pytest
import torch

from oracle import channels as och
from workloads import synthetic as syn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import paper_2206_08482_amd as lib
    return lib


def _buffers(g, inst, T, n, ld, O, A, col0=0):
    from paper_2206_08482_amd.runner import RolloutBuffers
    rb = RolloutBuffers(T, ld, O, A, torch.device("cuda:0"))
    torch.cuda.synchronize()
    return rb, g.gmi_buffer_bind(inst, rb.desc(col0, n))


def _upload(rb, b, col0):
    n = b["logp"].shape[1]
    for k in och.TYPES:
        getattr(rb, k)[:, col0:col0 + n].copy_(torch.tensor(b[k], device="cuda"))
    torch.cuda.synchronize()


@pytest.mark.parametrize("mode", ["multi", "uni"])
@pytest.mark.parametrize("T,n,O,A", [(4, 6, 5, 3), (16, 300, 60, 8), (3, 1000, 107, 21)])
def test_push_pop_matches_oracle(g, mode, T, n, O, A):
    agent, trainer = g.gmi_create(), g.gmi_create()
    cap = 4
    ch = g.gmi_channels_create(T, n, O, A, cap, g.CHANNELS_MULTI if mode == "multi" else g.CHANNELS_UNI)
    ref = och.Channels(T, n, O, A, cap)
    src_rb, src = _buffers(g, agent, T, n, n + 7, O, A, col0=3)          # the agent's buffer is a column slice
    k_stack, take, env0 = 2, max(1, n // 2), n - max(1, n // 2)
    dst_rb, dst = _buffers(g, trainer, T, 5 + k_stack * n, 5 + k_stack * n, O, A)
    last_out = torch.zeros(k_stack * n, device="cuda")
    seeds = iter(range(100))

    def push():
        b = syn.make_rollout_batch(T, n, O, A, seed=next(seeds), done_prob=0.3)
        _upload(src_rb, b, 3)
        lv = torch.tensor(b["last_val"], device="cuda")
        torch.cuda.synchronize()
        g.gmi_channels_push(agent, ch, src, lv)
        g.gmi_sync(agent)
        ref.push(b, b["last_val"])

    def pop_and_check(k, e0, tk, col0):
        want = ref.pop(k, e0, tk)
        for t in ("obs", "act", "logp", "val", "rew", "done"):
            getattr(dst_rb, t).zero_()
        last_out.zero_()
        torch.cuda.synchronize()
        g.gmi_channels_pop(trainer, ch, k, e0, tk, dst, col0, last_out)
        g.gmi_sync(trainer)
        got = dst_rb.to_numpy()
        for t in och.TYPES:
            assert np.array_equal(got[t][:, col0:col0 + k * tk], want[t]), t
            assert not got[t][:, :col0].any() and not got[t][:, col0 + k * tk:].any()      # nothing else touched
        assert np.array_equal(last_out.cpu().numpy()[:k * tk], want["last_val"])

    push(); push(); push()
    assert g.gmi_channels_count(ch) == (3, 3, 0)
    pop_and_check(2, 0, n, 5)                      # two whole slabs stacked
    push(); push(); push()                         # the ring wraps
    assert g.gmi_channels_count(ch)[0] == 4
    with pytest.raises(g.GmiError):
        g.gmi_channels_push(agent, ch, src, last_out)            # full
    pop_and_check(2, env0, take, 0)                # slices of two slabs stacked
    pop_and_check(1, 0, 1, 2)                      # a single env column
    pop_and_check(1, 0, n, 0)
    assert g.gmi_channels_count(ch) == (0, 6, 6)
    with pytest.raises(g.GmiError):
        g.gmi_channels_pop(trainer, ch, 1, 0, n, dst, 0, last_out)      # empty
    g.gmi_buffer_destroy(src); g.gmi_buffer_destroy(dst)
    g.gmi_channels_destroy(ch)
    g.gmi_destroy(agent); g.gmi_destroy(trainer)


@pytest.mark.parametrize("mode", ["multi", "uni"])
def test_drop_makes_room_and_the_reused_slab_holds_the_new_round(g, mode):
    """Two agents on streams of their own fill a ring of 3; the oldest slabs are discarded unread and their places
    refilled by the OTHER agent without any host wait in between (the refill has to wait, on the device, for the
    discarded push): what the trainer pops is what the oracle's queue holds, bit for bit."""
    T, n, O, A, cap = 5, 200, 33, 6, 3
    agents = [g.gmi_create(), g.gmi_create()]
    trainer = g.gmi_create()
    ch = g.gmi_channels_create(T, n, O, A, cap, g.CHANNELS_MULTI if mode == "multi" else g.CHANNELS_UNI)
    ref = och.Channels(T, n, O, A, cap)
    srcs = [_buffers(g, a, T, n, n, O, A) for a in agents]
    lvs = [torch.zeros(n, device="cuda") for _ in agents]
    dst_rb, dst = _buffers(g, trainer, T, cap * n, cap * n, O, A)
    last_out = torch.zeros(cap * n, device="cuda")

    def push(i, seed, wait):
        b = syn.make_rollout_batch(T, n, O, A, seed=seed, done_prob=0.3)
        g.gmi_sync(agents[i])                     # the agent's buffer is free again (its last push has run)
        _upload(srcs[i][0], b, 0)
        lvs[i].copy_(torch.tensor(b["last_val"], device="cuda"))
        torch.cuda.synchronize()
        g.gmi_channels_push(agents[i], ch, srcs[i][1], lvs[i])
        if wait:
            g.gmi_sync(agents[i])
        ref.push(b, b["last_val"])

    push(0, 1, True); push(1, 2, True); push(0, 3, False)        # ring full: slabs 0, 1, 2
    with pytest.raises(g.GmiError):
        g.gmi_channels_drop(ch, 4)                               # more than are waiting
    g.gmi_channels_drop(ch, 2); ref.drop(2)                      # slabs 0 and 1 discarded unread
    assert g.gmi_channels_count(ch) == (1, 3, 0)
    push(1, 4, False); push(1, 5, False)                         # refills slabs 0 and 1 from the other stream
    assert g.gmi_channels_count(ch) == (3, 5, 0)
    want = ref.pop(3)
    g.gmi_channels_pop(trainer, ch, 3, 0, n, dst, 0, last_out)
    g.gmi_sync(trainer)
    got = dst_rb.to_numpy()
    for t in och.TYPES:
        assert np.array_equal(got[t], want[t]), t
    assert np.array_equal(last_out.cpu().numpy(), want["last_val"])
    assert g.gmi_channels_count(ch) == (0, 5, 3)
    g.gmi_channels_drop(ch, 0)
    # a ring of one slab: agent 0's push is discarded while it may still be running, agent 1's push into the same
    # slab is queued at once on another stream and must wait for it on the device
    ch1 = g.gmi_channels_create(T, n, O, A, 1, g.CHANNELS_MULTI if mode == "multi" else g.CHANNELS_UNI)
    b0 = syn.make_rollout_batch(T, n, O, A, seed=11, done_prob=0.3)
    b1 = syn.make_rollout_batch(T, n, O, A, seed=12, done_prob=0.3)
    for i, b in enumerate((b0, b1)):
        g.gmi_sync(agents[i])
        _upload(srcs[i][0], b, 0)
        lvs[i].copy_(torch.tensor(b["last_val"], device="cuda"))
    torch.cuda.synchronize()
    g.gmi_channels_push(agents[0], ch1, srcs[0][1], lvs[0])
    g.gmi_channels_drop(ch1, 1)
    g.gmi_channels_push(agents[1], ch1, srcs[1][1], lvs[1])
    g.gmi_channels_pop(trainer, ch1, 1, 0, n, dst, 0, last_out)
    g.gmi_sync(trainer)
    got = dst_rb.to_numpy()
    for t in och.TYPES:
        assert np.array_equal(got[t][:, :n], b1[t]), t
    assert np.array_equal(last_out.cpu().numpy()[:n], b1["last_val"])
    g.gmi_channels_destroy(ch1)
    for (_, h) in srcs:
        g.gmi_buffer_destroy(h)
    g.gmi_buffer_destroy(dst)
    g.gmi_channels_destroy(ch)
    for a in agents:
        g.gmi_destroy(a)
    g.gmi_destroy(trainer)


def test_hand_off_is_ordered_by_events_not_by_the_host(g):
    """The agent refills its buffer right after the push and the trainer pops at once, with no host
    synchronisation in between: the trainer must see the pushed values (masked instances on disjoint CUs)."""
    from paper_2206_08482_amd.instances import cu_masks
    probe = g.gmi_create(); n_cu = g.gmi_cu_count(probe); g.gmi_destroy(probe)
    masks = cu_masks(n_cu, [n_cu // 2 // 8 * 8, n_cu - n_cu // 2 // 8 * 8])
    agent, trainer = g.gmi_create(masks[0]), g.gmi_create(masks[1])
    T, n, O, A = 16, 4096, 60, 8
    ch = g.gmi_channels_create(T, n, O, A, 2)
    src_rb, src = _buffers(g, agent, T, n, n, O, A)
    dst_rb, dst = _buffers(g, trainer, T, 2 * n, 2 * n, O, A)
    b1 = syn.make_rollout_batch(T, n, O, A, seed=1)
    b2 = syn.make_rollout_batch(T, n, O, A, seed=2)
    dev = {k: (torch.tensor(b1[k], device="cuda"), torch.tensor(b2[k], device="cuda")) for k in och.TYPES}
    lv = (torch.tensor(b1["last_val"], device="cuda"), torch.tensor(b2["last_val"], device="cuda"))
    last_out = torch.zeros(2 * n, device="cuda")
    torch.cuda.synchronize()
    for rep in range(3):
        for i in (0, 1):          # fill (device-to-device on the agent's stream), push, refill, push: no host waits
            for k in och.TYPES:
                t = getattr(src_rb, k)
                g.gmi_transfer(agent, agent, dev[k][i], t, t.numel() * t.element_size())
            g.gmi_channels_push(agent, ch, src, lv[i])
        g.gmi_channels_pop(trainer, ch, 2, 0, n, dst, 0, last_out)
        g.gmi_sync(trainer)
        got = dst_rb.to_numpy()
        for k in och.TYPES:
            assert np.array_equal(got[k][:, :n], b1[k]) and np.array_equal(got[k][:, n:], b2[k]), (rep, k)
        assert np.array_equal(last_out.cpu().numpy(), np.concatenate([b1["last_val"], b2["last_val"]]))
    g.gmi_sync(agent)
    g.gmi_buffer_destroy(src); g.gmi_buffer_destroy(dst)
    g.gmi_channels_destroy(ch)
    g.gmi_destroy(agent); g.gmi_destroy(trainer)


def test_channel_error_paths(g):
    inst = g.gmi_create()
    with pytest.raises(g.GmiError):
        g.gmi_channels_create(0, 4, 3, 2, 1)
    with pytest.raises(g.GmiError):
        g.gmi_channels_create(4, 4, 3, 2, 1, mode=7)
    ch = g.gmi_channels_create(4, 8, 3, 2, 1)
    rb, wrong = _buffers(g, inst, 4, 6, 6, 3, 2)             # 6 envs, slabs hold 8
    lv = torch.zeros(8, device="cuda")
    with pytest.raises(g.GmiError):
        g.gmi_channels_push(inst, ch, wrong, lv)
    rb2, ok = _buffers(g, inst, 4, 8, 8, 3, 2)
    g.gmi_channels_push(inst, ch, ok, lv)
    with pytest.raises(g.GmiError):
        g.gmi_channels_pop(inst, ch, 1, 4, 8, ok, 0, lv)     # slice past the slab
    with pytest.raises(g.GmiError):
        g.gmi_channels_pop(inst, ch, 1, 0, 8, ok, 1, lv)     # columns past the buffer
    with pytest.raises(g.GmiError):
        g.gmi_channels_pop(inst, ch, 2, 0, 8, ok, 0, lv)     # more than waiting
    g.gmi_channels_pop(inst, ch, 1, 0, 8, ok, 0, lv)
    g.gmi_sync(inst)
    g.gmi_buffer_destroy(wrong); g.gmi_buffer_destroy(ok)
    g.gmi_channels_destroy(ch)
    g.gmi_destroy(inst)


def test_channel_pipeline_equals_the_direct_hand_off_bit_for_bit(g):
    """The same agents, seeds and schedule through channels (both forms) and through the direct column-slice
    hand-off: the trainer sees identical batches, so the parameters after two iterations are identical."""
    from paper_2206_08482_amd.channels import ChannelPipeline
    from paper_2206_08482_amd.instances import InstancePipeline
    cfg = syn.get_config("C2")
    n_ag, n, T, mb = 3, 96, 4, 288
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    states = [syn.make_initial_state(n, cfg.obs_dim, 40 + i) for i in range(n_ag)]
    common = dict(n_agents=n_ag, n_envs=n, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim, hidden=cfg.hidden, horizon=T,
                  dtype="bf16", theta=theta, a_mat=a_mat, b_mat=b_mat, state0=states, noise_std=cfg.noise_std,
                  reward_scale=1.0, done_period=0, done_threshold=(1 << 32) // 50, seed=3, minibatch=mb)
    targs = dict(gamma=0.99, lam=0.95, epochs=2, minibatch=mb, clip=0.2, c_v=0.5, c_e=0.0, lr=3e-4)
    results = []
    for make in (lambda: InstancePipeline(**common), lambda: ChannelPipeline(mode=g.CHANNELS_MULTI, **common),
                 lambda: ChannelPipeline(mode=g.CHANNELS_UNI, **common)):
        pipe = make()
        pipe.prologue_pipelined()
        for k in range(2):
            pipe.iteration_pipelined(k, **targs)
        pipe.sync_all()
        results.append((pipe.theta.cpu().numpy().copy(), pipe.bufs[1].to_numpy()))     # slot 1 holds the second collection in both
        pipe.close()
    for th, buf in results[1:]:
        assert np.array_equal(th, results[0][0])
        for k in och.TYPES + ("adv", "ret"):
            assert np.array_equal(buf[k], results[0][1][k]), k


def _lag_common(cfg, n_ag, n, T, mb, lr=3e-4):
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    states = [syn.make_initial_state(n, cfg.obs_dim, 70 + i) for i in range(n_ag)]
    common = dict(n_agents=n_ag, n_envs=n, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim, hidden=cfg.hidden, horizon=T,
                  dtype="bf16", theta=theta, a_mat=a_mat, b_mat=b_mat, state0=states, noise_std=cfg.noise_std,
                  reward_scale=1.0, done_period=0, done_threshold=(1 << 32) // 50, seed=5, minibatch=mb)
    targs = dict(gamma=0.99, lam=0.95, epochs=2, minibatch=mb, clip=0.2, c_v=0.5, c_e=0.0, lr=lr)
    return theta, a_mat, b_mat, states, common, targs


@pytest.mark.parametrize("host_ordered", [False, True])
def test_lagged_schedule_bit_for_bit(g, host_ordered):
    """lag = 1 is the pipelined schedule; for lag = 3 the concurrent form (agents and trainer overlap) gives the
    same bits as the same stages run one at a time with the host waiting in between."""
    from paper_2206_08482_amd.channels import ChannelPipeline
    cfg = syn.get_config("C2")
    n_ag, n, T, mb = 2, 64, 4, 128
    _, _, _, _, common, targs = _lag_common(cfg, n_ag, n, T, mb)
    out = {}
    for name in ("pipelined", "lag1", "lag3", "lag3_sequential"):
        lag = 3 if name.startswith("lag3") else 1
        pipe = ChannelPipeline(mode=g.CHANNELS_MULTI, capacity=(lag + 1) * n_ag, host_ordered=host_ordered, **common)
        if name == "pipelined":
            pipe.prologue_pipelined()
            for k in range(3):
                pipe.iteration_pipelined(k, **targs)
        elif name == "lag3_sequential":
            pipe.prologue_lagged(lag); pipe.sync_all()
            for k in range(3):      # the same stages in an order that never overlaps two instances
                pipe.collect(k + lag, 0); pipe.sync_all()
                pipe.train(k, k % 2, **targs); pipe.sync_all()
                pipe.publish(); pipe.sync_all()
        else:
            pipe.prologue_lagged(lag)
            for k in range(3):
                pipe.iteration_lagged(k, lag, **targs)
        pipe.sync_all()
        out[name] = (pipe.theta.cpu().numpy().copy(), pipe.bufs[0].to_numpy())
        assert g.gmi_channels_count(pipe.channels)[0] == lag * n_ag        # the agents stay `lag` rounds ahead
        pipe.close()
    assert np.array_equal(out["lag1"][0], out["pipelined"][0])
    assert np.array_equal(out["lag3"][0], out["lag3_sequential"][0])
    for key in och.TYPES + ("adv", "ret"):
        assert np.array_equal(out["lag3"][1][key], out["lag3_sequential"][1][key]), key
    assert not np.array_equal(out["lag3"][0], out["lag1"][0])           # staleness changes the result


def test_lagged_schedule_uses_the_parameters_it_states(g):
    """Oracle replay with a step size large enough that parameter versions differ visibly: round r is collected
    with theta_{max(0, r - lag)}; replaying with any other version misses by far more than the bf16 band."""
    from oracle import ppo as oppo
    from paper_2206_08482_amd.channels import ChannelPipeline
    from gpu_util import rel_l2
    cfg = syn.get_config("C2")
    n_ag, n, T, mb, lag, lr = 2, 64, 4, 256, 2, 2e-2
    theta, a_mat, b_mat, states, common, targs = _lag_common(cfg, n_ag, n, T, mb, lr=lr)
    shape = oppo.ModelShape(cfg.obs_dim, cfg.act_dim, tuple(cfg.hidden))
    envs = [oppo.EnvSpec(a_mat, b_mat, cfg.noise_std, 1.0, 0, (1 << 32) // 50, 5 + i) for i in range(n_ag)]

    class Replay:
        def __init__(self):
            self.states = [s.copy() for s in states]
            self.eps = [np.zeros(n, np.uint32) for _ in envs]

        def collect(self, th, r, keep=True):
            buf = oppo.new_buffer(T, n_ag * n, cfg.obs_dim, cfg.act_dim)
            last = np.zeros(n_ag * n, np.float32)
            st, ep = [], []
            for i, env in enumerate(envs):
                s2, e2, lv = oppo.rollout(th, shape, env, self.states[i], self.eps[i], buf, env.seed, r, col0=i * n)
                st.append(s2); ep.append(e2)
                last[i * n:(i + 1) * n] = lv
            if keep:
                self.states, self.eps = st, ep
            buf["adv"], buf["ret"] = oppo.gae(buf["rew"], buf["val"], buf["done"], last, 0.99, 0.95, True)
            return buf

    pipe = ChannelPipeline(mode=g.CHANNELS_MULTI, capacity=(lag + 1) * n_ag, **common)
    rep = Replay()
    th = [theta]            # the trainer's own parameter versions (Adam at this step size amplifies bf16 noise in
                            # near-zero gradients, so the update itself is compared elsewhere, at the usual step size)
    rounds = [rep.collect(theta, r) for r in range(lag)]
    pipe.prologue_lagged(lag)
    for k in range(3):
        pipe.iteration_lagged(k, lag, **targs)
        pipe.sync_all()
        th.append(pipe.theta.cpu().numpy().copy())
        newer = rep.collect(th[k + 1], k + lag, keep=False)       # what agents that had not lagged would have collected
        rounds.append(rep.collect(th[k], k + lag))
        # the trainer's batch of iteration k is round k; what the agents just pushed is round k + lag (their own
        # buffers still hold it)
        got = pipe.bufs[k % 2].to_numpy()
        for name in ("obs", "act", "rew"):
            assert rel_l2(got[name], rounds[k][name]) <= 2e-2, (k, name)
        own_act = np.concatenate([rb.to_numpy()["act"] for rb, _, _ in pipe.own], axis=1)
        err = rel_l2(own_act, rounds[k + lag]["act"])
        assert err <= 2e-2, (k, err)
        assert rel_l2(own_act, newer["act"]) > 5 * err, k
    pipe.close()
