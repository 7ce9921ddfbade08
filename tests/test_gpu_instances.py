"""GPU parity of the multi-instance layout (several agent instances + one trainer instance on CU-masked
streams) against the oracle, for the synchronous and the lag-1 pipelined schedule."""
import numpy as np
import pytest
import torch

from oracle import ppo as oppo
from workloads import synthetic as syn
from gpu_util import rel_l2, rel_max

pytestmark = pytest.mark.gpu


def _setup(cfg, n_agents, n_envs, horizon, minibatch):
    shape = oppo.ModelShape(cfg.obs_dim, cfg.act_dim, tuple(cfg.hidden))
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    thr = oppo.done_threshold_from_inverse(cfg.done_prob_inv)
    envs = [oppo.EnvSpec(a_mat, b_mat, cfg.noise_std, cfg.reward_scale, cfg.done_period, thr, cfg.seed + i)
            for i in range(n_agents)]
    states = [syn.make_initial_state(n_envs, cfg.obs_dim, cfg.seed + 10 + i) for i in range(n_agents)]
    hp = oppo.PPOHyper(clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, lr=cfg.lr, epochs=2, minibatch=minibatch)
    return shape, theta, a_mat, b_mat, thr, envs, states, hp


class _OracleAgents:
    def __init__(self, shape, envs, states, n_envs, horizon, cfg):
        self.shape, self.envs, self.N, self.T, self.cfg = shape, envs, n_envs, horizon, cfg
        self.states = [s.copy() for s in states]
        self.eps = [np.zeros(n_envs, np.uint32) for _ in envs]

    def collect(self, theta, k):
        n_ag = len(self.envs)
        buf = oppo.new_buffer(self.T, n_ag * self.N, self.cfg.obs_dim, self.cfg.act_dim)
        last = np.zeros(n_ag * self.N, np.float32)
        for i, env in enumerate(self.envs):
            self.states[i], self.eps[i], lv = oppo.rollout(theta, self.shape, env, self.states[i], self.eps[i], buf,
                                                           env.seed, k, col0=i * self.N)
            last[i * self.N:(i + 1) * self.N] = lv
        buf["adv"], buf["ret"] = oppo.gae(buf["rew"], buf["val"], buf["done"], last, self.cfg.gamma, self.cfg.lam, True)
        return buf


def _pipeline(cfg, dtype, n_agents, n_envs, horizon, minibatch, theta, a_mat, b_mat, thr, states, masked,
              host_ordered=False):
    import paper_2206_08482_amd as g
    from paper_2206_08482_amd.instances import InstancePipeline, cu_masks
    probe = g.gmi_create()
    n_cu = g.gmi_cu_count(probe)
    g.gmi_destroy(probe)
    agent_masks = trainer_mask = None
    if masked == "agents":      # the agents on disjoint CU sets, the trainer on the whole device
        agent_masks = cu_masks(n_cu, [(n_cu // n_agents) // 8 * 8] * n_agents, "interleaved")
    elif masked:
        share = (n_cu // 2 // n_agents) // 8 * 8
        masks = cu_masks(n_cu, [share] * n_agents + [n_cu - share * n_agents], "contiguous")
        agent_masks, trainer_mask = masks[:n_agents], masks[n_agents]
    return InstancePipeline(n_agents=n_agents, n_envs=n_envs, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim,
                            hidden=cfg.hidden, horizon=horizon, dtype=dtype, theta=theta, a_mat=a_mat, b_mat=b_mat,
                            state0=states, noise_std=cfg.noise_std, reward_scale=cfg.reward_scale,
                            done_period=cfg.done_period, done_threshold=thr, seed=cfg.seed, minibatch=minibatch,
                            agent_masks=agent_masks, trainer_mask=trainer_mask, host_ordered=host_ordered)


def _train_args(cfg, minibatch):
    return dict(gamma=cfg.gamma, lam=cfg.lam, epochs=2, minibatch=minibatch, clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e,
                lr=cfg.lr)


def test_cu_masks_are_disjoint_and_sized():
    from paper_2206_08482_amd.instances import cu_masks
    for style in ("contiguous", "interleaved"):
        masks = cu_masks(256, [48, 48, 48, 48, 64], style)
        ints = [sum(w << (32 * i) for i, w in enumerate(m)) for m in masks]
        assert [bin(x).count("1") for x in ints] == [48, 48, 48, 48, 64]
        for i in range(5):
            for j in range(i):
                assert ints[i] & ints[j] == 0
        assert sum(ints) == (1 << 256) - 1
        for x in ints:      # every instance has CUs on each of the 8 dies (bit index mod 8)
            assert all(any((x >> b) & 1 for b in range(d, 256, 8)) for d in range(8))


@pytest.mark.parametrize("masked,host_ordered", [(False, False), (True, False), (True, True), ("agents", True)])
def test_sync_schedule_matches_oracle_fp32(masked, host_ordered):
    cfg = syn.get_config("C1")
    n_agents, n_envs, horizon, minibatch = 3, 32, 8, 192
    shape, theta, a_mat, b_mat, thr, envs, states, hp = _setup(cfg, n_agents, n_envs, horizon, minibatch)
    pipe = _pipeline(cfg, "f32", n_agents, n_envs, horizon, minibatch, theta, a_mat, b_mat, thr, states, masked,
                     host_ordered)
    if masked:
        a_cus, t_cus = pipe.cu_counts()
        assert len(set(a_cus)) == 1 and sum(a_cus) + t_cus > 0
    ora = _OracleAgents(shape, envs, states, n_envs, horizon, cfg)
    th, m, v, kk = theta, np.zeros_like(theta), np.zeros_like(theta), 0
    for k in range(3):
        pipe.iteration_sync(k, **_train_args(cfg, minibatch))
        pipe.sync_all()
        buf = ora.collect(th, k)
        got = pipe.bufs[0].to_numpy()
        assert np.array_equal(got["done"], buf["done"])
        for name in ("obs", "act", "logp", "val", "rew", "adv", "ret"):
            assert rel_l2(got[name], buf[name]) <= 5e-5, (k, name, rel_l2(got[name], buf[name]))
        th, m, v, kk, _ = oppo.ppo_update(th, m, v, kk, shape, buf, hp, cfg.seed, k)
        assert rel_l2(pipe.theta.cpu().numpy(), th) <= 2e-5
        assert np.array_equal(pipe.theta_pub.cpu().numpy(), pipe.theta.cpu().numpy())   # published
    pipe.close()


@pytest.mark.parametrize("host_ordered", [False, True])
def test_pipelined_schedule_matches_oracle_fp32(host_ordered):
    cfg = syn.get_config("C1")
    n_agents, n_envs, horizon, minibatch = 2, 64, 8, 256
    shape, theta, a_mat, b_mat, thr, envs, states, hp = _setup(cfg, n_agents, n_envs, horizon, minibatch)
    pipe = _pipeline(cfg, "f32", n_agents, n_envs, horizon, minibatch, theta, a_mat, b_mat, thr, states, True,
                     host_ordered)
    ora = _OracleAgents(shape, envs, states, n_envs, horizon, cfg)
    # oracle replay of the lag-1 schedule: D_0 and D_1 are both collected with theta_0
    th = [theta]
    m, v, kk = np.zeros_like(theta), np.zeros_like(theta), 0
    bufs = [ora.collect(theta, 0)]
    pipe.prologue_pipelined()
    for k in range(3):
        pipe.iteration_pipelined(k, **_train_args(cfg, minibatch))
        pipe.sync_all()
        bufs.append(ora.collect(th[k], k + 1))                   # agents still hold theta_k
        new_th, m, v, kk, _ = oppo.ppo_update(th[k], m, v, kk, shape, bufs[k], hp, cfg.seed, k)
        th.append(new_th)
        got = pipe.bufs[(k + 1) % 2].to_numpy()
        for name in ("obs", "act", "logp", "val", "rew"):
            assert rel_l2(got[name], bufs[k + 1][name]) <= 5e-5, (k, name)
        assert rel_l2(pipe.theta.cpu().numpy(), th[k + 1]) <= 2e-5, k
    pipe.close()


@pytest.mark.parametrize("host_ordered", [False, True])
def test_pipelined_schedule_bf16_matches_oracle_replay(host_ordered):
    """The multi-instance configuration's model in bf16, lag-1 schedule on masked instances, against the oracle's
    replay of the same schedule (round k + 1 collected with the parameters after k updates).  The step size is
    large enough for a round collected with the wrong parameter version to miss its reference by far more than
    the bf16 band, which is asserted for the round that would show it.  The trainer's parameters: relative to
    their own size they are the start parameters (trivial); relative to the update they follow the oracle's
    to the extent Adam allows -- its early steps are lr * sign-like, so the ~0.5 % of weights whose bf16
    gradient error exceeds their gradient move the other way (bound 0.25 on the step, derived from that share)."""
    cfg = syn.get_config("C3")
    n_agents, n_envs, horizon, minibatch = 4, 128, 4, 1024
    shape, theta, a_mat, b_mat, thr, envs, states, hp = _setup(cfg, n_agents, n_envs, horizon, minibatch)
    hp.lr = 2e-3
    pipe = _pipeline(cfg, "bf16", n_agents, n_envs, horizon, minibatch, theta, a_mat, b_mat, thr, states, True,
                     host_ordered)
    ora = _OracleAgents(shape, envs, states, n_envs, horizon, cfg)
    args = _train_args(cfg, minibatch)
    args["lr"] = hp.lr
    th = [theta]
    m, v, kk = np.zeros_like(theta), np.zeros_like(theta), 0
    bufs = [ora.collect(theta, 0)]
    pipe.prologue_pipelined()
    for k in range(3):
        pipe.iteration_pipelined(k, **args)
        pipe.sync_all()
        bufs.append(ora.collect(th[k], k + 1))                   # agents still hold theta_k
        new_th, m, v, kk, _ = oppo.ppo_update(th[k], m, v, kk, shape, bufs[k], hp, cfg.seed, k)
        th.append(new_th)
        got = pipe.bufs[(k + 1) % 2].to_numpy()
        assert np.array_equal(got["done"], bufs[k + 1]["done"])
        for name in ("obs", "act", "val", "rew"):
            assert rel_l2(got[name], bufs[k + 1][name]) <= 2e-2, (k, name, rel_l2(got[name], bufs[k + 1][name]))
            assert rel_max(got[name], bufs[k + 1][name]) <= 2e-2, (k, name)
        # noise and log_std only; log_std is a trained parameter here, so it carries the trainer's bf16 error
        assert rel_l2(got["logp"], bufs[k + 1]["logp"]) <= 1e-4
        got_th = pipe.theta.cpu().numpy()
        assert rel_l2(got_th, th[k + 1]) <= 2e-2, k
        step, ref_step = got_th - theta, th[k + 1] - theta
        assert rel_l2(step, ref_step) <= 0.25, (k, rel_l2(step, ref_step))
        if k == 1:
            # collection round k + 1 = 2 used theta_1; a rollout under theta_0 or theta_2 is NOT what the buffer holds
            st, ep = [s.copy() for s in ora.states], [e.copy() for e in ora.eps]
            for wrong in (th[0], th[2]):
                probe = _OracleAgents(shape, envs, states, n_envs, horizon, cfg)
                probe.collect(theta, 0); probe.collect(th[0], 1)
                assert rel_l2(got["val"], probe.collect(wrong, 2)["val"]) > 5e-2
            ora.states, ora.eps = st, ep
    pipe.close()


@pytest.mark.parametrize("fused_rollout", [True, False])
def test_sync_schedule_bf16_runs_and_stays_close(fused_rollout):
    cfg = syn.get_config("C3")
    n_agents, n_envs, horizon, minibatch = 4, 128, 4, 1024
    shape, theta, a_mat, b_mat, thr, envs, states, hp = _setup(cfg, n_agents, n_envs, horizon, minibatch)
    pipe = _pipeline(cfg, "bf16", n_agents, n_envs, horizon, minibatch, theta, a_mat, b_mat, thr, states, True)
    pipe.fused_rollout = fused_rollout
    ora = _OracleAgents(shape, envs, states, n_envs, horizon, cfg)
    pipe.iteration_sync(0, **_train_args(cfg, minibatch))
    pipe.sync_all()
    assert pipe.fused_rollout == fused_rollout        # the one-launch collection really ran for this model
    buf = ora.collect(theta, 0)
    got = pipe.bufs[0].to_numpy()
    assert np.array_equal(got["done"], buf["done"])
    for name in ("obs", "act", "val", "rew", "ret"):
        assert rel_l2(got[name], buf[name]) <= 2e-2, name
    assert rel_l2(got["logp"], buf["logp"]) <= 1e-5
    # the published shadow equals the trainer's shadow after the update
    assert torch.equal(pipe.shadow[0], pipe.shadow[1])
    assert torch.isfinite(pipe.theta).all().item()
    pipe.close()


def test_instance_exploration_on_real_trial_runs():
    """Algorithm 2 with profile() = real PPO iterations on CU-masked holistic instances: every point of a
    small grid runs, throughput and memory are positive, and the pair the library returns is the one the
    oracle picks from the very same measurements (replayed as a table)."""
    import paper_2206_08482_amd as g
    from gpu_util import make_session, oracle_pieces
    from oracle import selection as osel
    from paper_2206_08482_amd.selection import InstanceProfiler, cus_per_instance

    cfg = syn.get_config("C2")
    shape, theta, env, _, hp = oracle_pieces(cfg, n_envs=64)

    def build(num_env, cu_mask):
        from paper_2206_08482_amd.runner import PPOSession
        state0 = syn.make_initial_state(num_env, cfg.obs_dim, cfg.seed)
        return PPOSession(n_envs=num_env, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim, hidden=cfg.hidden, horizon=4,
                          dtype="bf16", theta=theta, a_mat=env.a_mat, b_mat=env.b_mat, state0=state0,
                          noise_std=env.noise_std, reward_scale=env.reward_scale, done_period=env.done_period,
                          done_threshold=env.done_threshold, seed=env.seed, minibatch=2 * num_env, cu_mask=cu_mask)

    def step(ses, it):
        ses.rollout(it)
        ses.gae(cfg.gamma, cfg.lam, True)
        ses.update(it, epochs=1, minibatch=2 * ses.N, clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, lr=cfg.lr)

    prof = InstanceProfiler(build, step, lambda n: 4 * n, iterations=2)
    ks, ns = [4, 3, 1], [128, 256, 512]
    assert [cus_per_instance(prof.device_cus, k) for k in ks] == [prof.device_cus // 4, prof.device_cus // 3 // 8 * 8,
                                                                 prof.device_cus]
    ninf = float("-inf")                                  # no Sat is below it: the search never stops early
    got = g.gmi_explore(prof, 1, ninf, ks, ns)
    assert len(prof.log) == 9 and all(r["runnable"] for r in prof.log), prof.log
    assert all(r["samples_per_s"] > 0 and r["bytes"] >= 0 for r in prof.log)
    table = {(r["gmi_per_gpu"], r["num_env"]): (True, r["samples_per_s"], r["bytes"]) for r in prof.log}
    ref = osel.explore(lambda k, n: table[(k, n)], lambda k, gpus, top: top * k * gpus, 1, ninf, ks, ns)
    assert (got is None and ref is None) or got[:2] == ref
    # a point that cannot run (fewer than one CU per die for each instance) is reported as not runnable
    prof2 = InstanceProfiler(build, step, lambda n: 4 * n, iterations=1)
    assert prof2(prof.device_cus, 128) == (False, 0.0, 0.0)
    assert prof2.log[-1]["runnable"] is False
