"""The asynchronous schedule (agents and trainer on host threads of their own, experience through the channels):
the run is timing-dependent, so it is checked by replaying its recorded trace with the oracle -- every round with
the parameter version the trace says it was collected with, every update on the slabs the trace says it popped."""
import numpy as np
import pytest

from oracle import fp8model as f8
from oracle import ppo as oppo
from workloads import synthetic as syn
from gpu_util import rel_l2

pytestmark = pytest.mark.gpu


def _make(cfg, dtype, n_agents, n_envs, horizon, minibatch, slabs, capacity, on_full, masked=False,
          agent_precision="model"):
    import paper_2206_08482_amd as g
    from paper_2206_08482_amd.async_schedule import AsyncPipeline
    from paper_2206_08482_amd.instances import cu_masks
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    thr = oppo.done_threshold_from_inverse(cfg.done_prob_inv)
    states = [syn.make_initial_state(n_envs, cfg.obs_dim, cfg.seed + 10 + i) for i in range(n_agents)]
    agent_masks = None
    if masked:
        probe = g.gmi_create()
        n_cu = g.gmi_cu_count(probe)
        g.gmi_destroy(probe)
        agent_masks = cu_masks(n_cu, [(n_cu // n_agents) // 8 * 8] * n_agents, "contiguous")
    pipe = AsyncPipeline(n_agents=n_agents, n_envs=n_envs, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim,
                         hidden=cfg.hidden, horizon=horizon, dtype=dtype, theta=theta, a_mat=a_mat, b_mat=b_mat,
                         state0=states, noise_std=cfg.noise_std, reward_scale=cfg.reward_scale,
                         done_period=cfg.done_period, done_threshold=thr, seed=cfg.seed, minibatch=minibatch,
                         slabs_per_update=slabs, capacity=capacity, on_full=on_full, agent_masks=agent_masks,
                         agent_precision=agent_precision)
    envs = [oppo.EnvSpec(a_mat, b_mat, cfg.noise_std, cfg.reward_scale, cfg.done_period, thr, cfg.seed + i)
            for i in range(n_agents)]
    return pipe, theta, envs, states


def _rollout_fp8(theta, shape, env, state, eps, buf, seed, r):
    """oracle.ppo.rollout with the agent's decisions (and the bootstrap value) taken by the fp8 model."""
    T = buf["obs"].shape[0]
    for t in range(T):
        step = r * T + t
        act, logp, val, _ = f8.agent_act(theta, shape, state, seed, step)
        nxt, rew, done, eps = oppo.env_step(env, state, act, eps, step, np.float32, 0)
        oppo.collect_experience(buf, t, state, act, logp, val, rew, done, 0)
        state = nxt
    return state, eps, f8.agent_forward(theta, shape, state)[1]


def _replay(trace, cfg, theta, envs, states, n_envs, horizon, hp, fp8=False):
    """The oracle walks the trace; returns the parameter versions and the number of rounds it collected."""
    shape = oppo.ModelShape(cfg.obs_dim, cfg.act_dim, tuple(cfg.hidden))
    th = [theta]
    m, v, kk = np.zeros_like(theta), np.zeros_like(theta), 0
    st = [s.copy() for s in states]
    ep = [np.zeros(n_envs, np.uint32) for _ in envs]
    nxt = [0] * len(envs)
    slabs = {}
    for ev in trace:
        if ev[0] == "push":
            i, r, ver = ev[1]
            assert r == nxt[i], "an agent's rounds enter the ring in order"
            assert ver < len(th), "a round cannot use parameters that did not exist yet"
            buf = oppo.new_buffer(horizon, n_envs, cfg.obs_dim, cfg.act_dim)
            if fp8:
                st[i], ep[i], last = _rollout_fp8(th[ver], shape, envs[i], st[i], ep[i], buf, envs[i].seed, r)
            else:
                st[i], ep[i], last = oppo.rollout(th[ver], shape, envs[i], st[i], ep[i], buf, envs[i].seed, r)
            slabs[(i, r)] = (buf, last)
            nxt[i] += 1
        elif ev[0] == "drop":
            i, r, _ = ev[1]
            del slabs[(i, r)]
        else:
            _, k, took = ev
            assert k == len(th) - 1
            S = len(took)
            buf = oppo.new_buffer(horizon, S * n_envs, cfg.obs_dim, cfg.act_dim)
            last = np.zeros(S * n_envs, np.float32)
            for j, (i, r, _) in enumerate(took):
                sb, sl = slabs.pop((i, r))
                for name in ("obs", "act", "logp", "val", "rew", "done"):
                    buf[name][:, j * n_envs:(j + 1) * n_envs] = sb[name]
                last[j * n_envs:(j + 1) * n_envs] = sl
            buf["adv"], buf["ret"] = oppo.gae(buf["rew"], buf["val"], buf["done"], last, cfg.gamma, cfg.lam, True)
            new_th, m, v, kk, _ = oppo.ppo_update(th[k], m, v, kk, shape, buf, hp, cfg.seed, k)
            th.append(new_th)
    return th, sum(nxt)


@pytest.mark.parametrize("on_full,masked", [("block", False), ("drop_oldest", False), ("block", True)])
def test_async_fp32_trace_replays_to_the_same_parameters(on_full, masked):
    cfg = syn.get_config("C1")
    n_agents, n_envs, horizon, slabs, updates = 3, 32, 8, 2, 4
    minibatch = slabs * n_envs * horizon // 2
    pipe, theta, envs, states = _make(cfg, "f32", n_agents, n_envs, horizon, minibatch, slabs, 4, on_full, masked)
    args = dict(gamma=cfg.gamma, lam=cfg.lam, epochs=2, minibatch=minibatch, clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e,
                lr=cfg.lr)
    rates = pipe.run(updates, **args)
    assert rates["updates"] == updates
    trace = list(pipe.trace)
    kinds = [e[0] for e in trace]
    assert kinds.count("update") == updates
    # every update consumed the oldest waiting slabs, in the order they entered the ring
    waiting = []
    for e in trace:
        if e[0] == "push":
            waiting.append(e[1])
        elif e[0] == "drop":
            assert waiting.pop(0) == e[1]
        else:
            assert list(e[2]) == waiting[:slabs]
            del waiting[:slabs]
    # parameter versions never run ahead of the updates done when the round entered the ring
    done = 0
    for e in trace:
        if e[0] == "update":
            done += 1
        elif e[0] == "push":
            assert 0 <= e[1][2] <= done
    hp = oppo.PPOHyper(clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, lr=cfg.lr, epochs=2, minibatch=minibatch)
    th, n_rounds = _replay(trace, cfg, theta, envs, states, n_envs, horizon, hp)
    assert len(th) == updates + 1
    got = pipe.theta.cpu().numpy()
    assert rel_l2(got, th[-1]) <= 2e-5, rel_l2(got, th[-1])
    assert rel_l2(got - theta, th[-1] - theta) <= 1e-3
    assert rates["rounds_collected"] >= n_rounds >= updates * slabs
    if on_full == "block":
        assert rates["slabs_discarded"] == 0
    assert rates["pps_env_steps_per_s"] > 0 and rates["ttop_samples_per_s"] > 0
    pipe.close()


def test_async_bf16_bounded_rounds_replay():
    """bf16 model through the one-launch collection; the agents stop after a fixed number of rounds, the trainer
    consumes what the ring can feed.  Same bounds as the lag-1 schedule's replay test."""
    cfg = syn.get_config("C3")
    n_agents, n_envs, horizon, slabs = 4, 128, 4, 4
    minibatch = 1024
    pipe, theta, envs, states = _make(cfg, "bf16", n_agents, n_envs, horizon, minibatch, slabs, 8, "block")
    args = dict(gamma=cfg.gamma, lam=cfg.lam, epochs=2, minibatch=minibatch, clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e,
                lr=2e-3)
    rates = pipe.run(3, max_rounds=3, **args)
    assert rates["updates"] == 3 and rates["rounds_collected"] == 12
    hp = oppo.PPOHyper(clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, lr=2e-3, epochs=2, minibatch=minibatch)
    th, _ = _replay(list(pipe.trace), cfg, theta, envs, states, n_envs, horizon, hp)
    got = pipe.theta.cpu().numpy()
    assert rel_l2(got, th[-1]) <= 2e-2
    assert rel_l2(got - theta, th[-1] - theta) <= 0.25, rel_l2(got - theta, th[-1] - theta)
    pipe.close()


def test_async_fp8_agents_bf16_trainer_replay():
    """Agents that serve in fp8 (weights re-quantised from every parameter version they take) feeding a bf16
    trainer: the trace replayed with the oracle's fp8 agent and fp32 trainer, bounds of the bf16 trainer."""
    cfg = syn.get_config("C3")
    n_agents, n_envs, horizon, slabs = 2, 128, 4, 2
    minibatch = 512
    pipe, theta, envs, states = _make(cfg, "bf16", n_agents, n_envs, horizon, minibatch, slabs, 4, "block",
                                      agent_precision="fp8")
    args = dict(gamma=cfg.gamma, lam=cfg.lam, epochs=2, minibatch=minibatch, clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e,
                lr=2e-3)
    rates = pipe.run(3, max_rounds=3, **args)
    assert rates["updates"] == 3 and rates["rounds_collected"] == 6
    hp = oppo.PPOHyper(clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, lr=2e-3, epochs=2, minibatch=minibatch)
    th, _ = _replay(list(pipe.trace), cfg, theta, envs, states, n_envs, horizon, hp, fp8=True)
    got = pipe.theta.cpu().numpy()
    assert rel_l2(got, th[-1]) <= 2e-2
    assert rel_l2(got - theta, th[-1] - theta) <= 0.25, rel_l2(got - theta, th[-1] - theta)
    pipe.close()
    # the agents really serve in fp8: one round of one agent of a fresh pipeline under theta_0 (no training yet, so the
    # parameters are exactly the oracle's) follows the fp8 oracle and is E4M3's 5-9 % away from the exact network
    pipe, theta, envs, states = _make(cfg, "bf16", n_agents, n_envs, horizon, minibatch, slabs, 4, "block",
                                      agent_precision="fp8")
    ag = pipe.agents[0]
    assert pipe._take_newest(ag) == 0
    pipe._collect(ag, 0)
    pipe.sync_all()
    shape = oppo.ModelShape(cfg.obs_dim, cfg.act_dim, tuple(cfg.hidden))
    val0 = ag.rb.to_numpy()["val"][0]
    v8 = f8.agent_forward(theta, shape, states[0])[1]
    vx = oppo.value_only(theta, shape, states[0])
    assert rel_l2(val0, v8) <= 2e-2, rel_l2(val0, v8)
    assert rel_l2(val0, vx) > 4e-2, rel_l2(val0, vx)
    pipe.close()
