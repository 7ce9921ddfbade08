"""Auxiliary guarantees of the hot path on the GPU: a run resumed from a snapshot of its state continues bit for
bit, and a hand-off between instances leaves no element of the receiver's batch unwritten (the batch is poisoned
with NaN before every round)."""
import numpy as np
import pytest
import torch

from oracle import ppo as oppo
from workloads import synthetic as syn
from gpu_util import make_session, oracle_pieces

pytestmark = pytest.mark.gpu


def _iterate(ses, cfg, it, minibatch):
    ses.rollout(it)
    ses.gae(cfg.gamma, cfg.lam, True)
    ses.update(it, epochs=2, minibatch=minibatch, clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, lr=cfg.lr)
    ses.sync()


@pytest.mark.parametrize("name,dtype,n_envs,horizon", [("C1", "f32", 64, 8), ("C2", "bf16", 512, 4), ("C4", "bf16", 384, 3)])
def test_resume_from_a_snapshot_continues_bit_for_bit(name, dtype, n_envs, horizon):
    """Three iterations in one session against two iterations, a snapshot of everything the method carries
    (parameters, Adam moments and step count, env states, episode counters) and a third iteration in a NEW session
    built from the snapshot: parameters, moments, states and the third round's experience are identical."""
    import paper_2206_08482_amd as g
    cfg = syn.get_config(name)
    shape, theta, env, state0, hp = oracle_pieces(cfg, n_envs=n_envs)
    mb = n_envs * horizon // 2
    a = make_session(cfg, theta, env, state0, n_envs=n_envs, minibatch=mb, horizon=horizon, dtype=dtype)
    for it in range(2):
        _iterate(a, cfg, it, mb)
    snap = dict(theta=a.theta.cpu().numpy().copy(), m=a.adam_m.clone(), v=a.adam_v.clone(), steps=a.adam_steps,
                state=a.state().cpu().numpy().copy(), ep=a.episode_step.clone())
    _iterate(a, cfg, 2, mb)
    b = make_session(cfg, snap["theta"], env, snap["state"], n_envs=n_envs, minibatch=mb, horizon=horizon, dtype=dtype)
    b.adam_m.copy_(snap["m"]); b.adam_v.copy_(snap["v"]); b.episode_step.copy_(snap["ep"])
    b.adam_steps = snap["steps"]
    torch.cuda.synchronize()
    g.gmi_wait_stream(b.gmi)
    _iterate(b, cfg, 2, mb)
    assert torch.equal(a.theta, b.theta) and torch.equal(a.adam_m, b.adam_m) and torch.equal(a.adam_v, b.adam_v)
    assert torch.equal(a.state(), b.state()) and torch.equal(a.episode_step, b.episode_step)
    ga, gb = a.buf.to_numpy(), b.buf.to_numpy()
    for k in ("obs", "act", "logp", "val", "rew", "done", "adv", "ret"):
        assert np.array_equal(ga[k], gb[k]), k
    assert not torch.equal(a.theta, torch.tensor(snap["theta"], device="cuda"))      # the third iteration did train
    a.close()
    b.close()


@pytest.mark.parametrize("through_channels", [False, True])
def test_hand_off_overwrites_every_element_of_a_poisoned_batch(through_channels):
    """Agents on masked instances hand their rounds to the trainer (directly into column slices, or through the
    channels); before every round all experience arrays of the trainer's batch are filled with NaN.  After the
    round's update nothing in the batch or the parameters is NaN: every element was written before it was read."""
    import paper_2206_08482_amd as g
    from paper_2206_08482_amd.channels import ChannelPipeline
    from paper_2206_08482_amd.instances import InstancePipeline, cu_masks
    cfg = syn.get_config("C3")
    n_agents, n_envs, horizon, minibatch = 3, 100, 4, 600
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    thr = oppo.done_threshold_from_inverse(cfg.done_prob_inv)
    states = [syn.make_initial_state(n_envs, cfg.obs_dim, cfg.seed + 10 + i) for i in range(n_agents)]
    probe = g.gmi_create()
    n_cu = g.gmi_cu_count(probe)
    g.gmi_destroy(probe)
    masks = cu_masks(n_cu, [n_cu // 4 // 8 * 8] * n_agents + [n_cu // 4 // 8 * 8], "contiguous")
    cls = ChannelPipeline if through_channels else InstancePipeline
    pipe = cls(n_agents=n_agents, n_envs=n_envs, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim, hidden=cfg.hidden,
               horizon=horizon, dtype="bf16", theta=theta, a_mat=a_mat, b_mat=b_mat, state0=states,
               noise_std=cfg.noise_std, reward_scale=cfg.reward_scale, done_period=cfg.done_period,
               done_threshold=thr, seed=cfg.seed, minibatch=minibatch, agent_masks=masks[:n_agents],
               trainer_mask=masks[n_agents])
    args = dict(gamma=cfg.gamma, lam=cfg.lam, epochs=1, minibatch=minibatch, clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e,
                lr=cfg.lr)
    for k in range(3):
        for rb in pipe.bufs:
            for name in ("obs", "act", "logp", "val", "rew", "adv", "ret"):
                getattr(rb, name).fill_(float("nan"))
        for lv in pipe.last_value:
            lv.fill_(float("nan"))
        torch.cuda.synchronize()
        pipe.iteration_sync(k, **args)
        pipe.sync_all()
        got = pipe.bufs[0].to_numpy()
        for name in ("obs", "act", "logp", "val", "rew", "adv", "ret"):
            assert np.isfinite(got[name]).all(), (k, name)
        assert torch.isfinite(pipe.last_value[0]).all() and torch.isfinite(pipe.theta).all()
    pipe.close()
