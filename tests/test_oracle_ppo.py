"""Pins for oracle.ppo: closed forms, brute force, finite differences and independent libraries
(PyTorch CPU autograd / optim / distributions in float64)."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import philox as px
from oracle import ppo
from workloads import synthetic as syn

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
F64 = np.float64


# ------------------------------------------------------------------ model shapes
def test_param_counts_match_the_papers_table():
    for line in open(os.path.join(GOLDEN, "policy_param_counts.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        _, shape_s, printed = line.split()
        dims = [int(x) for x in shape_s.split(":")]
        shape = ppo.ModelShape(dims[0], dims[-1], tuple(dims[1:-1]))
        n = shape.n_params()
        assert n == syn.param_count(dims[0], dims[-1], dims[1:-1])
        # printed with two significant digits
        assert abs(n - float(printed)) / float(printed) < 0.05
    assert ppo.ModelShape(8, 2, (32, 32)).n_params() == 2789


def test_unpack_layout():
    shape = ppo.ModelShape(3, 2, (4,))
    theta = np.arange(shape.n_params(), dtype=np.float64)
    pol, val, log_std = ppo.unpack(theta, shape)
    assert pol[0][0].shape == (4, 3) and pol[0][0][1, 0] == 3          # W[out,in] row-major
    assert pol[0][1][0] == 12 and pol[1][0].shape == (2, 4)
    assert val[1][0].shape == (1, 4) and log_std.shape == (2,)
    assert log_std[-1] == theta[-1]


# ------------------------------------------------------------------ torch re-statement of the loss
def _torch_loss(theta_t, shape, obs, act, logp_old, adv, ret, hp):
    off = 0
    outs = []
    for out_dim in (shape.act_dim, 1):
        h = obs
        dims = shape.layer_dims(out_dim)
        for li, (i, o) in enumerate(dims):
            w = theta_t[off:off + i * o].view(o, i); off += i * o
            b = theta_t[off:off + o]; off += o
            h = torch.nn.functional.linear(h, w, b)
            if li < len(dims) - 1:
                h = torch.nn.functional.elu(h)
        outs.append(h)
    log_std = theta_t[off:off + shape.act_dim]
    mu, v = outs[0], outs[1][:, 0]
    dist = torch.distributions.Normal(mu, log_std.exp())
    logp = dist.log_prob(act).sum(-1)
    ratio = (logp - logp_old).exp()
    l_pi = -torch.min(ratio * adv, torch.clamp(ratio, 1 - hp.clip, 1 + hp.clip) * adv).mean()
    l_v = torch.nn.functional.mse_loss(v, ret)
    ent = dist.entropy().sum(-1).mean()
    return l_pi + hp.c_v * l_v - hp.c_e * ent, (l_pi, l_v, ent, logp)


def _random_minibatch(shape, m, seed, spread=0.3):
    rng = np.random.default_rng(seed)
    theta = syn.make_model_params(shape.obs_dim, shape.act_dim, shape.hidden, seed,
                                  policy_head_scale=1.0).astype(F64)
    theta[-shape.act_dim:] = 0.2 * rng.standard_normal(shape.act_dim)
    obs = rng.standard_normal((m, shape.obs_dim))
    act = rng.standard_normal((m, shape.act_dim))
    # logp_old near the current logp so that ratios straddle the clip range
    st, _ = ppo.ppo_loss_and_grad(theta, shape, obs, act, np.zeros(m), np.zeros(m), np.zeros(m),
                                  ppo.PPOHyper(), F64, want_grad=False)
    pol, _, log_std = ppo.unpack(theta, shape)
    mu, _ = ppo.mlp_forward(obs, pol)
    z = (act - mu) * np.exp(-log_std)
    logp = (-0.5 * z * z - log_std - 0.5 * ppo.LOG_2PI).sum(1)
    logp_old = logp + spread * rng.standard_normal(m)
    adv = rng.standard_normal(m)
    ret = rng.standard_normal(m)
    return theta, obs, act, logp_old, adv, ret


@pytest.mark.parametrize("dims", [(8, 2, (32, 32)), (5, 3, (7,)), (13, 4, (17, 9, 6))])
def test_loss_and_gradient_match_torch_autograd(dims):
    shape = ppo.ModelShape(*dims)
    hp = ppo.PPOHyper(clip=0.2, c_v=0.5, c_e=0.01)
    theta, obs, act, logp_old, adv, ret = _random_minibatch(shape, 50, seed=4)
    stats, grad = ppo.ppo_loss_and_grad(theta, shape, obs, act, logp_old, adv, ret, hp, F64)
    tt = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    loss, (l_pi, l_v, ent, logp) = _torch_loss(tt, shape, *[torch.tensor(a) for a in
                                                            (obs, act, logp_old, adv, ret)], hp)
    loss.backward()
    assert abs(stats[0] - l_pi.item()) < 1e-12
    assert abs(stats[1] - l_v.item()) < 1e-12
    assert abs(stats[2] - ent.item()) < 1e-12
    assert abs(ppo.total_loss(stats, hp) - loss.item()) < 1e-12
    assert abs(stats[3] - (torch.tensor(logp_old) - logp).mean().item()) < 1e-12
    ratio = np.exp(logp.detach().numpy() - logp_old)
    assert 0.05 < stats[4] < 0.95 and abs(stats[4] - (np.abs(ratio - 1) > 0.2).mean()) < 1e-12
    g_ref = tt.grad.numpy()
    assert np.abs(grad - g_ref).max() < 1e-12 * (1 + np.abs(g_ref).max())
    assert np.abs(g_ref).max() > 1e-3


def test_gradient_matches_central_finite_differences_on_c1():
    cfg = syn.get_config("C1")
    shape = ppo.ModelShape(cfg.obs_dim, cfg.act_dim, cfg.hidden)
    hp = ppo.PPOHyper(c_e=0.01)
    theta, obs, act, logp_old, adv, ret = _random_minibatch(shape, 32, seed=5, spread=0.05)
    _, grad = ppo.ppo_loss_and_grad(theta, shape, obs, act, logp_old, adv, ret, hp, F64)
    rng = np.random.default_rng(0)
    # every parameter tensor is sampled: walk the layout and take a few entries of each
    idx, off = [], 0
    for out_dim in (shape.act_dim, 1):
        for i, o in shape.layer_dims(out_dim):
            idx += list(off + rng.choice(i * o, 6, replace=False)); off += i * o
            idx += list(off + rng.choice(o, min(o, 3), replace=False)); off += o
    idx += list(range(off, off + shape.act_dim))
    h = 1e-5
    for p in idx:
        tp, tm = theta.copy(), theta.copy()
        tp[p] += h
        tm[p] -= h
        lp = ppo.total_loss(ppo.ppo_loss_and_grad(tp, shape, obs, act, logp_old, adv, ret, hp, F64,
                                                  False)[0], hp)
        lm = ppo.total_loss(ppo.ppo_loss_and_grad(tm, shape, obs, act, logp_old, adv, ret, hp, F64,
                                                  False)[0], hp)
        fd = (lp - lm) / (2 * h)
        assert abs(fd - grad[p]) < 1e-7 + 1e-5 * abs(fd), (p, fd, grad[p])


def test_elu_and_its_derivative_at_zero():
    z = np.array([-1e-9, 0.0, 1e-9, -30.0, 2.0])
    h = ppo.elu(z)
    assert np.allclose(h, [np.expm1(-1e-9), 0.0, 1e-9, -1.0, 2.0], atol=1e-15)
    # derivative through the output: continuous across 0
    d = np.where(h > 0, 1.0, h + 1)
    assert abs(d[0] - 1) < 1e-8 and d[1] == 1 and d[2] == 1 and d[3] < 1e-12


# ------------------------------------------------------------------ Gaussian log-prob / entropy
def test_logprob_and_entropy_closed_forms():
    shape = ppo.ModelShape(6, 3, (5,))
    theta = syn.make_model_params(6, 3, (5,), 1).astype(F64)
    theta[-3:] = [0.3, -0.2, 0.1]
    obs = np.random.default_rng(0).standard_normal((40, 6))
    act, logp, val, mu = ppo.agent_act(theta, shape, obs, seed=1, step=0, dtype=F64)
    ref = torch.distributions.Normal(torch.tensor(mu), torch.tensor(theta[-3:]).exp()) \
        .log_prob(torch.tensor(act)).sum(-1).numpy()
    assert np.abs(logp - ref).max() < 1e-12
    # at a = mu the density is -sum(log_std) - A/2 ln(2 pi)
    hp = ppo.PPOHyper()
    st, _ = ppo.ppo_loss_and_grad(theta, shape, obs, mu, np.zeros(40), np.ones(40), np.zeros(40),
                                  hp, F64, False)
    assert abs(-st[3] - (-theta[-3:].sum() - 1.5 * math.log(2 * math.pi))) < 1e-12
    # entropy at sigma = 1 is A/2 (1 + ln 2 pi)
    theta[-3:] = 0
    st, _ = ppo.ppo_loss_and_grad(theta, shape, obs, mu, np.zeros(40), np.ones(40), np.zeros(40),
                                  hp, F64, False)
    assert abs(st[2] - 1.5 * (1 + math.log(2 * math.pi))) < 1e-12


def test_agent_act_uses_the_documented_noise():
    shape = ppo.ModelShape(6, 3, (5,))
    theta = syn.make_model_params(6, 3, (5,), 1)
    theta[-3:] = [0.3, -0.2, 0.1]
    obs = syn.make_initial_state(10, 6, 0)
    act, logp, val, mu = ppo.agent_act(theta, shape, obs, seed=77, step=5)
    eps = px.normal_field(77, px.STREAM_ACTION, 5, 10, 3)
    assert np.allclose(act, mu + np.exp(theta[-3:]) * eps, rtol=1e-6, atol=1e-7)
    assert act.dtype == np.float32 and logp.dtype == np.float32 and val.dtype == np.float32
    assert np.allclose(val, ppo.value_only(theta, shape, obs))


# ------------------------------------------------------------------ GAE
def _gae_brute(rew, val, done, last_val, gamma, lam):
    T, N = rew.shape
    vnext = np.concatenate([val[1:], last_val[None]], 0)
    nd = 1.0 - done
    delta = rew + gamma * vnext * nd - val
    adv = np.zeros((T, N))
    for t in range(T):
        for l in range(T - t):
            w = (gamma * lam) ** l
            for j in range(t, t + l):
                w = w * nd[j]
            adv[t] += w * delta[t + l]
    return adv


def test_gae_matches_brute_force_sum():
    b = syn.make_rollout_batch(8, 13, 3, 2, seed=2, done_prob=0.2)
    adv, ret = ppo.gae(b["rew"], b["val"], b["done"], b["last_val"], 0.97, 0.9, False, F64)
    ref = _gae_brute(b["rew"].astype(F64), b["val"].astype(F64), b["done"].astype(F64),
                     b["last_val"].astype(F64), 0.97, 0.9)
    assert b["done"].sum() > 5
    assert np.abs(adv - ref).max() < 1e-12
    assert np.abs(ret - (ref + b["val"])).max() < 1e-12


def test_gae_special_cases():
    T, N = 7, 5
    b = syn.make_rollout_batch(T, N, 3, 2, seed=3, done_prob=0.3)
    rew, val, lastv = b["rew"].astype(F64), b["val"].astype(F64), b["last_val"].astype(F64)
    done = b["done"]
    nodone = np.zeros_like(done)
    vnext = np.concatenate([val[1:], lastv[None]], 0)
    g = 0.9
    # lambda = 0: one-step TD error
    adv, _ = ppo.gae(rew, val, done, lastv, g, 0.0, False, F64)
    assert np.abs(adv - (rew + g * vnext * (1 - done) - val)).max() < 1e-13
    # lambda = 1, no dones: discounted return + bootstrap - value
    adv, ret = ppo.gae(rew, val, nodone, lastv, g, 1.0, False, F64)
    for t in range(T):
        mc = sum(g ** l * rew[t + l] for l in range(T - t)) + g ** (T - t) * lastv
        assert np.abs(adv[t] - (mc - val[t])).max() < 1e-12
        assert np.abs(ret[t] - mc).max() < 1e-12
    # gamma = 0, or done at every step: A = r - v
    adv, _ = ppo.gae(rew, val, done, lastv, 0.0, 0.7, False, F64)
    assert np.abs(adv - (rew - val)).max() < 1e-13
    adv, _ = ppo.gae(rew, val, np.ones_like(done), lastv, g, 0.7, False, F64)
    assert np.abs(adv - (rew - val)).max() < 1e-13
    # r = 1, v = 0, lambda = 1: geometric series
    adv, _ = ppo.gae(np.ones((T, N)), np.zeros((T, N)), nodone, np.zeros(N), g, 1.0, False, F64)
    for t in range(T):
        assert np.abs(adv[t] - (1 - g ** (T - t)) / (1 - g)).max() < 1e-12
    # episode ends exactly at the horizon (periodic done with period T): no dependence on v_T
    last = np.zeros_like(done)
    last[-1] = 1
    a1, _ = ppo.gae(rew, val, last, lastv, g, 0.95, False, F64)
    a2, _ = ppo.gae(rew, val, last, lastv + 100.0, g, 0.95, False, F64)
    assert np.array_equal(a1, a2)


def test_gae_normalisation():
    b = syn.make_rollout_batch(6, 11, 3, 2, seed=4)
    raw, ret0 = ppo.gae(b["rew"], b["val"], b["done"], b["last_val"], 0.99, 0.95, False, F64)
    adv, ret = ppo.gae(b["rew"], b["val"], b["done"], b["last_val"], 0.99, 0.95, True, F64)
    assert abs(adv.mean()) < 1e-12 and abs(adv.std() - 1) < 1e-6
    assert np.array_equal(ret, ret0)                      # returns use the raw advantage
    assert np.allclose(adv, (raw - raw.mean()) / (np.sqrt(((raw - raw.mean()) ** 2).mean()) + 1e-8),
                       atol=1e-12)
    a32, r32 = ppo.gae(b["rew"], b["val"], b["done"], b["last_val"], 0.99, 0.95, True, np.float32)
    assert a32.dtype == np.float32 and np.abs(a32 - adv).max() < 1e-5


# ------------------------------------------------------------------ clipped surrogate
def _vanilla_policy_gradient(theta, shape, obs, act, adv):
    """-mean(A * dlogp/dtheta) by autograd of the plain log-density."""
    tt = torch.tensor(theta, requires_grad=True)
    hp = ppo.PPOHyper(c_v=0.0)
    off, h = 0, torch.tensor(obs)
    dims = shape.layer_dims(shape.act_dim)
    for li, (i, o) in enumerate(dims):
        w = tt[off:off + i * o].view(o, i); off += i * o
        b = tt[off:off + o]; off += o
        h = h @ w.T + b
        if li < len(dims) - 1:
            h = torch.where(h > 0, h, torch.expm1(h))
    log_std = tt[-shape.act_dim:]
    a = torch.tensor(act)
    logp = (-0.5 * ((a - h) / log_std.exp()) ** 2 - log_std - 0.5 * math.log(2 * math.pi)).sum(-1)
    (-(torch.tensor(adv) * logp).mean()).backward()
    return tt.grad.numpy(), logp.detach().numpy()


def test_ratio_one_gives_vanilla_policy_gradient():
    shape = ppo.ModelShape(7, 3, (9, 6))
    theta, obs, act, _, adv, ret = _random_minibatch(shape, 64, seed=6)
    g_ref, logp = _vanilla_policy_gradient(theta, shape, obs, act, adv)
    hp = ppo.PPOHyper(c_v=0.0, c_e=0.0)
    stats, grad = ppo.ppo_loss_and_grad(theta, shape, obs, act, logp, adv, ret, hp, F64)
    assert abs(stats[3]) < 1e-14 and stats[4] == 0                 # KL 0, nothing clipped
    assert abs(stats[0] + adv.mean()) < 1e-13                      # L_pi = -mean(A)
    assert np.abs(grad - g_ref).max() < 1e-12
    # with normalised advantages the policy loss itself is 0 at theta_old
    adv_n = (adv - adv.mean()) / adv.std()
    stats, _ = ppo.ppo_loss_and_grad(theta, shape, obs, act, logp, adv_n, ret, hp, F64)
    assert abs(stats[0]) < 1e-13


def test_clipping_sign_cases():
    shape = ppo.ModelShape(4, 2, (5,))
    theta, obs, act, _, _, _ = _random_minibatch(shape, 8, seed=7)
    _, logp = _vanilla_policy_gradient(theta, shape, obs, act, np.ones(8))
    hp = ppo.PPOHyper(clip=0.2, c_v=0.0)
    n_pol = sum(i * o + o for i, o in shape.layer_dims(shape.act_dim))

    def pol_grad(shift, adv_sign):
        lo = logp - shift                                            # ratio = exp(shift)
        _, g = ppo.ppo_loss_and_grad(theta, shape, obs, act, lo, adv_sign * np.ones(8),
                                     np.zeros(8), hp, F64)
        return np.concatenate([g[:n_pol], g[-shape.act_dim:]])

    up, down = math.log(1.5), math.log(0.5)
    assert np.abs(pol_grad(up, +1)).max() == 0                      # A>0, ratio>1+c : clipped
    assert np.abs(pol_grad(down, -1)).max() == 0                    # A<0, ratio<1-c : clipped
    assert np.abs(pol_grad(down, +1)).max() > 1e-4                  # A>0, ratio<1-c : unclipped
    assert np.abs(pol_grad(up, -1)).max() > 1e-4                    # A<0, ratio>1+c : unclipped
    g_ref, _ = _vanilla_policy_gradient(theta, shape, obs, act, 0.5 * np.ones(8))
    g_ref = np.concatenate([g_ref[:n_pol], g_ref[-shape.act_dim:]])
    assert np.abs(pol_grad(down, +1) - g_ref).max() < 1e-12         # = ratio * vanilla gradient


# ------------------------------------------------------------------ Adam
def test_adam_first_step_and_constant_gradient():
    hp = ppo.PPOHyper(lr=1e-2)
    g = np.array([0.3, -2.0, 1e-3, 5.0])
    th, m, v = ppo.adam_step(np.zeros(4), np.zeros(4), np.zeros(4), g, 1, hp, F64)
    assert np.abs(th - (-hp.lr * g / (np.abs(g) + hp.adam_eps))).max() < 1e-12
    for k in range(2, 200):
        th_prev = th
        th, m, v = ppo.adam_step(th, m, v, g, k, hp, F64)
    assert np.abs((th - th_prev) - (-hp.lr * np.sign(g))).max() < 1e-6


def test_adam_matches_torch_optim():
    rng = np.random.default_rng(0)
    hp = ppo.PPOHyper(lr=3e-3, beta1=0.8, beta2=0.95, adam_eps=1e-6)
    p = torch.tensor(rng.standard_normal(50), requires_grad=True)
    opt = torch.optim.Adam([p], lr=hp.lr, betas=(hp.beta1, hp.beta2), eps=hp.adam_eps)
    th, m, v = p.detach().numpy().copy(), np.zeros(50), np.zeros(50)
    for k in range(1, 8):
        g = rng.standard_normal(50)
        p.grad = torch.tensor(g)
        opt.step()
        th, m, v = ppo.adam_step(th, m, v, g, k, hp, F64)
        assert np.abs(th - p.detach().numpy()).max() < 1e-12


# ------------------------------------------------------------------ environment
def _env(o, a, period=0, prob_inv=0, noise=0.0, seed=0, scale=1.0):
    am, bm = syn.make_env_matrices(o, a, seed)
    return ppo.EnvSpec(am, bm, noise, scale, period, ppo.done_threshold_from_inverse(prob_inv), seed)


def test_env_without_noise_is_a_matrix_power():
    env = _env(6, 2)
    s0 = syn.make_initial_state(9, 6, 1).astype(F64)
    s, ep = s0, np.zeros(9, np.uint32)
    for t in range(12):
        s, r, d, ep = ppo.env_step(env, s, np.zeros((9, 2)), ep, t, F64)
        assert d.sum() == 0
    ref = s0 @ np.linalg.matrix_power(env.a_mat.astype(F64), 12).T
    assert np.abs(s - ref).max() < 1e-12
    assert np.array_equal(ep, np.full(9, 12, np.uint32))


def test_env_reward_and_input_matrix():
    env = _env(6, 2, scale=0.01)
    rng = np.random.default_rng(3)
    s, a = rng.standard_normal((5, 6)), rng.standard_normal((5, 2))
    nxt, r, d, _ = ppo.env_step(env, s, a, np.zeros(5, np.uint32), 0, F64)
    for e in range(5):
        assert abs(r[e] - 0.01 * (-(s[e] ** 2).sum() - 0.01 * (a[e] ** 2).sum())) < 1e-14
        ref = env.a_mat.astype(F64) @ s[e] + env.b_mat.astype(F64) @ a[e]
        assert np.abs(nxt[e] - ref).max() < 1e-13
    # A = 0.95 I exactly: discounted return of the zero-action policy is a geometric series
    env2 = ppo.EnvSpec(0.95 * np.eye(6), np.zeros((6, 2)), 0.0, 1.0, 0, 0, 0)
    st, ep, ret = s.copy(), np.zeros(5, np.uint32), np.zeros(5)
    gam = 0.9
    for t in range(400):
        st, r, _, ep = ppo.env_step(env2, st, np.zeros((5, 2)), ep, t, F64)
        ret += gam ** t * r
    assert np.abs(ret - (-(s ** 2).sum(1) / (1 - gam * 0.9025))).max() < 1e-9


def test_env_noise_and_periodic_done_and_reset():
    env = _env(6, 2, period=4, noise=0.01, seed=5)
    s = syn.make_initial_state(7, 6, 1)
    ep = np.array([0, 1, 2, 3, 0, 1, 2], np.uint32)
    nxt, r, d, ep2 = ppo.env_step(env, s, np.zeros((7, 2), np.float32), ep, 9)
    assert list(d) == [0, 0, 0, 1, 0, 0, 0]
    assert list(ep2) == [1, 2, 3, 0, 1, 2, 3]
    xi = px.normal_field(5, px.STREAM_ENV, 9, 7, 6)
    reset = px.normal_field(5, px.STREAM_RESET, 9, 7, 6)
    det = s @ env.a_mat.T
    assert np.allclose(nxt[:3], det[:3] + 0.01 * xi[:3], rtol=1e-6, atol=1e-7)
    assert np.array_equal(nxt[3], reset[3])
    assert nxt.dtype == np.float32 and r.dtype == np.float32 and d.dtype == np.uint8
    # periodicity over a longer run: done exactly every 4th step for an env starting at 0
    ep, dones = np.zeros(1, np.uint32), []
    st = s[:1]
    for t in range(12):
        st, _, dd, ep = ppo.env_step(env, st, np.zeros((1, 2), np.float32), ep, t)
        dones.append(int(dd[0]))
    assert dones == [0, 0, 0, 1] * 3


def test_env_bernoulli_done_uses_the_integer_threshold():
    env = _env(4, 1, prob_inv=10, seed=8)
    n = 20000
    s = np.zeros((n, 4), np.float32)
    _, _, d, ep = ppo.env_step(env, s, np.zeros((n, 1), np.float32), np.full(n, 5, np.uint32), 3)
    w = px.done_words(8, 3, n)
    assert np.array_equal(d.astype(bool), w < np.uint32((1 << 32) // 10))
    assert abs(d.mean() - 0.1) < 4 * math.sqrt(0.09 / n)
    assert np.array_equal(ep, np.where(d, 0, 6))


# ------------------------------------------------------------------ update loop and whole step
def test_ppo_update_visits_every_sample_once_per_epoch_and_counts_steps():
    cfg = syn.get_config("C1")
    shape = ppo.ModelShape(cfg.obs_dim, cfg.act_dim, cfg.hidden)
    b = syn.make_rollout_batch(cfg.horizon, cfg.n_envs, cfg.obs_dim, cfg.act_dim, seed=1)
    b["adv"], b["ret"] = ppo.gae(b["rew"], b["val"], b["done"], b["last_val"], 0.99, 0.95, True)
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, 0)
    hp = ppo.PPOHyper(epochs=2, minibatch=256)
    z = np.zeros_like(theta)
    th, m, v, k, stats = ppo.ppo_update(theta, z, z, 3, shape, b, hp, seed=0, iteration=0)
    assert k == 3 + 2 * 4 and stats.shape == (8, 5)
    assert th.dtype == np.float32 and np.isfinite(th).all() and not np.array_equal(th, theta)
    # first minibatch reproduces a hand-made call
    flat = ppo.flatten_buffer(b)
    idx = px.feistel_permutation(1024, 0, 0, 0)[:256]
    st, g = ppo.ppo_loss_and_grad(theta, shape, flat["obs"][idx], flat["act"][idx],
                                  flat["logp"][idx], flat["adv"][idx], flat["ret"][idx], hp)
    assert np.array_equal(st, stats[0])
    # sample index = t*N + env
    assert np.array_equal(flat["obs"][5 * cfg.n_envs + 7], b["obs"][5, 7])


def test_whole_iteration_on_c1_is_deterministic_and_learns_something():
    cfg = syn.get_config("C1")
    shape = ppo.ModelShape(cfg.obs_dim, cfg.act_dim, cfg.hidden)
    am, bm = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, cfg.seed)
    env = ppo.EnvSpec(am, bm, cfg.noise_std, cfg.reward_scale, cfg.done_period, 0, cfg.seed)
    hp = ppo.PPOHyper(epochs=cfg.epochs, minibatch=cfg.minibatch)
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    s0 = syn.make_initial_state(cfg.n_envs, cfg.obs_dim, cfg.seed)
    z = np.zeros_like(theta)
    out1 = ppo.ppo_iteration(theta, z, z, 0, shape, env, s0, np.zeros(cfg.n_envs, np.uint32),
                             cfg.horizon, hp, cfg.gamma, cfg.lam, cfg.seed, 0)
    out2 = ppo.ppo_iteration(theta, z, z, 0, shape, env, s0, np.zeros(cfg.n_envs, np.uint32),
                             cfg.horizon, hp, cfg.gamma, cfg.lam, cfg.seed, 0)
    assert np.array_equal(out1["theta"], out2["theta"])
    buf = out1["buf"]
    assert buf["done"][-1].all() and not buf["done"][:-1].any()      # done every 16 steps
    assert np.array_equal(buf["obs"][0], s0)
    # the stored log-prob is the density of the stored action under the stored policy
    st, _ = ppo.ppo_loss_and_grad(theta, shape, buf["obs"][3], buf["act"][3], buf["logp"][3],
                                  np.ones(cfg.n_envs), np.zeros(cfg.n_envs), hp, want_grad=False)
    assert abs(st[3]) < 1e-5 and st[4] == 0
    # value loss goes down over the four minibatch steps of one epoch on average
    assert out1["k"] == 4 and out1["stats"].shape == (4, 5)
    assert np.isfinite(out1["stats"]).all()


# ----------------------------------------------------------------------------- several trainer instances
def test_rollout_bootstraps_from_the_state_after_the_last_step():
    """Stage (i) of Section 5.1 ends with the value of the state the last interaction led to.  On an env
    without done flags the T rounds are replayed by hand with agent_act / env_step; `rollout` must return the
    value net's output on the state AFTER round T - 1 (not the one stored in the buffer's last slot), and the
    advantages must depend on it."""
    shape = ppo.ModelShape(5, 2, (7, 6))
    theta = syn.make_model_params(5, 2, (7, 6), 4)
    am, bm_ = syn.make_env_matrices(5, 2, 4)
    env = ppo.EnvSpec(am, bm_, 0.05, 1.0, 0, 0, 9)          # done_period 0, threshold 0: never done
    T, N = 6, 11
    s0 = syn.make_initial_state(N, 5, 4)
    buf = ppo.new_buffer(T, N, 5, 2)
    state, ep, last_val = ppo.rollout(theta, shape, env, s0, np.zeros(N, np.uint32), buf, seed=9, iteration=2)
    s, e = s0.astype(np.float32), np.zeros(N, np.uint32)
    for t in range(T):
        a, _, _, _ = ppo.agent_act(theta, shape, s, 9, 2 * T + t)
        assert np.array_equal(buf["obs"][t], s)
        pre = s
        s, _, d, e = ppo.env_step(env, s, a, e, 2 * T + t)
        assert not d.any()
    assert np.array_equal(state, s) and np.array_equal(ep, e)
    assert np.array_equal(last_val, ppo.value_only(theta, shape, s))
    v_pre = ppo.value_only(theta, shape, pre)                # the state stored in the last slot
    assert np.array_equal(v_pre, buf["val"][T - 1])
    assert np.abs(last_val - v_pre).max() > 1e-3              # the two candidates can be told apart
    adv1, ret1 = ppo.gae(buf["rew"], buf["val"], buf["done"], last_val, 0.99, 0.95, False)
    adv2, _ = ppo.gae(buf["rew"], buf["val"], buf["done"], v_pre, 0.99, 0.95, False)
    # with no done flag the bootstrap enters every advantage of an env: A_t changes by (gamma lam)^(T-1-t) gamma dv
    dv = (last_val - v_pre).astype(np.float64)
    for t in range(T):
        want = (0.99 * 0.95) ** (T - 1 - t) * 0.99 * dv
        assert np.allclose((adv1[t] - adv2[t]).astype(np.float64), want, rtol=1e-3, atol=1e-6)


def _random_buffer(rng, T, N, O, A):
    b = ppo.new_buffer(T, N, O, A, np.float64)
    b["obs"] = rng.standard_normal((T, N, O))
    b["act"] = rng.standard_normal((T, N, A))
    b["logp"] = -0.5 * (b["act"] ** 2).sum(-1) - A * 0.9189385332 + 0.05 * rng.standard_normal((T, N))
    b["adv"] = rng.standard_normal((T, N))
    b["ret"] = rng.standard_normal((T, N))
    return b


def test_group_update_of_one_instance_is_the_plain_update():
    rng = np.random.default_rng(11)
    shape = ppo.ModelShape(5, 2, (8, 6))
    theta = syn.make_model_params(5, 2, (8, 6), 3).astype(np.float64)
    buf = _random_buffer(rng, 4, 8, 5, 2)
    hp = ppo.PPOHyper(epochs=2, minibatch=16, c_e=0.01)
    z = np.zeros_like(theta)
    a = ppo.ppo_update(theta, z, z, 0, shape, buf, hp, 7, 3, np.float64)
    b = ppo.ppo_update_group(theta, z, z, 0, shape, [buf], hp, 7, 3, np.float64)
    for x, y in zip(a, b):
        assert np.array_equal(np.asarray(x), np.asarray(y))


def test_group_step_is_the_step_on_the_union_minibatch():
    """Mean of the instances' minibatch-mean gradients = gradient of the mean loss over the union of their
    (equally sized) slices.  With one minibatch per buffer the union is all rows of all buffers, whatever
    the shuffles: the group's single Adam step must equal the step computed by ppo_loss_and_grad on the
    concatenated rows (a wrong 1/n, a sum instead of a mean, or per-instance Adam steps all fail this)."""
    rng = np.random.default_rng(5)
    O, A = 6, 3
    shape = ppo.ModelShape(O, A, (7,))
    theta = syn.make_model_params(O, A, (7,), 1).astype(np.float64)
    bufs = [_random_buffer(rng, 2, 4, O, A) for _ in range(3)]
    hp = ppo.PPOHyper(epochs=1, minibatch=8, c_e=0.02, lr=1e-3)
    z = np.zeros_like(theta)
    th, m, v, k, stats = ppo.ppo_update_group(theta, z, z, 0, shape, bufs, hp, 21, 0, np.float64)
    assert k == 1 and stats.shape == (1, 5)
    cat = {key: np.concatenate([ppo.flatten_buffer(b)[key] for b in bufs]) for key in ("obs", "act", "logp", "adv", "ret")}
    st, g = ppo.ppo_loss_and_grad(theta, shape, cat["obs"], cat["act"], cat["logp"], cat["adv"], cat["ret"], hp,
                                  np.float64)
    th1, m1, v1 = ppo.adam_step(theta, z, z, g, 1, hp, np.float64)
    assert np.allclose(stats[0], st, rtol=1e-12, atol=1e-14)
    assert np.allclose(m, m1, rtol=1e-10, atol=1e-18) and np.allclose(v, v1, rtol=1e-10, atol=1e-30)
    assert np.allclose(th, th1, rtol=1e-12, atol=1e-15)
    assert np.abs(th - theta).max() > 1e-4
    # replicas holding identical data: the group step equals the single-instance step
    a = ppo.ppo_update_group(theta, z, z, 0, shape, [bufs[0], bufs[0]], hp, 21, 0, np.float64)
    b = ppo.ppo_update(theta, z, z, 0, shape, bufs[0], hp, 21, 0, np.float64)
    assert np.allclose(a[0], b[0], rtol=1e-12, atol=1e-15)


def test_group_instances_shuffle_with_their_own_keys():
    # two epochs of two minibatches: instance i must use the permutation of seed + i (same key for all
    # instances, or a shared permutation, changes which rows meet in a minibatch and so the result)
    rng = np.random.default_rng(9)
    O, A = 4, 2
    shape = ppo.ModelShape(O, A, (5,))
    theta = syn.make_model_params(O, A, (5,), 2).astype(np.float64)
    bufs = [_random_buffer(rng, 2, 8, O, A) for _ in range(2)]
    hp = ppo.PPOHyper(epochs=2, minibatch=8, lr=1e-3)
    z = np.zeros_like(theta)
    th, m, v, k, stats = ppo.ppo_update_group(theta, z, z, 0, shape, bufs, hp, 40, 2, np.float64)
    assert k == 4
    # replay by hand
    t2, m2, v2, kk = theta, z, z, 0
    flats = [ppo.flatten_buffer(b) for b in bufs]
    for e in range(2):
        perms = [px.feistel_permutation(16, 40 + i, 2, e) for i in range(2)]
        for j in range(2):
            gs = []
            for i in range(2):
                idx = perms[i][8 * j:8 * j + 8]
                f = flats[i]
                gs.append(ppo.ppo_loss_and_grad(t2, shape, f["obs"][idx], f["act"][idx], f["logp"][idx], f["adv"][idx],
                                                f["ret"][idx], hp, np.float64)[1])
            kk += 1
            t2, m2, v2 = ppo.adam_step(t2, m2, v2, 0.5 * (gs[0] + gs[1]), kk, hp, np.float64)
    assert np.allclose(th, t2, rtol=1e-12, atol=1e-15)
    wrong = [px.feistel_permutation(16, 40, 2, 0), px.feistel_permutation(16, 41, 2, 0)]
    assert not np.array_equal(wrong[0], wrong[1])
