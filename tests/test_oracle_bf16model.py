"""Pins of the oracle's bf16 error model (oracle/bf16model.py): the rounding against an independent library's
conversion and against hand-made ties, and the model against the exact one where nothing needs rounding."""
import numpy as np
import torch

from oracle import bf16model as bm
from oracle import ppo
from workloads import synthetic as syn


def test_rounding_matches_an_independent_conversion():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, 100000),
                        np.array([0.0, -0.0, 1.0, -1.0, np.inf, -np.inf, 3.3895314e38, 1e-40, -1e-45], np.float32)])
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = bm.round_bf16(x)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    assert np.isnan(bm.round_bf16(np.array([np.nan], np.float32))[0])


def test_rounding_ties_go_to_even():
    # bf16 keeps 8 significand bits: the spacing at 1.0 is 2^-7, a tie sits at odd multiples of 2^-8
    one = np.float32(1.0)
    ulp = np.float32(2.0 ** -7)
    assert bm.round_bf16(np.array([one + ulp / 2]))[0] == one                    # tie -> even (1.0)
    assert bm.round_bf16(np.array([one + ulp + ulp / 2]))[0] == one + 2 * ulp    # tie -> even (1 + 2 ulp)
    assert bm.round_bf16(np.array([one + ulp / 2 + np.float32(2.0 ** -20)]))[0] == one + ulp
    assert bm.round_bf16(np.array([one + ulp / 2 - np.float32(2.0 ** -20)]))[0] == one
    # idempotent
    x = np.random.default_rng(1).standard_normal(1000).astype(np.float32)
    assert np.array_equal(bm.round_bf16(bm.round_bf16(x)), bm.round_bf16(x))


def test_model_equals_the_exact_one_where_nothing_is_rounded():
    # small integers and halves are exact in bf16, and so are their short sums and the ELU of non-negative sums:
    # weights, inputs and biases >= 0 keep every activation on the identity branch
    shape = ppo.ModelShape(4, 2, (3, 3))
    rng = np.random.default_rng(2)
    theta = (rng.integers(0, 3, shape.n_params()) * 0.5).astype(np.float32)
    theta[-2:] = 0.0
    obs = rng.integers(0, 4, (8, 4)).astype(np.float32)
    mu, v = bm.agent_forward(theta, shape, obs)
    pol, val, _ = ppo.unpack(theta, shape)
    assert np.array_equal(mu, ppo.mlp_forward(obs, pol)[0])
    assert np.array_equal(v, ppo.mlp_forward(obs, val)[0][:, 0])


def test_model_stays_within_the_bf16_band_of_the_exact_one_and_is_not_identical():
    cfg = syn.get_config("C2")
    shape = ppo.ModelShape(cfg.obs_dim, cfg.act_dim, cfg.hidden)
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, 1, policy_head_scale=0.5)
    rng = np.random.default_rng(3)
    m = 512
    obs = rng.standard_normal((m, cfg.obs_dim)).astype(np.float32)
    act = rng.standard_normal((m, cfg.act_dim)).astype(np.float32)
    pol, _, log_std = ppo.unpack(theta.astype(np.float64), shape)
    mu, _ = ppo.mlp_forward(obs.astype(np.float64), pol)
    z = (act - mu) * np.exp(-log_std)
    logp = ((-0.5 * z * z - log_std - 0.5 * ppo.LOG_2PI).sum(1) + 0.05 * rng.standard_normal(m)).astype(np.float32)
    adv = rng.standard_normal(m).astype(np.float32)
    ret = rng.standard_normal(m).astype(np.float32)
    hp = ppo.PPOHyper(c_e=0.01)
    s_ref, g_ref = ppo.ppo_loss_and_grad(theta, shape, obs, act, logp, adv, ret, hp)
    s_bf, g_bf = bm.ppo_loss_and_grad(theta, shape, obs, act, logp, adv, ret, hp)
    err = np.linalg.norm(g_bf - g_ref) / np.linalg.norm(g_ref)
    assert 1e-4 < err < 2e-2, err
    assert abs(s_bf[1] - s_ref[1]) < 2e-2 * abs(s_ref[1])
    # the log-std gradient layout and the entropy (no rounding involved) are the exact model's
    assert s_bf[2] == s_ref[2]
