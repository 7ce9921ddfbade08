"""Pins of the fp8 inference oracle (oracle/fp8model.py) against the E4M3 format's definition (OCP 8-bit floating
point specification: bias 7, 3 mantissa bits, largest finite value 448 = 0x7E, smallest normal 2^-6 = 0x08,
smallest subnormal 2^-9 = 0x01), brute force over its 256 patterns, and cases where rounding is the identity."""
import numpy as np

from oracle import fp8model as f8
from oracle import ppo as oppo
from workloads import synthetic as syn

CODES = [c for c in range(256) if (c & 0x7F) != 0x7F]
TABLE = np.array([f8.decode_e4m3(c) for c in CODES])


def test_format_constants():
    assert f8.decode_e4m3(0x7E) == 448.0 and f8.decode_e4m3(0xFE) == -448.0
    assert f8.decode_e4m3(0x08) == 2.0 ** -6 and f8.decode_e4m3(0x01) == 2.0 ** -9
    assert f8.decode_e4m3(0x38) == 1.0 and f8.decode_e4m3(0x00) == 0.0
    assert np.isnan(f8.decode_e4m3(0x7F)) and np.isnan(f8.decode_e4m3(0xFF))
    assert len(set(TABLE[TABLE > 0])) == 126      # 2 * 126 non-zero finite values, two zeros


def test_every_finite_pattern_is_a_fixed_point():
    assert np.array_equal(f8.round_e4m3(TABLE), TABLE.astype(np.float32))


def test_rounding_is_nearest_by_brute_force():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.normal(0, 1, 4000), rng.normal(0, 100, 2000), rng.uniform(-2 ** -5, 2 ** -5, 2000),
                        rng.uniform(-500, 500, 2000)])
    got = f8.round_e4m3(x).astype(np.float64)
    d = np.abs(x[:, None] - TABLE[None, :])
    best = d.min(axis=1)
    assert np.all(np.abs(got - x) == best)        # random reals hit no tie: the nearest value is unique
    assert np.all(np.isin(got, TABLE))


def test_ties_go_to_the_even_mantissa_and_neighbours_to_the_nearest():
    pos = sorted(c for c in CODES if c < 0x80)
    for lo, hi in zip(pos[:-1], pos[1:]):
        a, b = f8.decode_e4m3(lo), f8.decode_e4m3(hi)
        mid = 0.5 * (a + b)                        # exact: both are short binary fractions
        even = a if lo % 2 == 0 else b
        assert f8.round_e4m3(mid) == np.float32(even), (lo, hi)
        assert f8.round_e4m3(-mid) == np.float32(-even)
        eps = (b - a) / 64
        assert f8.round_e4m3(mid - eps) == np.float32(a) and f8.round_e4m3(mid + eps) == np.float32(b)


def test_saturation():
    assert f8.round_e4m3(1000.0) == 448.0 and f8.round_e4m3(-1e9) == -448.0
    assert f8.round_e4m3(464.0) == 448.0 and f8.round_e4m3(479.9) == 448.0     # past the last midpoint: still 448
    assert f8.round_e4m3(2.0 ** -10) == 0.0                                      # half the smallest subnormal: tie to 0
    assert f8.round_e4m3(2.0 ** -10 * 1.01) == np.float32(2.0 ** -9)


def test_layer_scale_is_the_smallest_power_of_two_that_fits():
    for k in (-9, -3, 0, 2):
        w = np.array([[448.0 * 2.0 ** k, -1e-3]])
        assert f8.layer_scale(w) == 2.0 ** k
        assert f8.layer_scale(w * (1 + 1e-6)) == 2.0 ** (k + 1)
    assert f8.layer_scale(np.zeros((2, 2))) == 1.0
    rng = np.random.default_rng(9)
    for _ in range(20):
        w = rng.normal(0, 10.0 ** rng.uniform(-4, 2), (7, 5))
        s = f8.layer_scale(w)
        m = np.abs(w).max() / s
        assert 224.0 < m <= 448.0 and np.log2(s) == np.round(np.log2(s))


def test_forward_is_exact_when_nothing_needs_rounding():
    """Small-integer weights scaled by a power of two, inputs and pre-activations positive integers <= 16 (all
    representable): the fp8 forward equals the exact one, scale, bias and ELU included."""
    rng = np.random.default_rng(2)
    x = rng.integers(0, 3, (9, 6)).astype(np.float32)
    w0 = rng.integers(0, 2, (5, 6)).astype(np.float32)          # z0 = x w0^T + 1 in [1, 13]
    b0 = np.ones(5, np.float32)
    w1 = (rng.integers(-3, 4, (4, 5)) * 0.125).astype(np.float32)
    b1 = rng.normal(0, 1, 4).astype(np.float32)                 # biases are fp32, any value
    layers = [(w0, b0), (w1, b1)]
    ref, _ = oppo.mlp_forward(x, layers)
    got = f8.mlp_forward(x, layers)
    assert np.allclose(got, ref, rtol=0, atol=1e-6)
    # and the scale really is applied: the same weights times 2^-5 give outputs that differ by the bias-free part
    layers2 = [(w0, b0), (w1 * 2.0 ** -5, b1)]
    got2 = f8.mlp_forward(x, layers2)
    assert np.allclose(got2 - b1, (got - b1) * 2.0 ** -5, rtol=0, atol=1e-6)


def test_precision_cost_against_the_exact_network_is_a_few_percent():
    cfg = syn.get_config("C2")
    shape = oppo.ModelShape(cfg.obs_dim, cfg.act_dim, tuple(cfg.hidden))
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    obs = syn.make_initial_state(256, cfg.obs_dim, cfg.seed)
    mu, v = f8.agent_forward(theta, shape, obs)
    pol, val, _ = oppo.unpack(theta.astype(np.float32), shape)
    mu_ref, _ = oppo.mlp_forward(obs.astype(np.float32), pol)
    v_ref, _ = oppo.mlp_forward(obs.astype(np.float32), val)
    for got, ref in ((mu, mu_ref), (v, v_ref[:, 0])):
        rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        assert 1e-3 < rel < 0.1, rel


def test_agent_act_uses_the_same_noise_as_the_exact_agent():
    cfg = syn.get_config("C1")
    shape = oppo.ModelShape(cfg.obs_dim, cfg.act_dim, tuple(cfg.hidden))
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, cfg.seed)
    obs = syn.make_initial_state(16, cfg.obs_dim, cfg.seed)
    act, logp, v, mu = f8.agent_act(theta, shape, obs, cfg.seed, 3)
    act_r, logp_r, _, mu_r = oppo.agent_act(theta, shape, obs, cfg.seed, 3)
    assert np.array_equal(logp, logp_r)                        # the log-density depends on the noise alone
    assert np.allclose(act - mu, act_r - mu_r, atol=1e-6)
