"""GPU parity of the bf16 path against the oracle's bf16 error model (oracle/bf16model.py), and the bf16 path at
the sizes the benchmark runs.

The fp32 oracle bounds the bf16 path only through the 2e-2 band of the problem statement; inside that band a small
indexing mistake (one wrong row in thousands) and rounding look alike.  The error model rounds exactly what the
bf16 path stores in bf16, so what is left between it and the HIP result is the order of the fp32 sums, the
exponential's last bits, and activations that sit within an fp32 rounding error of a bf16 tie: ~1e-3."""
import numpy as np
import pytest
import torch

from oracle import bf16model as bm
from oracle import ppo as oppo
from workloads import synthetic as syn
from gpu_util import make_session, oracle_pieces, rel_l2, rel_max
from test_gpu_parity import _bind_buffer, _bind_model, _filled_buffer, dev, zeros, g, inst, _keep_device_inputs_alive  # noqa: F401

pytestmark = pytest.mark.gpu

TOL_MODEL = 1e-3       # HIP bf16 path against the bf16 error model, per tensor, relative L2
TOL_MODEL_MAX = 3e-3   # the same, largest element error over largest element (a hidden activation within an fp32
                       # rounding error of a bf16 tie rounds the other way and moves single outputs by ~2e-3)
TOL16 = 2e-2


@pytest.mark.parametrize("name,n", [("C2", 4096), ("C3", 777), ("C4", 5000), ("SH", 700), ("C2", 33)])
@pytest.mark.parametrize("fused", [True, False])
def test_agent_forward_matches_the_bf16_error_model(g, inst, name, n, fused):
    g.gmi_set_fusion(inst, 1 if fused else 0)
    cfg = syn.get_config(name)
    shape = oppo.ModelShape(cfg.obs_dim, cfg.act_dim, tuple(cfg.hidden))
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, 3, policy_head_scale=1.0)
    obs = syn.make_initial_state(n, cfg.obs_dim, 5)
    hm, keep = _bind_model(g, inst, cfg, theta, max(n, 64), "bf16", with_adam=False)
    A = cfg.act_dim
    act, logp, val, mu = zeros(n, A), zeros(n), zeros(n), zeros(n, A)
    g.agent_act(inst, hm, dev(obs), n, 42, 9, 100, act, logp, val, mu)
    g.gmi_sync(inst)
    m_mu, m_val = bm.agent_forward(theta, shape, obs)
    for got, ref in ((mu.cpu().numpy(), m_mu), (val.cpu().numpy(), m_val)):
        assert rel_l2(got, ref) <= TOL_MODEL, rel_l2(got, ref)
        assert rel_max(got, ref) <= TOL_MODEL_MAX, rel_max(got, ref)
    # every row on its own, the ragged last tile included: a wrong row would stand out by orders of magnitude
    row_err = np.abs(mu.cpu().numpy() - m_mu).max(axis=1) / np.abs(m_mu).max()
    assert row_err.max() <= TOL_MODEL_MAX, (int(row_err.argmax()), row_err.max())
    g.gmi_model_destroy(hm)
    g.gmi_set_fusion(inst, 1)


def _gradient_case(g, inst, name, T, N, rows, seed=1):
    cfg = syn.get_config(name)
    shape = oppo.ModelShape(cfg.obs_dim, cfg.act_dim, tuple(cfg.hidden))
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, seed, policy_head_scale=0.5)
    b, rb, hb = _filled_buffer(g, inst, cfg, T, N, seed=2)
    flat = oppo.flatten_buffer(b)
    pol, _, log_std = oppo.unpack(theta.astype(np.float64), shape)
    mu, _ = oppo.mlp_forward(flat["obs"].astype(np.float64), pol)
    z = (flat["act"] - mu) * np.exp(-log_std)
    logp = (-0.5 * z * z - log_std - 0.5 * oppo.LOG_2PI).sum(1)
    rng = np.random.default_rng(3)
    # ratios well inside or well outside the clip range: the yes/no clipping decisions agree in every arithmetic
    sign = np.where(rng.random(T * N) < 0.5, -1.0, 1.0)
    jitter = sign * np.where(rng.random(T * N) < 0.5, 0.08 * rng.random(T * N), 0.32 + 0.3 * rng.random(T * N))
    b["logp"] = (logp + jitter).astype(np.float32).reshape(T, N)
    b["adv"], b["ret"] = oppo.gae(b["rew"], b["val"], b["done"], b["last_val"], 0.99, 0.95, True)
    rb.logp.copy_(dev(b["logp"])); rb.adv.copy_(dev(b["adv"])); rb.ret.copy_(dev(b["ret"]))
    torch.cuda.synchronize()
    hm, keep = _bind_model(g, inst, cfg, theta, rows, "bf16")
    idx = rng.permutation(T * N)[:rows].astype(np.int32)
    hp = g.ppo_hparams(clip=0.2, c_v=0.5, c_e=0.01, minibatch=rows)
    grad, stats = zeros(theta.size), zeros(5)
    g.ppo_gradient(inst, hm, hb, hp, dev(idx), rows, grad, stats)
    g.gmi_sync(inst)
    flat = oppo.flatten_buffer(b)
    args = (theta, shape, flat["obs"][idx], flat["act"][idx], flat["logp"][idx], flat["adv"][idx], flat["ret"][idx],
            oppo.PPOHyper(clip=0.2, c_v=0.5, c_e=0.01))
    got = grad.cpu().numpy(), stats.cpu().numpy()
    g.gmi_model_destroy(hm)
    g.gmi_buffer_destroy(hb)
    return shape, got, args


def _per_tensor(shape, got, ref, tol):
    off = 0
    for out_dim in (shape.act_dim, 1):
        for i, o in shape.layer_dims(out_dim):
            for n_el in (i * o, o):
                seg = slice(off, off + n_el)
                assert rel_l2(got[seg], ref[seg]) <= tol, (off, rel_l2(got[seg], ref[seg]))
                off += n_el
    assert rel_l2(got[off:], ref[off:]) <= tol


@pytest.mark.parametrize("name,T,N,rows", [("C2", 4, 512, 2048), ("C3", 2, 1024, 2048), ("C4", 2, 700, 1400),
                                           ("C2", 3, 500, 1111), ("HM", 2, 700, 1400), ("SH", 2, 600, 1111)])
@pytest.mark.parametrize("path", ["fused", "layers"])
def test_gradient_matches_the_bf16_error_model(g, inst, name, T, N, rows, path):
    g.gmi_set_fusion(inst, 1 if path == "fused" else 0)
    shape, (got_g, got_s), args = _gradient_case(g, inst, name, T, N, rows)
    m_stats, m_grad = bm.ppo_loss_and_grad(*args)
    assert rel_l2(got_g, m_grad) <= TOL_MODEL, rel_l2(got_g, m_grad)
    assert rel_max(got_g, m_grad) <= TOL_MODEL_MAX, rel_max(got_g, m_grad)
    _per_tensor(shape, got_g, m_grad, 2 * TOL_MODEL)
    assert np.allclose(got_s[:2], m_stats[:2], rtol=TOL_MODEL, atol=1e-5)
    g.gmi_set_fusion(inst, 1)


def test_gradient_of_a_benchmark_sized_minibatch_c4(g, inst):
    """32768 rows of the largest workload's model, the launch configuration the benchmark times (512 workgroups
    of the trainer kernel, every row split of the weight-gradient kernel), against the fp32 oracle and the
    error model."""
    shape, (got_g, got_s), args = _gradient_case(g, inst, "C4", 2, 16384, 32768)
    r_stats, r_grad = oppo.ppo_loss_and_grad(*args)
    assert rel_l2(got_g, r_grad) <= TOL16, rel_l2(got_g, r_grad)
    assert rel_max(got_g, r_grad) <= TOL16, rel_max(got_g, r_grad)
    _per_tensor(shape, got_g, r_grad, 2 * TOL16)
    m_stats, m_grad = bm.ppo_loss_and_grad(*args)
    assert rel_l2(got_g, m_grad) <= TOL_MODEL, rel_l2(got_g, m_grad)
    assert rel_max(got_g, m_grad) <= TOL_MODEL_MAX, rel_max(got_g, m_grad)
    assert abs(got_s[0] - r_stats[0]) <= 1e-2 * max(1, abs(r_stats[0]))
    assert abs(got_s[1] - r_stats[1]) <= 1e-2 * max(1, abs(r_stats[1]))


def test_whole_iteration_c2_at_benchmark_size(g):
    """One whole iteration of the 4096-env workload at its full size (horizon 16, minibatch 32768, two minibatches
    per epoch, here two epochs), one-launch collection and the fused trainer kernels, against the fp32 oracle."""
    from oracle import philox as px
    from test_gpu_parity import _run_iteration_both
    cfg = syn.get_config("C2")
    ref, ses, stats, (shape, theta, env, hp) = _run_iteration_both(g, cfg, cfg.n_envs, cfg.minibatch, cfg.horizon, 2,
                                                                   "bf16", True)
    got = ses.buf.to_numpy()
    rb = ref["buf"]
    assert np.array_equal(got["done"], rb["done"])
    for k in ("obs", "act", "val", "rew", "ret"):
        assert rel_l2(got[k], rb[k]) <= TOL16, (k, rel_l2(got[k], rb[k]))
        assert rel_max(got[k], rb[k]) <= TOL16, (k, rel_max(got[k], rb[k]))
    assert rel_l2(got["logp"], rb["logp"]) <= 1e-5
    assert stats.shape == ref["stats"].shape == (4, 5)
    assert np.abs(stats - ref["stats"]).max() <= 2e-2 * max(1.0, np.abs(ref["stats"]).max())
    step, ref_step = ses.theta.cpu().numpy() - theta, ref["theta"] - theta
    assert np.abs(ref_step).max() > 1e-4
    assert rel_l2(ses.theta.cpu().numpy(), ref["theta"]) <= 1e-3
    ses.close()


@pytest.mark.parametrize("name", ["C4", "C3"])
def test_collection_at_benchmark_size_on_sampled_envs(g, name):
    """The collection stage of a benchmark workload at its full size (C4: 16384 envs x 16 steps through the
    two-launches-per-step form of rollout_collect; C3: 4096 envs x 32 steps in one launch), in the launch
    configuration bench.py times.  Envs are independent and the generator's counters carry the env index, so the
    oracle computes blocks of 192 envs from three places of the range (first tile, a ragged middle, the last envs)
    with env_offset = the block's first env, and every array of the buffer is compared on those columns."""
    cfg = syn.get_config(name)
    shape, theta, env, state0, hp = oracle_pieces(cfg)
    ses = make_session(cfg, theta, env, state0, fused_rollout=True)
    ses.rollout(0)
    ses.sync()
    assert ses.fused_rollout
    got = ses.buf.to_numpy()
    last = ses.last_value.cpu().numpy()
    final = ses.state().cpu().numpy()
    n, T, blk = cfg.n_envs, cfg.horizon, 192
    for k0 in (0, n // 2 - 77, n - blk):
        buf = oppo.new_buffer(T, blk, cfg.obs_dim, cfg.act_dim)
        st, ep, lv = oppo.rollout(theta, shape, env, state0[k0:k0 + blk], np.zeros(blk, np.uint32), buf, env.seed, 0,
                                  env_offset=k0)
        sl = slice(k0, k0 + blk)
        assert np.array_equal(got["done"][:, sl], buf["done"]), k0
        for key in ("obs", "act", "val", "rew"):
            assert rel_l2(got[key][:, sl], buf[key]) <= TOL16, (k0, key, rel_l2(got[key][:, sl], buf[key]))
            assert rel_max(got[key][:, sl], buf[key]) <= TOL16, (k0, key, rel_max(got[key][:, sl], buf[key]))
        assert rel_l2(got["logp"][:, sl], buf["logp"]) <= 1e-5
        assert rel_l2(last[sl], lv) <= TOL16 and rel_l2(final[sl], st) <= TOL16
    ses.close()
