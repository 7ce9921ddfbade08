"""GPU parity: every step of the hot path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Tolerances: bit-exact for noise, done flags, counters and the shuffle;
1e-5 (relative, per tensor, plus an elementwise bound) for env states/rewards, GAE, returns, Adam
and the fp32 model path; 2e-2 for everything that goes through bf16 matrix cores."""
import numpy as np
import pytest
import torch

from oracle import philox as px
from oracle import ppo as oppo
from workloads import synthetic as syn
from gpu_util import make_session, oracle_pieces, rel_l2, rel_max

pytestmark = pytest.mark.gpu

TOL32 = 1e-5
TOL16 = 2e-2


@pytest.fixture(scope="module")
def g():
    import paper_2206_08482_amd as g_
    return g_


@pytest.fixture(scope="module")
def inst(g):
    h = g.gmi_create()
    yield h
    g.gmi_destroy(h)


# Tensors handed to the library must outlive the asynchronous work that reads them: a temporary passed straight
# into a call is freed when the call returns, and the allocator may hand its memory to the next tensor (whose fill
# runs on torch's stream) while the kernel is still reading it.  Everything dev() makes lives until the test ends.
_KEEP = []


@pytest.fixture(autouse=True)
def _keep_device_inputs_alive():
    yield
    if torch.cuda.is_available():
        torch.cuda.synchronize()
    _KEEP.clear()


def dev(x, dtype=None):
    t = torch.tensor(np.ascontiguousarray(x), device="cuda:0")
    if dtype is not None:
        t = t.to(dtype)
    torch.cuda.synchronize()
    _KEEP.append(t)
    return t


def zeros(*shape, dtype=torch.float32):
    t = torch.zeros(*shape, dtype=dtype, device="cuda:0")
    torch.cuda.synchronize()
    return t


def close32(x, ref, tol=TOL32):
    x, ref = np.asarray(x, np.float64), np.asarray(ref, np.float64)
    assert rel_l2(x, ref) <= tol, rel_l2(x, ref)
    assert np.all(np.abs(x - ref) <= 10 * tol * np.abs(ref) + 10 * tol * max(1e-6, np.abs(ref).max())), \
        np.abs(x - ref).max()


# ----------------------------------------------------------------------------- random numbers
@pytest.mark.parametrize("n,dim,stream,step,off", [(1, 1, 0, 0, 0), (1000, 7, 1, 12345, 17),
                                                   (1 << 18, 8, 3, 0xFFFFFFFF, 0), (4096, 211, 1, 31, 4096)])
def test_noise_is_bit_exact(g, inst, n, dim, stream, step, off):
    seed = 0x1234567890ABCDEF
    out = zeros(n, dim)
    g.gmi_noise_fill(inst, seed, stream, step, off, n, dim, out)
    g.gmi_sync(inst)
    ref = px.normal_field(seed, stream, step, n, dim, env_offset=off)
    got = out.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("n", [1, 2, 3, 64, 1000, 1024, 65536, 100003])
def test_shuffle_is_bit_exact(g, inst, n):
    out = zeros(n, dtype=torch.int32)
    g.gmi_permutation(inst, n, 7, 3, 2, out)
    g.gmi_sync(inst)
    assert np.array_equal(out.cpu().numpy().astype(np.int64), px.feistel_permutation(n, 7, 3, 2))


# ----------------------------------------------------------------------------- environment
@pytest.mark.parametrize("n,o,a,period,prob_inv", [(64, 8, 2, 16, 0), (1000, 60, 8, 0, 10), (333, 108, 21, 0, 1000),
                                                   (257, 211, 20, 3, 0), (5, 3, 5, 0, 2), (20000, 60, 8, 0, 1000)])
def test_env_step_matches_oracle(g, inst, n, o, a, period, prob_inv):
    rng = np.random.default_rng(n + o)
    am, bm = syn.make_env_matrices(o, a, 1)
    thr = oppo.done_threshold_from_inverse(prob_inv)
    seed, off = 99, 1000
    env = oppo.EnvSpec(am, bm, 0.01, 0.5, period, thr, seed)
    s = rng.standard_normal((n, o)).astype(np.float32)
    act = rng.standard_normal((n, a)).astype(np.float32)
    ep = rng.integers(0, 7, n).astype(np.uint32)
    d_ep = dev(ep.astype(np.int32))
    e_desc = g.env_desc(n, o, a, 0.01, 0.5, period, thr, seed, off)
    h = g.gmi_env_bind(inst, e_desc, dev(am), dev(bm), d_ep)
    nxt, rew, done = zeros(n, o), zeros(n), zeros(n, dtype=torch.uint8)
    d_s, d_a = dev(s), dev(act)
    for step in (5, 6):
        g.env_step(inst, h, d_s, d_a, step, nxt, rew, done)
        g.gmi_sync(inst)
        r_nxt, r_rew, r_done, ep = oppo.env_step(env, s, act, ep, step, env_offset=off)
        assert np.array_equal(done.cpu().numpy(), r_done)
        assert np.array_equal(d_ep.cpu().numpy().astype(np.uint32), ep)
        close32(rew.cpu().numpy(), r_rew)
        got = nxt.cpu().numpy()
        close32(got, r_nxt)
        if r_done.any():     # reset states are pure noise: bit-exact
            assert np.array_equal(got[r_done.astype(bool)], r_nxt[r_done.astype(bool)])
        s = r_nxt
        d_s = dev(s)
    g.gmi_env_destroy(h)


# ----------------------------------------------------------------------------- experience + GAE
def _bind_buffer(g, inst, T, N, ld, O, A, col0=0):
    from paper_2206_08482_amd.runner import RolloutBuffers
    rb = RolloutBuffers(T, ld, O, A, torch.device("cuda:0"))
    torch.cuda.synchronize()
    return rb, g.gmi_buffer_bind(inst, rb.desc(col0, N))


def test_collect_experience_fills_slot_t_of_a_column_slice(g, inst):
    T, N, ld, O, A, col0 = 5, 37, 64, 6, 3, 11
    rb, hb = _bind_buffer(g, inst, T, N, ld, O, A, col0)
    rng = np.random.default_rng(0)
    data = [rng.standard_normal((N, O)), rng.standard_normal((N, A)), rng.standard_normal(N),
            rng.standard_normal(N), rng.standard_normal(N)]
    data = [x.astype(np.float32) for x in data] + [(rng.random(N) < 0.3).astype(np.uint8)]
    g.collect_experience(inst, hb, 3, *[dev(x) for x in data])
    g.gmi_sync(inst)
    out = rb.to_numpy()
    for name, x in zip(("obs", "act", "logp", "val", "rew", "done"), data):
        assert np.array_equal(out[name][3, col0:col0 + N], x)
        rest = out[name].copy()
        rest[3, col0:col0 + N] = 0
        assert not rest.any()
    with pytest.raises(g.GmiError):
        g.collect_experience(inst, hb, T, *[dev(x) for x in data])
    g.gmi_buffer_destroy(hb)


@pytest.mark.parametrize("T,N,ld,normalize", [(16, 64, 64, True), (1, 1, 1, False), (32, 4096, 4096, True),
                                              (7, 1000, 1024, True), (64, 300, 300, False), (16, 70000, 70000, True)])
@pytest.mark.parametrize("variant", [0, 1])
def test_gae_matches_oracle(g, inst, T, N, ld, normalize, variant):
    """variant 0: the serial walk with a lane per env (the default); 1: the wavefront scan with lanes over time."""
    g.gmi_bench_gae_variant(variant)
    b = syn.make_rollout_batch(T, N, 3, 2, seed=T + N, done_prob=0.1)
    rb, hb = _bind_buffer(g, inst, T, N, ld, 3, 2)
    rb.rew[:, :N] = dev(b["rew"])
    rb.val[:, :N] = dev(b["val"])
    rb.done[:, :N] = dev(b["done"])
    torch.cuda.synchronize()
    g.gae_compute(inst, hb, dev(b["last_val"]), 0.99, 0.95, normalize)
    g.gmi_sync(inst)
    adv, ret = oppo.gae(b["rew"], b["val"], b["done"], b["last_val"], 0.99, 0.95, normalize)
    close32(rb.adv[:, :N].cpu().numpy(), adv)
    close32(rb.ret[:, :N].cpu().numpy(), ret)
    if ld > N:
        assert not rb.adv[:, N:].any().item()
    g.gmi_buffer_destroy(hb)
    g.gmi_bench_gae_variant(0)


# ----------------------------------------------------------------------------- agent
def _bind_model(g, inst, cfg, theta, rows, dtype=None, with_adam=True):
    dt = cfg.dtype if dtype is None else dtype
    desc = g.model_desc(cfg.obs_dim, cfg.act_dim, list(cfg.hidden), 0 if dt == "f32" else 1, rows)
    t = dev(theta)
    nb = g.gmi_model_shadow_bytes(desc)
    shadow = zeros(max(nb, 256), dtype=torch.uint8) if nb else None
    m, v = (zeros(theta.size), zeros(theta.size)) if with_adam else (None, None)
    torch.cuda.synchronize()      # the fills above run on torch's stream, the library on the instance's
    h = g.gmi_model_bind(inst, desc, t, shadow, m, v)
    g.gmi_model_refresh_shadow(inst, h)
    g.gmi_sync(inst)
    return h, (t, shadow, m, v)


@pytest.mark.parametrize("name,n,dtype", [("C1", 64, "f32"), ("C1", 1, "f32"), ("C2", 1000, "f32"), ("C2", 4096, "bf16"),
                                          ("C3", 777, "bf16"), ("C4", 600, "bf16"), ("C1", 100, "bf16"),
                                          ("C3", 4096, "bf16"), ("C4", 5000, "bf16"), ("C2", 33, "bf16"), ("SH", 700, "bf16")])
@pytest.mark.parametrize("fused", [True, False])
def test_agent_act_matches_oracle(g, inst, name, n, dtype, fused):
    g.gmi_set_fusion(inst, 1 if fused else 0)
    cfg = syn.get_config(name)
    shape, theta, env, _, _ = oracle_pieces(cfg, n_envs=n)
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, 3, policy_head_scale=1.0)
    theta[-cfg.act_dim:] = 0.1 * np.random.default_rng(0).standard_normal(cfg.act_dim)
    obs = syn.make_initial_state(n, cfg.obs_dim, 5)
    hm, keep = _bind_model(g, inst, cfg, theta, max(n, 64), dtype, with_adam=False)
    A = cfg.act_dim
    act, logp, val, mu = zeros(n, A), zeros(n), zeros(n), zeros(n, A)
    g.agent_act(inst, hm, dev(obs), n, 42, 9, 100, act, logp, val, mu)
    val2 = zeros(n)
    g.agent_value(inst, hm, dev(obs), n, val2)
    g.gmi_sync(inst)
    r_act, r_logp, r_val, r_mu = oppo.agent_act(theta, shape, obs, 42, 9, env_offset=100)
    tol = TOL32 if dtype == "f32" else TOL16
    for got_x, ref_x in ((mu, r_mu), (val, r_val), (act, r_act)):
        assert rel_l2(got_x.cpu().numpy(), ref_x) <= tol
        assert rel_max(got_x.cpu().numpy(), ref_x) <= tol          # no single element further off than tol * max|ref|
    assert np.array_equal(val2.cpu().numpy(), val.cpu().numpy())
    # the log-prob depends on the noise and log_std only: tight in both precisions
    close32(logp.cpu().numpy(), r_logp)
    # the sampled action is consistent with the HIP path's own mean and the bit-exact noise
    eps = px.normal_field(42, px.STREAM_ACTION, 9, n, A, env_offset=100)
    close32(act.cpu().numpy(), mu.cpu().numpy() + np.exp(theta[-A:]) * eps)
    g.gmi_model_destroy(hm)
    g.gmi_set_fusion(inst, 1)


# ----------------------------------------------------------------------------- trainer
def _filled_buffer(g, inst, cfg, T, N, seed):
    b = syn.make_rollout_batch(T, N, cfg.obs_dim, cfg.act_dim, seed=seed, done_prob=0.05)
    rb, hb = _bind_buffer(g, inst, T, N, N, cfg.obs_dim, cfg.act_dim)
    for k in ("obs", "act", "logp", "val", "rew", "done"):
        getattr(rb, k).copy_(dev(b[k]))
    torch.cuda.synchronize()
    return b, rb, hb


def _theta_and_batch(cfg, T, N, seed=1):
    """Parameters with O(1) policy outputs, and a batch whose stored log-probs are near the current
    policy's so that ratios straddle the clip range."""
    shape = oppo.ModelShape(cfg.obs_dim, cfg.act_dim, tuple(cfg.hidden))
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, seed, policy_head_scale=0.5)
    return shape, theta


@pytest.mark.parametrize("name,T,N,rows,dtype,ratios", [
    ("C1", 16, 64, 256, "f32", "straddle"), ("C1", 4, 50, 77, "f32", "straddle"),
    ("C2", 4, 512, 2048, "bf16", "bimodal"), ("C2", 3, 500, 1111, "bf16", "bimodal"),
    ("C3", 2, 1024, 2048, "bf16", "bimodal"), ("C4", 2, 700, 1400, "bf16", "bimodal"),
    ("C2", 4, 512, 2048, "bf16", "straddle"),
    # large-tile kernels (rows >= 8192), ragged against their 256-row tiles
    ("C4", 2, 4200, 8400, "bf16", "bimodal"), ("C3", 3, 3000, 8999, "bf16", "bimodal"),
    ("C2", 2, 8192, 16384, "bf16", "bimodal"),
    # the paper's Table 6 model shapes under their own layer orders
    ("BB", 3, 400, 1200, "bf16", "bimodal"), ("FC", 2, 300, 555, "bf16", "bimodal"),
    ("AY", 2, 512, 1024, "bf16", "bimodal"), ("HM", 2, 700, 1400, "bf16", "bimodal"),
    ("SH", 2, 600, 1111, "bf16", "bimodal")])
@pytest.mark.parametrize("path", ["chain", "layers"])
def test_gradient_and_stats_match_oracle(g, inst, name, T, N, rows, dtype, ratios, path):
    """path: which trainer kernels compute forward, loss and input gradients: "chain" the one-launch kernels (the
    register-chained kernel or, for the 512-wide shapes, the row-tile kernel; the library's default for the model
    shapes they are compiled for), "layers" the per-layer kernels.
    ratios = "straddle": old/new probability ratios spread smoothly across the clip range, so some
    samples sit within rounding distance of a clip boundary.  Which side such a sample falls on is a
    yes/no decision taken in the arithmetic of the forward pass; in fp32 both sides agree, in bf16 a
    boundary sample may be clipped on one side and not on the other, which changes the policy
    gradient by that sample's whole contribution.  ratios = "bimodal" keeps every ratio either well
    inside or well outside the clip range, so the decisions agree and the comparison measures the
    arithmetic of the products alone."""
    if path == "chain" and (dtype == "f32" or name == "C1"):
        pytest.skip("the register-chained kernel covers the bf16 benchmark shapes")
    fused = path != "layers"
    g.gmi_set_fusion(inst, {"chain": 1, "layers": 0}[path])
    cfg = syn.get_config(name)
    shape, theta = _theta_and_batch(cfg, T, N)
    b, rb, hb = _filled_buffer(g, inst, cfg, T, N, seed=2)
    # consistent log-probs: density of the stored actions under theta, jittered
    flat = oppo.flatten_buffer(b)
    pol, _, log_std = oppo.unpack(theta.astype(np.float64), shape)
    mu, _ = oppo.mlp_forward(flat["obs"].astype(np.float64), pol)
    z = (flat["act"] - mu) * np.exp(-log_std)
    logp = (-0.5 * z * z - log_std - 0.5 * oppo.LOG_2PI).sum(1)
    rng = np.random.default_rng(3)
    if ratios == "straddle":
        jitter = 0.2 * rng.standard_normal(T * N)
    else:
        sign = np.where(rng.random(T * N) < 0.5, -1.0, 1.0)
        jitter = sign * np.where(rng.random(T * N) < 0.5, 0.08 * rng.random(T * N), 0.32 + 0.3 * rng.random(T * N))
    b["logp"] = (logp + jitter).astype(np.float32).reshape(T, N)
    b["adv"], b["ret"] = oppo.gae(b["rew"], b["val"], b["done"], b["last_val"], 0.99, 0.95, True)
    rb.logp.copy_(dev(b["logp"])); rb.adv.copy_(dev(b["adv"])); rb.ret.copy_(dev(b["ret"]))
    torch.cuda.synchronize()
    hm, keep = _bind_model(g, inst, cfg, theta, rows, dtype)
    idx = rng.permutation(T * N)[:rows].astype(np.int32)
    hp = g.ppo_hparams(clip=0.2, c_v=0.5, c_e=0.01, minibatch=rows)
    grad, stats, stats2 = zeros(theta.size), zeros(5), zeros(5)
    g.ppo_gradient(inst, hm, hb, hp, dev(idx), rows, grad, stats)
    g.ppo_evaluate(inst, hm, hb, hp, dev(idx), rows, stats2)
    g.gmi_sync(inst)
    flat = oppo.flatten_buffer(b)
    ohp = oppo.PPOHyper(clip=0.2, c_v=0.5, c_e=0.01)
    r_stats, r_grad = oppo.ppo_loss_and_grad(theta, shape, flat["obs"][idx], flat["act"][idx], flat["logp"][idx],
                                             flat["adv"][idx], flat["ret"][idx], ohp)
    got_g, got_s = grad.cpu().numpy(), stats.cpu().numpy()
    # evaluate = forward + loss only.  With the one-launch trainer kernels the two calls run different kernels
    # (other order of the fp32 sums, bias inside or after them): a few bf16 activations round the other way,
    # which moves the batch statistics by ~1e-5 of their scale (the approximate KL is a mean of small signed
    # terms, hence the absolute floor).
    assert np.allclose(got_s, stats2.cpu().numpy(), rtol=2e-3 if fused else 1e-5, atol=2e-5 if fused else 1e-7)
    assert 0.02 < r_stats[4] < 0.9                         # the clip is active for part of the batch
    tol = 2e-4 if dtype == "f32" else TOL16
    n_pol = sum(i * o + o for i, o in shape.layer_dims(shape.act_dim))
    n_val = sum(i * o + o for i, o in shape.layer_dims(1))
    val_seg = slice(n_pol, n_pol + n_val)
    if dtype == "bf16" and ratios == "straddle":
        # value net: no yes/no decision involved -> full tolerance; policy net: bounded by the share
        # of samples within 2 % of a clip boundary (each may flip and move the gradient by its term)
        assert rel_l2(got_g[val_seg], r_grad[val_seg]) <= tol
        pol, _, log_std = oppo.unpack(theta.astype(np.float64), shape)
        mu, _ = oppo.mlp_forward(flat["obs"][idx].astype(np.float64), pol)
        zz = (flat["act"][idx] - mu) * np.exp(-log_std)
        ratio = np.exp((-0.5 * zz * zz - log_std - 0.5 * oppo.LOG_2PI).sum(1) - flat["logp"][idx])
        band = ((np.abs(ratio / 1.2 - 1) < 0.02) | (np.abs(ratio / 0.8 - 1) < 0.02)).mean()
        pol_idx = np.r_[0:n_pol, n_pol + n_val:theta.size]
        assert 0 < band < 0.1
        assert rel_l2(got_g[pol_idx], r_grad[pol_idx]) <= tol + 2 * np.sqrt(band)
    else:
        assert rel_l2(got_g, r_grad) <= tol, rel_l2(got_g, r_grad)
        assert rel_max(got_g, r_grad) <= tol, rel_max(got_g, r_grad)
        # per parameter tensor
        off = 0
        for out_dim in (shape.act_dim, 1):
            for i, o in shape.layer_dims(out_dim):
                for n_el in (i * o, o):
                    seg = slice(off, off + n_el)
                    assert rel_l2(got_g[seg], r_grad[seg]) <= 2 * tol, (off, rel_l2(got_g[seg], r_grad[seg]))
                    off += n_el
        assert rel_l2(got_g[off:], r_grad[off:]) <= 2 * tol
    stol = 1e-4 if dtype == "f32" else 1e-2
    assert abs(got_s[0] - r_stats[0]) <= stol * max(1, abs(r_stats[0]))
    assert abs(got_s[1] - r_stats[1]) <= stol * max(1, abs(r_stats[1]))
    assert abs(got_s[2] - r_stats[2]) <= 1e-5 * max(1, abs(r_stats[2]))
    assert abs(got_s[3] - r_stats[3]) <= stol * max(1, abs(r_stats[3]))
    assert abs(got_s[4] - r_stats[4]) <= (2.0 / rows if dtype == "f32" else 0.01)
    g.gmi_model_destroy(hm)
    g.gmi_buffer_destroy(hb)
    g.gmi_set_fusion(inst, 1)


@pytest.mark.parametrize("n", [1, 1000, 2789, 1 << 20])
def test_adam_matches_oracle_given_identical_gradients(g, inst, n):
    rng = np.random.default_rng(n)
    th = rng.standard_normal(n).astype(np.float32)
    m = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32)
    d_th, d_m, d_v = dev(th), dev(m), dev(v)
    ohp = oppo.PPOHyper(lr=3e-4)
    hp = g.ppo_hparams(lr=3e-4)
    for k in range(1, 6):
        gr = (rng.standard_normal(n) * 10.0 ** rng.integers(-6, 1, n)).astype(np.float32)
        g.adam_update(inst, d_th, d_m, d_v, dev(gr), n, hp, k)
        g.gmi_sync(inst)
        th, m, v = oppo.adam_step(th, m, v, gr, k, ohp)
    close32(d_th.cpu().numpy(), th)
    close32(d_m.cpu().numpy(), m)
    close32(d_v.cpu().numpy(), v)


def _run_iteration_both(g, cfg, n_envs, minibatch, horizon, epochs, dtype, fused_rollout=True):
    shape, theta, env, state0, hp = oracle_pieces(cfg, n_envs=n_envs)
    hp.minibatch, hp.epochs = minibatch, epochs
    z = np.zeros_like(theta)
    ref = oppo.ppo_iteration(theta, z, z, 0, shape, env, state0, np.zeros(n_envs, np.uint32), horizon, hp,
                             cfg.gamma, cfg.lam, cfg.seed, 0)
    ses = make_session(cfg, theta, env, state0, n_envs=n_envs, minibatch=minibatch, horizon=horizon, dtype=dtype,
                       fused_rollout=fused_rollout)
    ses.rollout(0)
    # rollout_collect really ran (one launch; for C4's model, beyond that kernel's size limit, two launches per step)
    assert ses.fused_rollout == (fused_rollout and dtype == "bf16")
    ses.gae(cfg.gamma, cfg.lam, True)
    nup = epochs * (horizon * n_envs // minibatch)
    stats = zeros(nup, 5)
    ses.update(0, epochs=epochs, minibatch=minibatch, stats=stats, clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e,
               lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, adam_eps=cfg.adam_eps)
    ses.sync()
    return ref, ses, stats.cpu().numpy(), (shape, theta, env, hp)


def test_whole_iteration_c1_fp32_matches_oracle(g):
    cfg = syn.get_config("C1")
    ref, ses, stats, (shape, theta, env, hp) = _run_iteration_both(g, cfg, cfg.n_envs, cfg.minibatch, cfg.horizon,
                                                                   cfg.epochs, "f32")
    got = ses.buf.to_numpy()
    rb = ref["buf"]
    assert np.array_equal(got["done"], rb["done"])
    for k in ("obs", "act", "logp", "val", "rew", "ret", "adv"):
        assert rel_l2(got[k], rb[k]) <= 2e-5, (k, rel_l2(got[k], rb[k]))
    assert rel_l2(ses.state().cpu().numpy(), ref["state"]) <= 2e-5
    assert np.array_equal(ses.episode_step.cpu().numpy().astype(np.uint32), ref["episode_step"])
    # per-minibatch statistics and the parameters after the four Adam steps
    assert stats.shape == ref["stats"].shape
    assert np.abs(stats - ref["stats"]).max() <= 1e-3
    th = ses.theta.cpu().numpy()
    step = th - theta
    ref_step = ref["theta"] - theta
    assert np.abs(ref_step).max() > 1e-4
    assert rel_l2(th, ref["theta"]) <= 1e-5
    assert rel_l2(step, ref_step) <= 5e-2          # Adam's early steps are sign-like: tiny gradients flip
    # loss of the next forward after the update: within 1e-3 absolute
    flat = oppo.flatten_buffer(rb)
    idx = px.feistel_permutation(cfg.batch, cfg.seed, 0, 0)[:cfg.minibatch]
    r_stats, _ = oppo.ppo_loss_and_grad(ref["theta"], shape, flat["obs"][idx], flat["act"][idx], flat["logp"][idx],
                                        flat["adv"][idx], flat["ret"][idx], hp, want_grad=False)
    out = zeros(5)
    h = g.ppo_hparams(clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, minibatch=cfg.minibatch)
    g.ppo_evaluate(ses.gmi, ses.model, ses.buffer, h, dev(idx.astype(np.int32)), cfg.minibatch, out)
    ses.sync()
    o = out.cpu().numpy()
    assert abs(oppo.total_loss(o, hp) - oppo.total_loss(r_stats, hp)) <= 1e-3
    ses.close()


def test_update_over_more_epochs_than_one_shuffle_launch_covers(g):
    """The shuffles of 8 epochs are made by one launch; 11 epochs need a second one that refills the same
    array.  fp32, so the parameters after 22 Adam steps follow the oracle closely."""
    cfg = syn.get_config("C1")
    ref, ses, stats, _ = _run_iteration_both(g, cfg, cfg.n_envs, 512, cfg.horizon, 11, "f32")
    assert stats.shape == ref["stats"].shape == (22, 5)
    assert np.abs(stats - ref["stats"]).max() <= 2e-3
    assert rel_l2(ses.theta.cpu().numpy(), ref["theta"]) <= 1e-4
    ses.close()


@pytest.mark.parametrize("name,n_envs,minibatch,horizon", [("C2", 512, 2048, 8), ("C3", 256, 1024, 8),
                                                           ("C4", 320, 1280, 4), ("FC", 300, 600, 4)])
@pytest.mark.parametrize("fused_rollout", [True, False])
def test_whole_iteration_bf16_matches_oracle(g, name, n_envs, minibatch, horizon, fused_rollout):
    cfg = syn.get_config(name)
    ref, ses, stats, (shape, theta, env, hp) = _run_iteration_both(g, cfg, n_envs, minibatch, horizon, 2, "bf16",
                                                                   fused_rollout)
    assert rel_l2(ses.state().cpu().numpy(), ref["state"]) <= TOL16
    assert np.array_equal(ses.episode_step.cpu().numpy().astype(np.uint32), ref["episode_step"])
    got = ses.buf.to_numpy()
    rb = ref["buf"]
    assert np.array_equal(got["done"], rb["done"])
    for k in ("obs", "act", "val", "rew", "ret"):
        assert rel_l2(got[k], rb[k]) <= TOL16, (k, rel_l2(got[k], rb[k]))
        assert rel_max(got[k], rb[k]) <= TOL16, (k, rel_max(got[k], rb[k]))
    assert rel_l2(got["logp"], rb["logp"]) <= 1e-5          # noise and log_std only
    assert rel_l2(got["adv"], rb["adv"]) <= 5 * TOL16       # normalised difference of bf16 values
    assert np.abs(stats - ref["stats"]).max() <= 2e-2 * max(1.0, np.abs(ref["stats"]).max())
    # PPO loss of the next forward after the update, same minibatch on both sides: 1e-3 absolute
    flat = oppo.flatten_buffer(rb)
    B = n_envs * horizon
    idx = px.feistel_permutation(B, cfg.seed, 0, 0)[:minibatch]
    r_stats, _ = oppo.ppo_loss_and_grad(ref["theta"], shape, flat["obs"][idx], flat["act"][idx], flat["logp"][idx],
                                        flat["adv"][idx], flat["ret"][idx], hp, want_grad=False)
    # evaluate the HIP path's updated parameters on the oracle's buffer contents
    for k in ("obs", "act", "logp", "adv", "ret"):
        getattr(ses.buf, k).copy_(dev(rb[k]))
    torch.cuda.synchronize()
    out = zeros(5)
    h = g.ppo_hparams(clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, minibatch=minibatch)
    g.ppo_evaluate(ses.gmi, ses.model, ses.buffer, h, dev(idx.astype(np.int32)), minibatch, out)
    ses.sync()
    o = out.cpu().numpy()
    # policy part within 1e-3 absolute; the value part is O(|returns|^2) here, compare it relatively
    assert abs(o[0] - r_stats[0]) <= 1e-3
    assert abs(o[1] - r_stats[1]) <= 1e-3 * max(1.0, abs(r_stats[1]))
    ses.close()


@pytest.mark.parametrize("name,n_envs,horizon,prob_inv", [("C2", 100, 5, 4), ("C3", 257, 4, 0), ("C2", 4096, 16, 0),
                                                          ("C2", 33, 3, 2), ("C2", 6000, 3, 7), ("C4", 700, 3, 5),
                                                          ("SH", 333, 2, 0), ("C4", 5000, 4, 50)])
def test_rollout_collect_equals_the_step_by_step_calls(g, name, n_envs, horizon, prob_inv):
    """One-launch experience collection against agent_act / env_step / collect_experience called per step
    (same kernels' arithmetic, same Philox counters): every array it leaves must be identical, over two
    iterations in a row (state, episode counters and step offsets carry over), ragged last tile included.
    (6000 envs: more 16-env tiles than compute units, so a workgroup takes several tiles in turn.  C4 and SH: models
    beyond the one-launch kernel's size limit, collected with two launches per step.)"""
    import dataclasses
    cfg = syn.get_config(name)
    if prob_inv:
        cfg = dataclasses.replace(cfg, done_period=0, done_prob_inv=prob_inv)
    shape, theta, env, state0, hp = oracle_pieces(cfg, n_envs=n_envs)
    a = make_session(cfg, theta, env, state0, n_envs=n_envs, minibatch=n_envs, horizon=horizon, dtype="bf16",
                     fused_rollout=True)
    b = make_session(cfg, theta, env, state0, n_envs=n_envs, minibatch=n_envs, horizon=horizon, dtype="bf16",
                     fused_rollout=False)
    for it in range(2):
        a.rollout(it)
        b.rollout(it)
        a.sync()
        b.sync()
        assert a.fused_rollout and not b.fused_rollout
        ga, gb = a.buf.to_numpy(), b.buf.to_numpy()
        for k in ("obs", "act", "logp", "val", "rew", "done"):
            assert np.array_equal(ga[k], gb[k]), (it, k, np.abs(ga[k].astype(np.float64) - gb[k]).max())
        assert np.array_equal(a.state().cpu().numpy(), b.state().cpu().numpy())
        assert np.array_equal(a.last_value.cpu().numpy(), b.last_value.cpu().numpy())
        assert np.array_equal(a.episode_step.cpu().numpy(), b.episode_step.cpu().numpy())
    if prob_inv:
        assert 0 < ga["done"].sum() < ga["done"].size
    a.close()
    b.close()


def test_rollout_collect_refuses_fp32_models(g):
    cfg = syn.get_config("C1")
    shape, theta, env, state0, hp = oracle_pieces(cfg)
    ses = make_session(cfg, theta, env, state0, dtype="f32")
    with pytest.raises(g.GmiError) as ei:
        g.rollout_collect(ses.gmi, ses.model, ses.env, ses.buffer, ses.state(), cfg.seed, 0, 0, ses.last_value)
    assert ei.value.code == g.ERR_UNSUPPORTED and "BF16" in str(ei.value)
    ses.close()


# ----------------------------------------------------------------------------- boundary behaviour
def test_error_paths(g, inst):
    with pytest.raises(g.GmiError) as ei:
        g.gmi_create([0, 0, 0, 0, 0, 0, 0, 0])
    assert ei.value.code == g.ERR_INVALID_ARG
    with pytest.raises(g.GmiError) as ei:
        g.gmi_create(None, device=99)
    assert ei.value.code == g.ERR_INVALID_ARG
    with pytest.raises(g.GmiError) as ei:
        g.gmi_sync(0)
    assert ei.value.code == g.ERR_BAD_HANDLE
    cfg = syn.get_config("C1")
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, 0)
    hm, keep = _bind_model(g, inst, cfg, theta, 64, "f32", with_adam=False)
    obs = zeros(128, cfg.obs_dim)
    with pytest.raises(g.GmiError) as ei:     # more rows than the binding allows
        g.agent_act(inst, hm, obs, 128, 0, 0, 0, zeros(128, 2), zeros(128), zeros(128))
    assert ei.value.code == g.ERR_BAD_SHAPE
    g.agent_act(inst, hm, obs, 0, 0, 0, 0, None, None, None)       # empty input is a no-op
    b, rb, hb = _filled_buffer(g, inst, cfg, 4, 16, seed=0)
    with pytest.raises(g.GmiError) as ei:     # inference-only binding cannot train
        g.ppo_update(inst, hm, hb, g.ppo_hparams(minibatch=32))
    assert ei.value.code == g.ERR_INVALID_ARG
    g.gmi_model_destroy(hm)
    hm, keep = _bind_model(g, inst, cfg, theta, 64, "f32")
    with pytest.raises(g.GmiError) as ei:     # minibatch must divide the batch
        g.ppo_update(inst, hm, hb, g.ppo_hparams(minibatch=48))
    assert ei.value.code == g.ERR_BAD_SHAPE
    g.gmi_model_destroy(hm)
    with pytest.raises(g.GmiError) as ei:
        g.gmi_model_destroy(hm)               # double destroy
    assert ei.value.code == g.ERR_BAD_HANDLE
    g.gmi_buffer_destroy(hb)


def test_wait_stream_orders_the_instance_behind_a_caller_stream(g, inst):
    """Data produced on a stream of the caller, consumed by the instance with no host synchronisation between:
    gmi_wait_stream makes the instance's copy wait for the fills queued before it."""
    side = torch.cuda.Stream()
    n = 1 << 26
    dst = torch.zeros(n, device="cuda:0")
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        src = torch.empty(n, device="cuda:0")
        for k in range(8):                       # a few hundred microseconds of work on the caller's stream
            src.fill_(float(k))
        src.add_(1.0)
    g.gmi_wait_stream(inst, side)
    g.gmi_transfer(inst, inst, src, dst, n * 4)
    g.gmi_sync(inst)
    assert bool((dst == 8.0).all().item())
    side.synchronize()
    with pytest.raises(g.GmiError):
        g.gmi_wait_stream(0, side)


def test_masked_instances_and_transfer(g):
    full = g.gmi_create()
    n_cu = g.gmi_cu_count(full)
    words = (n_cu + 31) // 32
    half = [0xFFFFFFFF if w < words // 2 else 0 for w in range(words)]
    other = [0 if w < words // 2 else 0xFFFFFFFF for w in range(words)]
    if n_cu % 32:
        other[-1] = (1 << (n_cu % 32)) - 1
    a, b = g.gmi_create(half), g.gmi_create(other)
    assert g.gmi_cu_count(a) + g.gmi_cu_count(b) == n_cu
    # producer on instance a, consumer on instance b, ordered only by gmi_transfer
    n = 1 << 16
    src, dst = zeros(n, 8), zeros(n, 8)
    out = zeros(n, 8)
    for rep in range(3):
        g.gmi_noise_fill(a, 5, 1, rep, 0, n, 8, src)
        g.gmi_transfer(a, b, src, dst, src.numel() * 4)
        g.gmi_transfer(b, b, dst, out, dst.numel() * 4)
        g.gmi_sync(b)
        assert np.array_equal(out.cpu().numpy(), px.normal_field(5, 1, rep, n, 8))
        g.gmi_transfer(b, a, None, None, 0)       # ordering only: a may overwrite src again
    # a mask that leaves an accelerator die (bit index mod 8) without any CU is refused cleanly
    with pytest.raises(g.GmiError) as ei:
        g.gmi_create([0x55555555] * words)
    assert ei.value.code == g.ERR_INVALID_ARG
    for h in (a, b, full):
        g.gmi_destroy(h)
