"""Helpers of the GPU parity tests: oracle-side and HIP-side objects for one workload."""
import numpy as np

from oracle import ppo as oppo
from workloads import synthetic as syn


def rel_l2(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(x - ref) / den) if den > 0 else float(np.linalg.norm(x - ref))


def rel_max(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max()
    return float(np.abs(x - ref).max() / den) if den > 0 else float(np.abs(x - ref).max())


def oracle_pieces(cfg, n_envs=None, seed=None):
    n = cfg.n_envs if n_envs is None else n_envs
    seed = cfg.seed if seed is None else seed
    shape = oppo.ModelShape(cfg.obs_dim, cfg.act_dim, tuple(cfg.hidden))
    theta = syn.make_model_params(cfg.obs_dim, cfg.act_dim, cfg.hidden, seed)
    a_mat, b_mat = syn.make_env_matrices(cfg.obs_dim, cfg.act_dim, seed)
    thr = oppo.done_threshold_from_inverse(cfg.done_prob_inv)
    env = oppo.EnvSpec(a_mat, b_mat, cfg.noise_std, cfg.reward_scale, cfg.done_period, thr, seed)
    state0 = syn.make_initial_state(n, cfg.obs_dim, seed)
    hp = oppo.PPOHyper(clip=cfg.clip, c_v=cfg.c_v, c_e=cfg.c_e, lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2,
                       adam_eps=cfg.adam_eps, epochs=cfg.epochs, minibatch=cfg.minibatch)
    return shape, theta, env, state0, hp


def make_session(cfg, theta, env, state0, n_envs=None, minibatch=None, horizon=None, dtype=None,
                 fused_rollout=True):
    from paper_2206_08482_amd.runner import PPOSession
    n = cfg.n_envs if n_envs is None else n_envs
    return PPOSession(n_envs=n, obs_dim=cfg.obs_dim, act_dim=cfg.act_dim, hidden=cfg.hidden,
                      horizon=cfg.horizon if horizon is None else horizon,
                      dtype=cfg.dtype if dtype is None else dtype, theta=theta, a_mat=env.a_mat,
                      b_mat=env.b_mat, state0=state0, noise_std=env.noise_std, reward_scale=env.reward_scale,
                      done_period=env.done_period, done_threshold=env.done_threshold, seed=env.seed,
                      minibatch=cfg.minibatch if minibatch is None else minibatch, fused_rollout=fused_rollout)
