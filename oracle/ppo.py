"""Oracle: the PPO agent/trainer step on the CPU (test infrastructure only).

Roles as in the paper's Section 3: the *environment simulator* returns new states and rewards for
the actions it receives, the *agent* decides actions from states and records experience (state,
action, reward), the *trainer* runs forward and backward over the experience and updates the
policy.  Stages as in Section 5.1 (synchronized training): (i) experience collection for a fixed
number of interactions, (ii) model training.  The paper prints no formulas for any of these; each
function cites the public definition it writes out.

All functions take a numpy ``dtype`` (float32 is the oracle the HIP path is compared with;
float64 serves the pins: finite differences, closed forms, comparisons with independent
libraries).  Random numbers are never drawn from global state: they are functions of
(seed, stream, step, env, element) through ``oracle.philox``.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

from . import philox as px

LOG_2PI = math.log(2.0 * math.pi)


# ----------------------------------------------------------------------------------------------
# Model: two separate MLPs (policy, value) with ELU hidden layers and linear heads, plus a
# state-independent log-std vector.  Shapes follow the paper's Table 6 ("in:h1:..:out"); separate
# trunks are what reproduces Table 7's parameter counts.
# ----------------------------------------------------------------------------------------------
@dataclass
class ModelShape:
    obs_dim: int
    act_dim: int
    hidden: Tuple[int, ...]

    def layer_dims(self, out_dim: int) -> List[Tuple[int, int]]:
        dims, prev = [], self.obs_dim
        for h in self.hidden:
            dims.append((prev, h))
            prev = h
        dims.append((prev, out_dim))
        return dims

    def n_params(self) -> int:
        n = self.act_dim
        for out_dim in (self.act_dim, 1):
            n += sum(i * o + o for i, o in self.layer_dims(out_dim))
        return n


def unpack(theta: np.ndarray, shape: ModelShape):
    """Views into the flat vector: (policy layers [(W,b)...], value layers [(W,b)...], log_std).
    Layout: policy W0,b0,..,W_L,b_L, value W0,b0,..,W_L,b_L, log_std;  W is [out, in] row-major."""
    off = 0
    nets = []
    for out_dim in (shape.act_dim, 1):
        layers = []
        for i, o in shape.layer_dims(out_dim):
            w = theta[off:off + i * o].reshape(o, i)
            off += i * o
            b = theta[off:off + o]
            off += o
            layers.append((w, b))
        nets.append(layers)
    log_std = theta[off:off + shape.act_dim]
    off += shape.act_dim
    assert off == theta.size
    return nets[0], nets[1], log_std


def elu(z):
    """ELU with alpha = 1:  z for z > 0, exp(z) - 1 otherwise."""
    return np.where(z > 0, z, np.expm1(np.minimum(z, 0)))


def mlp_forward(x, layers):
    """h_0 = x; h_l = ELU(h_{l-1} W_l^T + b_l) for hidden layers; linear head.
    Returns (head output, [h_0, h_1, ..., h_L])."""
    acts = [x]
    h = x
    for w, b in layers[:-1]:
        h = elu(h @ w.T + b)
        acts.append(h)
    w, b = layers[-1]
    return h @ w.T + b, acts


def mlp_backward(d_out, acts, layers):
    """Exact reverse-mode derivative of ``mlp_forward``: given dL/d(head output) returns the list
    [(dW_l, db_l)].  ELU'(z) expressed through the stored output h = ELU(z): 1 if h > 0 else h + 1."""
    grads = [None] * len(layers)
    d = d_out
    for l in range(len(layers) - 1, -1, -1):
        w, _ = layers[l]
        grads[l] = (d.T @ acts[l], d.sum(axis=0))
        if l > 0:
            h = acts[l]
            d = (d @ w) * np.where(h > 0, np.ones_like(h), h + 1)
    return grads


# ----------------------------------------------------------------------------------------------
# Agent: action decision (Section 3, "DRL Agent").
# ----------------------------------------------------------------------------------------------
def agent_act(theta, shape: ModelShape, obs, seed: int, step: int, dtype=np.float32,
              env_offset: int = 0):
    """mu = pi(obs); value = V(obs); eps ~ N(0,1) from Philox stream 0;
    act = mu + exp(log_std) * eps;  logp = sum_j [-eps_j^2/2 - log_std_j - ln(2 pi)/2]
    (the diagonal-Gaussian log-density evaluated at the sampled action).
    Returns act [N,A], logp [N], value [N], mu [N,A]."""
    theta = theta.astype(dtype)
    obs = obs.astype(dtype)
    pol, val, log_std = unpack(theta, shape)
    mu, _ = mlp_forward(obs, pol)
    v, _ = mlp_forward(obs, val)
    eps = px.normal_field(seed, px.STREAM_ACTION, step, obs.shape[0], shape.act_dim,
                          env_offset).astype(dtype)
    act = mu + np.exp(log_std) * eps
    logp = (-0.5 * eps * eps - log_std - dtype(0.5 * LOG_2PI)).sum(axis=1)
    return act, logp.astype(dtype), v[:, 0], mu


def value_only(theta, shape: ModelShape, obs, dtype=np.float32):
    """V(obs): the bootstrap value of the state reached after the last collected step."""
    _, val, _ = unpack(theta.astype(dtype), shape)
    v, _ = mlp_forward(obs.astype(dtype), val)
    return v[:, 0]


# ----------------------------------------------------------------------------------------------
# Environment simulator (Section 3, "DRL Environment Simulator"): the synthetic stand-in.
# ----------------------------------------------------------------------------------------------
@dataclass
class EnvSpec:
    a_mat: np.ndarray          # [O,O]
    b_mat: np.ndarray          # [O,A]
    noise_std: float
    reward_scale: float
    done_period: int           # >0: periodic done
    done_threshold: int        # used when done_period == 0: done iff philox word < threshold
    seed: int


def done_threshold_from_inverse(prob_inv: int) -> int:
    """Integer threshold for 'done with probability 1/prob_inv': floor(2^32 / prob_inv)."""
    return (1 << 32) // prob_inv if prob_inv > 0 else 0


def env_step(env: EnvSpec, state, act, episode_step, step: int, dtype=np.float32,
             env_offset: int = 0):
    """One transition of every environment.

        s' = s A^T + a B^T + noise_std * xi          xi ~ N(0,1), Philox stream 1
        r  = reward_scale * (-|s|^2 - 0.01 |a|^2)    (pre-step state and the action taken)
        done: periodic, (episode_step + 1) % period == 0, or Bernoulli by the integer compare
              philox_word(stream 2) < done_threshold
        where done: s' <- fresh N(0,1) draw (Philox stream 3) and episode_step <- 0

    Returns (next_state [N,O], reward [N], done [N] uint8, next_episode_step [N] uint32)."""
    state = state.astype(dtype)
    act = act.astype(dtype)
    n, o = state.shape
    xi = px.normal_field(env.seed, px.STREAM_ENV, step, n, o, env_offset).astype(dtype)
    nxt = state @ env.a_mat.astype(dtype).T + act @ env.b_mat.astype(dtype).T \
        + dtype(env.noise_std) * xi
    rew = dtype(env.reward_scale) * (-(state * state).sum(axis=1)
                                     - dtype(0.01) * (act * act).sum(axis=1))
    if env.done_period > 0:
        done = ((episode_step.astype(np.uint64) + 1) % np.uint64(env.done_period)) == 0
    else:
        done = px.done_words(env.seed, step, n, env_offset) < np.uint32(env.done_threshold)
    reset = px.normal_field(env.seed, px.STREAM_RESET, step, n, o, env_offset).astype(dtype)
    nxt = np.where(done[:, None], reset, nxt)
    next_ep = np.where(done, 0, episode_step.astype(np.uint64) + 1).astype(np.uint32)
    return nxt.astype(dtype), rew.astype(dtype), done.astype(np.uint8), next_ep


# ----------------------------------------------------------------------------------------------
# Experience (Section 3: state, action, reward vectors; one array per type).
# ----------------------------------------------------------------------------------------------
def new_buffer(T: int, N: int, O: int, A: int, dtype=np.float32) -> dict:
    return {
        "obs": np.zeros((T, N, O), dtype), "act": np.zeros((T, N, A), dtype),
        "logp": np.zeros((T, N), dtype), "val": np.zeros((T, N), dtype),
        "rew": np.zeros((T, N), dtype), "done": np.zeros((T, N), np.uint8),
        "adv": np.zeros((T, N), dtype), "ret": np.zeros((T, N), dtype),
    }


def collect_experience(buf: dict, t: int, obs, act, logp, val, rew, done, col0: int = 0):
    """Store step t's experience (time-major buffer, envs [col0, col0+n))."""
    n = obs.shape[0]
    sl = slice(col0, col0 + n)
    buf["obs"][t, sl] = obs
    buf["act"][t, sl] = act
    buf["logp"][t, sl] = logp
    buf["val"][t, sl] = val
    buf["rew"][t, sl] = rew
    buf["done"][t, sl] = done


def rollout(theta, shape: ModelShape, env: EnvSpec, state, episode_step, buf: dict, seed: int,
            iteration: int, dtype=np.float32, col0: int = 0, env_offset: int = 0):
    """Stage (i) of Section 5.1: T rounds of [agent decides -> environment steps -> store].
    Global step index of round t is iteration*T + t.  Returns (state, episode_step, last_value)."""
    T = buf["obs"].shape[0]
    for t in range(T):
        step = iteration * T + t
        act, logp, val, _ = agent_act(theta, shape, state, seed, step, dtype, env_offset)
        nxt, rew, done, episode_step = env_step(env, state, act, episode_step, step, dtype,
                                                env_offset)
        collect_experience(buf, t, state, act, logp, val, rew, done, col0)
        state = nxt
    return state, episode_step, value_only(theta, shape, state, dtype)


# ----------------------------------------------------------------------------------------------
# Generalized advantage estimation (Schulman et al. 2016, eq. 16 with termination masks).
# ----------------------------------------------------------------------------------------------
def gae(rew, val, done, last_val, gamma: float, lam: float, normalize: bool, dtype=np.float32):
    """delta_t = r_t + gamma v_{t+1} (1 - d_t) - v_t,   v_T = last_val
       A_t = delta_t + gamma lam (1 - d_t) A_{t+1},     A_T = 0
       R_t = A_t + v_t
       normalize: A <- (A - mean A) / (std A + 1e-8) over the whole batch (population std).
    Inputs are [T,N]; returns (adv, ret)."""
    rew = rew.astype(dtype)
    val = val.astype(dtype)
    T = rew.shape[0]
    nd = (1 - done.astype(dtype))
    adv = np.zeros_like(rew)
    nxt_adv = np.zeros_like(rew[0])
    nxt_val = last_val.astype(dtype)
    g, gl = dtype(gamma), dtype(gamma * lam)
    for t in range(T - 1, -1, -1):
        delta = rew[t] + g * nxt_val * nd[t] - val[t]
        nxt_adv = delta + gl * nd[t] * nxt_adv
        adv[t] = nxt_adv
        nxt_val = val[t]
    ret = adv + val
    if normalize:
        adv = (adv - adv.mean()) / (adv.std() + dtype(1e-8))
    return adv.astype(dtype), ret.astype(dtype)


# ----------------------------------------------------------------------------------------------
# Trainer: clipped-surrogate loss, exact backward, Adam (Section 3, "DRL Trainer").
# ----------------------------------------------------------------------------------------------
@dataclass
class PPOHyper:
    clip: float = 0.2
    c_v: float = 0.5
    c_e: float = 0.0
    lr: float = 3e-4
    beta1: float = 0.9
    beta2: float = 0.999
    adam_eps: float = 1e-8
    epochs: int = 1
    minibatch: int = 256


def ppo_loss_and_grad(theta, shape: ModelShape, obs, act, logp_old, adv, ret, hp: PPOHyper,
                      dtype=np.float32, want_grad: bool = True):
    """PPO clipped-surrogate objective (Schulman et al. 2017, eq. 7 and 9) on one minibatch.

        logp   = sum_j [-((a_j - mu_j)/sigma_j)^2 / 2 - log_std_j - ln(2 pi)/2]
        ratio  = exp(logp - logp_old)
        L_pi   = -mean(min(ratio * A, clip(ratio, 1-c, 1+c) * A))
        L_v    = mean((V - R)^2)
        H      = sum_j [log_std_j + (1 + ln(2 pi))/2]        (state independent)
        L      = L_pi + c_v L_v - c_e H

    Returns (stats, grad) with stats = [L_pi, L_v, H, approx_kl = mean(logp_old - logp),
    clip_fraction = mean(|ratio - 1| > c)] and grad the flat dL/dtheta (None if not wanted).
    The surrogate's derivative w.r.t. logp is -A*ratio/M where the unclipped term is the minimum
    (ratio*A <= clipped*A) and 0 otherwise."""
    theta = theta.astype(dtype)
    obs, act = obs.astype(dtype), act.astype(dtype)
    logp_old, adv, ret = logp_old.astype(dtype), adv.astype(dtype), ret.astype(dtype)
    pol, val, log_std = unpack(theta, shape)
    m = obs.shape[0]
    mu, acts_p = mlp_forward(obs, pol)
    v, acts_v = mlp_forward(obs, val)
    v = v[:, 0]
    inv_sigma = np.exp(-log_std)
    z = (act - mu) * inv_sigma
    logp = (-0.5 * z * z - log_std - dtype(0.5 * LOG_2PI)).sum(axis=1)
    ratio = np.exp(logp - logp_old)
    s1 = ratio * adv
    s2 = np.clip(ratio, dtype(1.0 - hp.clip), dtype(1.0 + hp.clip)) * adv
    l_pi = -np.minimum(s1, s2).mean()
    l_v = ((v - ret) ** 2).mean()
    ent = (log_std + dtype(0.5 * (1.0 + LOG_2PI))).sum()
    kl = (logp_old - logp).mean()
    clipfrac = (np.abs(ratio - 1) > dtype(hp.clip)).mean()
    stats = np.array([l_pi, l_v, ent, kl, clipfrac], dtype=dtype)
    if not want_grad:
        return stats, None
    active = (s1 <= s2).astype(dtype)
    g_logp = -(adv * ratio * active) / dtype(m)                       # dL/dlogp   [M]
    d_mu = g_logp[:, None] * z * inv_sigma                            # dlogp/dmu_j = z_j / sigma_j
    d_logstd = (g_logp[:, None] * (z * z - 1)).sum(axis=0) - dtype(hp.c_e)
    d_v = (dtype(2.0 * hp.c_v) * (v - ret) / dtype(m))[:, None]
    gp = mlp_backward(d_mu, acts_p, pol)
    gv = mlp_backward(d_v, acts_v, val)
    parts = []
    for net in (gp, gv):
        for dw, db in net:
            parts.append(dw.reshape(-1))
            parts.append(db)
    parts.append(d_logstd)
    return stats, np.concatenate(parts).astype(dtype)


def total_loss(stats, hp: PPOHyper):
    return stats[0] + hp.c_v * stats[1] - hp.c_e * stats[2]


def adam_step(theta, m, v, grad, k: int, hp: PPOHyper, dtype=np.float32):
    """Adam (Kingma & Ba 2015, Algorithm 1), epsilon outside the square root, no weight decay:
        m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2
        theta <- theta - lr * (m / (1 - b1^k)) / (sqrt(v / (1 - b2^k)) + eps),   k = 1, 2, ...
    Returns new (theta, m, v)."""
    g = grad.astype(dtype)
    b1, b2 = dtype(hp.beta1), dtype(hp.beta2)
    m = b1 * m.astype(dtype) + (1 - b1) * g
    v = b2 * v.astype(dtype) + (1 - b2) * g * g
    c1 = dtype(1.0 - hp.beta1 ** k)
    c2 = dtype(1.0 - hp.beta2 ** k)
    theta = theta.astype(dtype) - dtype(hp.lr) * (m / c1) / (np.sqrt(v / c2) + dtype(hp.adam_eps))
    return theta.astype(dtype), m.astype(dtype), v.astype(dtype)


def flatten_buffer(buf: dict):
    """[T,N,...] -> [T*N,...]; sample index = t*N + env."""
    T, N = buf["logp"].shape
    fields = ("obs", "act", "logp", "val", "rew", "done", "adv", "ret")
    return {k: buf[k].reshape(T * N, *buf[k].shape[2:]) for k in fields if k in buf}


def ppo_update(theta, m, v, k0: int, shape: ModelShape, buf: dict, hp: PPOHyper, seed: int,
               iteration: int, dtype=np.float32):
    """Stage (ii) of Section 5.1.  For each epoch: a seeded permutation of the B = T*N samples
    (``feistel_permutation``), consecutive slices of ``hp.minibatch`` samples are the minibatches,
    each gives one loss/backward/Adam step.  ``k0`` = number of Adam steps taken before this call.
    Returns (theta, m, v, k, stats[epochs * n_minibatches, 5])."""
    flat = flatten_buffer(buf)
    B = flat["logp"].shape[0]
    assert B % hp.minibatch == 0
    nmb = B // hp.minibatch
    stats = []
    k = k0
    for e in range(hp.epochs):
        perm = px.feistel_permutation(B, seed, iteration, e)
        for j in range(nmb):
            idx = perm[j * hp.minibatch:(j + 1) * hp.minibatch]
            st, g = ppo_loss_and_grad(theta, shape, flat["obs"][idx], flat["act"][idx],
                                      flat["logp"][idx], flat["adv"][idx], flat["ret"][idx],
                                      hp, dtype)
            k += 1
            theta, m, v = adam_step(theta, m, v, g, k, hp, dtype)
            stats.append(st)
    return theta, m, v, k, np.stack(stats)


def ppo_update_group(theta, m, v, k0: int, shape: ModelShape, bufs, hp: PPOHyper, seed: int,
                     iteration: int, dtype=np.float32):
    """Synchronized training of several trainer instances that hold replicas of one model (Section 4.1:
    the replicas' gradients are reduced so that every replica applies the same update; with the instances
    of one GPU sharing an address space the reduction is a plain in-memory mean).

    Instance i owns buffer bufs[i] (all of the same size) and shuffles it with its own permutation, keyed
    by seed + i.  Minibatch j of an epoch is the union of the instances' j-th slices of ``hp.minibatch``
    samples each; its gradient is the mean of the instances' minibatch-mean gradients, followed by one
    Adam step on the shared parameters.  Statistics are the mean over the instances.
    Returns (theta, m, v, k, stats[epochs * n_minibatches, 5])."""
    flats = [flatten_buffer(b) for b in bufs]
    B = flats[0]["logp"].shape[0]
    assert all(f["logp"].shape[0] == B for f in flats) and B % hp.minibatch == 0
    n = len(flats)
    nmb = B // hp.minibatch
    stats = []
    k = k0
    for e in range(hp.epochs):
        perms = [px.feistel_permutation(B, seed + i, iteration, e) for i in range(n)]
        for j in range(nmb):
            g_sum = None
            st_sum = np.zeros(5, np.float64)
            for i, f in enumerate(flats):
                idx = perms[i][j * hp.minibatch:(j + 1) * hp.minibatch]
                st, g = ppo_loss_and_grad(theta, shape, f["obs"][idx], f["act"][idx], f["logp"][idx],
                                          f["adv"][idx], f["ret"][idx], hp, dtype)
                g_sum = g.astype(np.float64) if g_sum is None else g_sum + g
                st_sum += st
            k += 1
            theta, m, v = adam_step(theta, m, v, (g_sum / n).astype(dtype), k, hp, dtype)
            stats.append((st_sum / n).astype(dtype))
    return theta, m, v, k, np.stack(stats)


def ppo_iteration(theta, m, v, k0, shape: ModelShape, env: EnvSpec, state, episode_step,
                  T: int, hp: PPOHyper, gamma: float, lam: float, seed: int, iteration: int,
                  normalize: bool = True, dtype=np.float32):
    """One whole iteration: rollout, bootstrap value, GAE, update.
    Returns dict with the new trainer state, env state, the filled buffer and the stats."""
    N, O = state.shape
    buf = new_buffer(T, N, O, shape.act_dim, dtype)
    state, episode_step, last_val = rollout(theta, shape, env, state, episode_step, buf, seed,
                                            iteration, dtype)
    buf["adv"], buf["ret"] = gae(buf["rew"], buf["val"], buf["done"], last_val, gamma, lam,
                                 normalize, dtype)
    theta, m, v, k, stats = ppo_update(theta, m, v, k0, shape, buf, hp, seed, iteration, dtype)
    return {"theta": theta, "m": m, "v": v, "k": k, "state": state, "episode_step": episode_step,
            "buf": buf, "last_val": last_val, "stats": stats}
