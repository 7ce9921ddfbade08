"""Oracle, error model of the bf16 path (test infrastructure only).

The problem statement's reduced-precision path keeps weights and activations in bf16, multiplies them on the
matrix cores with fp32 accumulation, and keeps biases, loss arithmetic, the master parameters and Adam in fp32.
Its result differs from the fp32 oracle's (``oracle.ppo``) by rounding alone.  This module writes that rounding
out: the same network and the same backward pass as ``oracle.ppo``, with every value that the reduced-precision
path holds in bf16 rounded to bf16 (round to nearest, ties to even) at the point where it is stored, and every
sum accumulated in fp32.  A HIP result that agrees with the fp32 oracle only within the 2e-2 band but misses
this model by more than accumulation-order noise has an error that is not rounding.

What is rounded: the observation rows; the weights (not the biases); every hidden activation
h_l = ELU(h_{l-1} W_l^T + b_l) after the fp32 bias and ELU; the gradient at the head's output; every gradient
dz_{l-1} = (dz_l W_l) * ELU'(h_l) after the fp32 product with ELU' taken from the stored (rounded) h_l.
What is not: the heads' outputs, the loss, log-std and its gradient, the weight and bias gradients (fp32 sums of
products of rounded values).
"""
from __future__ import annotations

import numpy as np

from . import ppo as oppo


def round_bf16(x):
    """float32 -> nearest bf16 (ties to even), returned as float32.  bf16 is the upper 16 bits of the float32
    encoding: add 0x7FFF plus the lowest kept bit, then clear the lower 16 bits.  NaN stays NaN."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
    out = r.view(np.float32).reshape(a.shape)
    return np.where(np.isnan(a), a, out)


def mlp_forward(x, layers):
    """``oracle.ppo.mlp_forward`` with bf16 storage: returns (head output fp32, [h_0 .. h_L] as stored)."""
    h = round_bf16(x)
    acts = [h]
    for w, b in layers[:-1]:
        z = h @ round_bf16(w).T + b.astype(np.float32)
        h = round_bf16(oppo.elu(z).astype(np.float32))
        acts.append(h)
    w, b = layers[-1]
    return (h @ round_bf16(w).T + b.astype(np.float32)).astype(np.float32), acts


def mlp_backward(d_out, acts, layers):
    """``oracle.ppo.mlp_backward`` with bf16 storage of the layer gradients."""
    grads = [None] * len(layers)
    d = round_bf16(d_out)
    for l in range(len(layers) - 1, -1, -1):
        w, _ = layers[l]
        grads[l] = ((d.T @ acts[l]).astype(np.float32), d.sum(axis=0, dtype=np.float32))
        if l > 0:
            h = acts[l]
            d = round_bf16((d @ round_bf16(w)) * np.where(h > 0, np.float32(1), h + np.float32(1)))
    return grads


def agent_forward(theta, shape: oppo.ModelShape, obs):
    """Policy means [N, A] and values [N] of the bf16 path."""
    pol, val, _ = oppo.unpack(theta.astype(np.float32), shape)
    mu, _ = mlp_forward(obs.astype(np.float32), pol)
    v, _ = mlp_forward(obs.astype(np.float32), val)
    return mu, v[:, 0]


def ppo_loss_and_grad(theta, shape: oppo.ModelShape, obs, act, logp_old, adv, ret, hp: oppo.PPOHyper):
    """``oracle.ppo.ppo_loss_and_grad`` (same loss, same statistics, same gradient layout) through the bf16
    forward and backward above; everything between the heads' outputs and the heads' gradients is fp32."""
    f = np.float32
    theta = theta.astype(f)
    obs, act = obs.astype(f), act.astype(f)
    logp_old, adv, ret = logp_old.astype(f), adv.astype(f), ret.astype(f)
    pol, val, log_std = oppo.unpack(theta, shape)
    m = obs.shape[0]
    mu, acts_p = mlp_forward(obs, pol)
    v, acts_v = mlp_forward(obs, val)
    v = v[:, 0]
    inv_sigma = np.exp(-log_std)
    z = (act - mu) * inv_sigma
    logp = (-0.5 * z * z - log_std - f(0.5 * oppo.LOG_2PI)).sum(axis=1)
    ratio = np.exp(logp - logp_old)
    s1 = ratio * adv
    s2 = np.clip(ratio, f(1.0 - hp.clip), f(1.0 + hp.clip)) * adv
    stats = np.array([-np.minimum(s1, s2).mean(), ((v - ret) ** 2).mean(),
                      (log_std + f(0.5 * (1.0 + oppo.LOG_2PI))).sum(), (logp_old - logp).mean(),
                      (np.abs(ratio - 1) > f(hp.clip)).mean()], dtype=f)
    g_logp = -(adv * ratio * (s1 <= s2).astype(f)) / f(m)
    d_mu = g_logp[:, None] * z * inv_sigma
    d_logstd = (g_logp[:, None] * (z * z - 1)).sum(axis=0) - f(hp.c_e)
    d_v = (f(2.0 * hp.c_v) * (v - ret) / f(m))[:, None]
    parts = []
    for net in (mlp_backward(d_mu, acts_p, pol), mlp_backward(d_v, acts_v, val)):
        for dw, db in net:
            parts.append(dw.reshape(-1))
            parts.append(db)
    parts.append(d_logstd)
    return stats, np.concatenate(parts).astype(f)
