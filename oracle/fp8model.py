"""Oracle of the fp8 inference path (test infrastructure only).

Agents that only serve (Section 3 of the paper: the agent role needs the forward pass alone; the paper's workload
table leaves their precision open) may hold weights and activations in 8-bit floating point.  This module writes
out what that path computes: the network of ``oracle.ppo`` with

  * weights of every layer divided by a power-of-two scale s_l (the smallest power of two with max|W_l| / s_l <= 448)
    and rounded to E4M3;
  * the observation and every hidden activation rounded to E4M3 (no scale) where it is stored;
  * products summed without further rounding (float64 here; the device sums in fp32), then multiplied by s_l, the
    fp32 bias added, ELU in fp32; the heads' outputs stay fp32.

E4M3 is the 8-bit format of the OCP 8-bit floating point specification: 1 sign, 4 exponent bits (bias 7), 3
mantissa bits, subnormals, no infinities, one NaN pattern per sign (exponent and mantissa all ones), largest finite
value 448.  Rounding is to nearest, ties to even, and saturating: magnitudes above 448 become 448.
"""
from __future__ import annotations

import numpy as np

from . import philox as px
from . import ppo as oppo

E4M3_MAX = 448.0
E4M3_MIN_NORMAL_EXP = -6        # smallest normal 2^-6; subnormals are multiples of 2^-9


def decode_e4m3(code: int) -> float:
    """Value of an 8-bit pattern, from the bit fields."""
    s = -1.0 if code & 0x80 else 1.0
    e = (code >> 3) & 0xF
    m = code & 0x7
    if e == 0xF and m == 0x7:
        return float("nan")
    if e == 0:
        return s * m * 2.0 ** (1 - 7 - 3)
    return s * (1.0 + m / 8.0) * 2.0 ** (e - 7)


def round_e4m3(x):
    """Nearest E4M3 value (ties to even, saturating), as float32.  The spacing of the format at |x| is
    2^(floor(log2|x|) - 3), and 2^-9 below the smallest normal; |x| is rounded to a multiple of it."""
    a = np.asarray(x, dtype=np.float64)
    mag = np.abs(a)
    _, ex = np.frexp(mag)                       # mag = m * 2^ex with m in [0.5, 1)
    e = np.maximum(ex - 1, E4M3_MIN_NORMAL_EXP)
    q = np.ldexp(1.0, e - 3)
    r = np.minimum(np.rint(mag / q) * q, E4M3_MAX)     # np.rint: halves to even
    return (np.sign(a) * r).astype(np.float32)


def layer_scale(w) -> float:
    """The smallest power of two s with max|w| / s <= 448 (1 for an all-zero matrix)."""
    m = float(np.max(np.abs(w))) if w.size else 0.0
    if m == 0.0:
        return 1.0
    return float(2.0 ** np.ceil(np.log2(m / E4M3_MAX)))


def quantise_weights(w):
    """(E4M3 values of w / s as float32, s)."""
    s = layer_scale(w)
    return round_e4m3(np.asarray(w, np.float64) / s), s


def mlp_forward(x, layers):
    """``oracle.ppo.mlp_forward`` with E4M3 storage of weights and activations; returns the head's output."""
    h = round_e4m3(x).astype(np.float64)
    for w, b in layers[:-1]:
        wq, s = quantise_weights(w)
        z = (s * (h @ wq.astype(np.float64).T)).astype(np.float32) + b.astype(np.float32)
        h = round_e4m3(oppo.elu(z).astype(np.float32)).astype(np.float64)
    w, b = layers[-1]
    wq, s = quantise_weights(w)
    return ((s * (h @ wq.astype(np.float64).T)).astype(np.float32) + b.astype(np.float32)).astype(np.float32)


def agent_forward(theta, shape: oppo.ModelShape, obs):
    """Policy means [N, A] and values [N] of the fp8 path."""
    pol, val, _ = oppo.unpack(theta.astype(np.float32), shape)
    mu = mlp_forward(obs.astype(np.float32), pol)
    v = mlp_forward(obs.astype(np.float32), val)
    return mu, v[:, 0]


def agent_act(theta, shape: oppo.ModelShape, obs, seed: int, step: int, env_offset: int = 0):
    """``oracle.ppo.agent_act`` with the means and values of the fp8 path: the same noise, the same fp32
    sampling and log-density.  Returns act [N,A], logp [N], value [N], mu [N,A]."""
    f = np.float32
    _, _, log_std = oppo.unpack(theta.astype(f), shape)
    mu, v = agent_forward(theta, shape, obs)
    eps = px.normal_field(seed, px.STREAM_ACTION, step, obs.shape[0], shape.act_dim, env_offset).astype(f)
    act = mu + np.exp(log_std) * eps
    logp = (-0.5 * eps * eps - log_std - f(0.5 * oppo.LOG_2PI)).sum(axis=1)
    return act, logp.astype(f), v, mu
