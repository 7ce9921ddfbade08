"""Oracle: counter-based random numbers (test infrastructure only).

* ``philox4x32_10``      -- the Philox4x32 generator with 10 rounds (Salmon, Moraes, Dror, Shaw,
                            "Parallel random numbers: as easy as 1, 2, 3", SC'11), written from the
                            round definition in that paper.
* ``normal_pair``        -- Box-Muller map from two 32-bit words to two standard normals, written
                            only with integer operations and individually rounded fp32
                            add / multiply / divide / sqrt so that a second implementation of the
                            same written specification reproduces it bit for bit.
* ``normal_field``       -- the [n_env, dim] noise array for one (seed, stream, step).

Counter convention (all uint32):  counter = (env index, step, stream id, block),
key = (seed low word, seed high word).  Element j of a per-env vector uses block j // 4;
inside a block words (0,1) make normals 0,1 and words (2,3) make normals 2,3.
Stream ids: 0 action noise, 1 environment noise, 2 done draw, 3 reset state, 4 minibatch shuffle.
"""
from __future__ import annotations

import numpy as np

STREAM_ACTION = 0
STREAM_ENV = 1
STREAM_DONE = 2
STREAM_RESET = 3
STREAM_SHUFFLE = 4

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten Philox4x32 rounds.  Inputs broadcast against each other; returns four uint32 arrays.

    One round maps (c0,c1,c2,c3) with round key (k0,k1) to
        (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0))
    and the key is advanced by the Weyl constants (W0, W1) between rounds.
    """
    c0, c1, c2, c3 = np.broadcast_arrays(*(np.asarray(c, dtype=np.uint64) & _MASK
                                           for c in (c0, c1, c2, c3)))
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK
        hi1, lo1 = p1 >> _SH32, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def seed_key(seed: int):
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    return seed & 0xFFFFFFFF, seed >> 32


def _f32(hexstr: str) -> np.float32:
    return np.float32(float.fromhex(hexstr))


# fp32 constants of the normal map, as exact hexadecimal floats.
_SQRT2 = _f32("0x1.6a09e6p+0")
_LN2_HI = _f32("0x1.62e4p-1")       # ln 2 with the low 9 mantissa bits cleared: k*LN2_HI is exact
_LN2_LO = _f32("0x1.7f7d1cp-20")    # ln 2 - LN2_HI
_PIO2 = _f32("0x1.921fb6p+0")
# atanh series 1/(2i+1), i = 0..5
_L = [_f32(h) for h in ("0x1p+0", "0x1.555556p-2", "0x1.99999ap-3", "0x1.24924ap-3",
                        "0x1.c71c72p-4", "0x1.745d18p-4")]
# sine Taylor coefficients (-1)^i/(2i+1)!, i = 1..6
_S = [_f32(h) for h in ("-0x1.555556p-3", "0x1.111112p-7", "-0x1.a01a02p-13",
                        "0x1.71de3ap-19", "-0x1.ae6456p-26", "0x1.612462p-33")]
# cosine Taylor coefficients (-1)^i/(2i)!, i = 1..7
_C = [_f32(h) for h in ("-0x1p-1", "0x1.555556p-5", "-0x1.6c16c2p-10", "0x1.a01a02p-16",
                        "-0x1.27e4fcp-22", "0x1.1eed8ep-29", "-0x1.93974ap-37")]


def normal_pair(wa, wb):
    """Box-Muller: two uint32 words -> two fp32 standard normals (z0 = r cos(theta), z1 = r sin(theta)).

    u1 = (2*(wa >> 9) + 1) / 2^24 in (0,1);  r = sqrt(-2 ln u1)
    theta = 2 pi u2 with u2 built from wb: top two bits = quadrant, next 23 bits = position f in
    the quadrant, f = (2*((wb >> 7) & 0x7FFFFF) + 1) / 2^24.

    ln u1: write the odd integer j = 2*(wa>>9)+1 as m * 2^e with m in [1,2) from its fp32 bit
    pattern, fold m into [sqrt(1/2), sqrt(2)), then ln m = 2 atanh((m-1)/(m+1)) by a 6-term series
    and ln u1 = (e - 24) ln 2 + ln m with ln 2 split in two words.
    sin / cos of x = (pi/2) f by Taylor polynomials (degree 13 / 14), rotated by the quadrant.
    Every fp32 operation below is a single correctly rounded +, *, / or sqrt, evaluated in the
    order written (no fused multiply-add).
    """
    wa = np.asarray(wa, dtype=np.uint32)
    wb = np.asarray(wb, dtype=np.uint32)
    one = np.float32(1.0)

    # ---- radius
    j = ((wa >> np.uint32(9)) << np.uint32(1)) | np.uint32(1)          # odd, 1 .. 2^24-1
    fj = j.astype(np.float32)                                           # exact
    bits = fj.view(np.uint32)
    e = (bits >> np.uint32(23)).astype(np.int32) - 127                  # 0 .. 23
    m = ((bits & np.uint32(0x7FFFFF)) | np.uint32(0x3F800000)).view(np.float32)
    big = m > _SQRT2
    m = np.where(big, m * np.float32(0.5), m)
    e = np.where(big, e + 1, e)
    t = (m - one) / (m + one)
    t2 = t * t
    p = _L[5]
    for i in (4, 3, 2, 1, 0):
        p = p * t2 + _L[i]
    q = t * p
    lnm = q + q
    k = (e - 24).astype(np.float32)
    lnu = k * _LN2_HI + (k * _LN2_LO + lnm)
    r = np.sqrt(lnu * np.float32(-2.0))

    # ---- angle
    quad = wb >> np.uint32(30)
    jf = (((wb >> np.uint32(7)) & np.uint32(0x7FFFFF)) << np.uint32(1)) | np.uint32(1)
    f = jf.astype(np.float32) * np.float32(2.0 ** -24)                  # exact
    x = f * _PIO2
    x2 = x * x
    ps = _S[5]
    for i in (4, 3, 2, 1, 0):
        ps = ps * x2 + _S[i]
    s = x * (ps * x2 + one)
    pc = _C[6]
    for i in (5, 4, 3, 2, 1, 0):
        pc = pc * x2 + _C[i]
    c = pc * x2 + one
    cos_t = np.where(quad == 0, c, np.where(quad == 1, -s, np.where(quad == 2, -c, s)))
    sin_t = np.where(quad == 0, s, np.where(quad == 1, c, np.where(quad == 2, -s, -c)))
    return (r * cos_t).astype(np.float32), (r * sin_t).astype(np.float32)


def words_field(seed: int, stream: int, step: int, n_env: int, n_blocks: int, env_offset: int = 0):
    """Philox words for envs [env_offset, env_offset+n_env) and blocks [0, n_blocks):
    four uint32 arrays of shape [n_env, n_blocks]."""
    k0, k1 = seed_key(seed)
    env = (np.arange(n_env, dtype=np.uint64) + np.uint64(env_offset))[:, None]
    blk = np.arange(n_blocks, dtype=np.uint64)[None, :]
    return philox4x32_10(env, np.uint64(step & 0xFFFFFFFF), np.uint64(stream), blk, k0, k1)


def normal_field(seed: int, stream: int, step: int, n_env: int, dim: int, env_offset: int = 0):
    """fp32 standard normals of shape [n_env, dim] for one (seed, stream, step)."""
    n_blocks = (dim + 3) // 4
    w0, w1, w2, w3 = words_field(seed, stream, step, n_env, n_blocks, env_offset)
    z0, z1 = normal_pair(w0, w1)
    z2, z3 = normal_pair(w2, w3)
    z = np.stack([z0, z1, z2, z3], axis=-1).reshape(n_env, n_blocks * 4)
    return np.ascontiguousarray(z[:, :dim])


def done_words(seed: int, step: int, n_env: int, env_offset: int = 0):
    """Word 0 of block 0 of the done stream, one per env."""
    w0, _, _, _ = words_field(seed, STREAM_DONE, step, n_env, 1, env_offset)
    return w0[:, 0]


def feistel_permutation(n: int, seed: int, iteration: int, epoch: int, rounds: int = 6):
    """A seeded bijection on [0, n), computable per element (used as the minibatch shuffle).

    Alternating unbalanced Feistel network on b = ceil(log2 n) bits with cycle walking.
    State x of b bits is split as (L : wl bits | R : wr bits), wl = b // 2, wr = b - wl.
    One round:  x <- (R << wl) | (L ^ (F(R) & (2^wl - 1))), then (wl, wr) swap.
    F(R) = word 0 of Philox(counter = (R, iteration, 4, epoch * 256 + round), key = seed).
    If the result is >= n the network is applied again (cycle walking) until it falls in [0, n).
    Returns perm[i] for i in [0, n) as int64.
    """
    if n <= 1:
        return np.zeros(n, dtype=np.int64)
    b = int(n - 1).bit_length()
    k0, k1 = seed_key(seed)
    x = np.arange(n, dtype=np.uint64)
    out = np.empty(n, dtype=np.uint64)
    todo = np.arange(n)
    while todo.size:
        y = x[todo]
        wl, wr = b // 2, b - b // 2
        for r in range(rounds):
            left = y >> np.uint64(wr)
            right = y & np.uint64((1 << wr) - 1)
            f, _, _, _ = philox4x32_10(right, np.uint64(iteration & 0xFFFFFFFF),
                                       np.uint64(STREAM_SHUFFLE),
                                       np.uint64(((epoch << 8) + r) & 0xFFFFFFFF), k0, k1)
            y = (right << np.uint64(wl)) | (left ^ (f.astype(np.uint64) & np.uint64((1 << wl) - 1)))
            wl, wr = wr, wl
        good = y < np.uint64(n)
        out[todo[good]] = y[good]
        x[todo] = y
        todo = todo[~good]
    return out.astype(np.int64)
