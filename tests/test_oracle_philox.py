"""Pins for oracle.philox: the generator against its published known-answer vectors, the normal map
against a float64 Box-Muller and distribution tests, the shuffle against brute-force bijectivity."""
import math
import os

import numpy as np
import pytest
from scipy import stats as sps

from oracle import philox as px

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        v = [int(x, 16) for x in row]
        out = px.philox4x32_10(*[np.uint64(c) for c in v[0:4]], v[4], v[5])
        assert [int(o) for o in out] == v[6:10]


def test_philox_is_bijective_on_a_counter_slice():
    # for a fixed key each round is a bijection of the 128-bit counter: 2^16 distinct counters
    # must give 2^16 distinct outputs, and changing any counter word changes the output.
    c = np.arange(1 << 16, dtype=np.uint64)
    for pos in range(4):
        args = [np.uint64(7)] * 4
        args[pos] = c
        w = px.philox4x32_10(*args, 11, 13)
        packed = np.stack(w, axis=-1)
        assert len(np.unique(packed, axis=0)) == c.size


def test_philox_word_uniformity():
    w = px.philox4x32_10(np.arange(1 << 18, dtype=np.uint64), 3, 1, 0, 5, 0)
    for x in w:
        u = x.astype(np.float64) / 2.0 ** 32
        assert abs(u.mean() - 0.5) < 4 * (1 / math.sqrt(12 * u.size))
        # each of the 32 bits is set about half of the time
        for b in (0, 7, 16, 31):
            frac = ((x >> np.uint32(b)) & 1).mean()
            assert abs(frac - 0.5) < 4 * 0.5 / math.sqrt(u.size)


def _box_muller_f64(wa, wb):
    u1 = (2.0 * (wa >> np.uint32(9)).astype(np.float64) + 1.0) / 2.0 ** 24
    quad = (wb >> np.uint32(30)).astype(np.float64)
    f = (2.0 * ((wb >> np.uint32(7)) & np.uint32(0x7FFFFF)).astype(np.float64) + 1.0) / 2.0 ** 24
    theta = (quad + f) * (math.pi / 2)
    r = np.sqrt(-2.0 * np.log(u1))
    return r * np.cos(theta), r * np.sin(theta)


def test_normal_pair_matches_float64_box_muller():
    rng = np.random.default_rng(1)
    wa = rng.integers(0, 1 << 32, 2_000_000, dtype=np.uint64).astype(np.uint32)
    wb = rng.integers(0, 1 << 32, 2_000_000, dtype=np.uint64).astype(np.uint32)
    z0, z1 = px.normal_pair(wa, wb)
    assert z0.dtype == np.float32 and z1.dtype == np.float32
    r0, r1 = _box_muller_f64(wa, wb)
    err = np.maximum(np.abs(z0 - r0), np.abs(z1 - r1))
    scale = 1.0 + np.maximum(np.abs(r0), np.abs(r1))
    assert (err / scale).max() < 5e-7
    assert err.max() < 2e-6


def test_normal_pair_edge_words():
    edge = np.array([0, 1, 0x1FF, 0x200, 0x7FFFFFFF, 0x80000000, 0xFFFFFE00, 0xFFFFFFFF,
                     0x3FFFFFFF, 0x40000000, 0xBFFFFFFF, 0xC0000000], dtype=np.uint32)
    wa, wb = np.meshgrid(edge, edge)
    z0, z1 = px.normal_pair(wa.ravel(), wb.ravel())
    assert np.isfinite(z0).all() and np.isfinite(z1).all()
    r0, r1 = _box_muller_f64(wa.ravel(), wb.ravel())
    assert np.abs(z0 - r0).max() < 2e-6 and np.abs(z1 - r1).max() < 2e-6
    # largest radius: u1 = 2^-24  ->  r = sqrt(48 ln 2)
    zmax, _ = px.normal_pair(np.uint32(0), np.uint32(0))
    assert abs(math.hypot(*[float(v) for v in px.normal_pair(np.uint32(0), np.uint32(0))])
               - math.sqrt(48 * math.log(2))) < 2e-6
    assert zmax > 5.7


def test_radius_exhaustive_over_all_inputs():
    # the radius depends on 23 bits only: check every one of them against float64
    k = np.arange(1 << 23, dtype=np.uint32)
    z0, z1 = px.normal_pair(k << np.uint32(9), np.zeros_like(k))       # theta ~ 0: z0 ~ r
    r = np.hypot(z0.astype(np.float64), z1.astype(np.float64))
    ref = np.sqrt(-2.0 * np.log((2.0 * k + 1.0) / 2.0 ** 24))
    assert np.isfinite(r).all()
    assert (np.abs(r - ref) / (1 + ref)).max() < 4e-7


def test_normal_field_moments_and_ks():
    z = px.normal_field(seed=12345, stream=px.STREAM_ENV, step=3, n_env=250_000, dim=8)
    assert z.shape == (250_000, 8) and z.dtype == np.float32
    x = z.astype(np.float64).ravel()
    n = x.size
    assert abs(x.mean()) < 4 / math.sqrt(n)
    assert abs(x.var() - 1) < 4 * math.sqrt(2 / n)
    assert abs(sps.kurtosis(x)) < 4 * math.sqrt(24 / n)
    assert abs(sps.skew(x)) < 4 * math.sqrt(6 / n)
    assert sps.kstest(x[:500_000], "norm").pvalue > 1e-3
    # columns are uncorrelated, envs are uncorrelated
    c = np.corrcoef(z[:, :4].astype(np.float64), rowvar=False)
    assert np.abs(c - np.eye(4)).max() < 5 / math.sqrt(z.shape[0])


def test_normal_field_layout():
    # element j of env e: block j//4, pair (j%4)//2, component j%2; independent of how many
    # elements or envs are asked for
    full = px.normal_field(9, px.STREAM_ACTION, 17, 33, 11)
    part = px.normal_field(9, px.STREAM_ACTION, 17, 5, 6, env_offset=20)
    assert np.array_equal(full[20:25, :6], part)
    k0, k1 = px.seed_key(9)
    w = px.philox4x32_10(np.uint64(22), 17, px.STREAM_ACTION, 2, k0, k1)
    z2, z3 = px.normal_pair(w[2], w[3])
    assert full[22, 10] == z2 and np.isclose(full[22, 10], z2)
    z0, z1 = px.normal_pair(w[0], w[1])
    assert full[22, 8] == z0 and full[22, 9] == z1
    other = px.normal_field(9, px.STREAM_ENV, 17, 33, 11)
    assert not np.array_equal(full, other)
    assert not np.array_equal(full, px.normal_field(9, px.STREAM_ACTION, 18, 33, 11))
    assert not np.array_equal(full, px.normal_field(10, px.STREAM_ACTION, 17, 33, 11))
    assert not np.array_equal(full, px.normal_field(9 + (1 << 32), px.STREAM_ACTION, 17, 33, 11))


@pytest.mark.parametrize("n", [0, 1, 2, 3, 7, 64, 1000, 1024, 1 << 13, 12345])
def test_feistel_permutation_is_a_bijection(n):
    p = px.feistel_permutation(n, seed=3, iteration=2, epoch=1)
    assert p.shape == (n,)
    assert np.array_equal(np.sort(p), np.arange(n))


def test_feistel_permutation_depends_on_seed_iteration_epoch():
    base = px.feistel_permutation(4096, 3, 2, 1)
    assert np.array_equal(base, px.feistel_permutation(4096, 3, 2, 1))
    for args in ((4, 2, 1), (3, 3, 1), (3, 2, 0)):
        other = px.feistel_permutation(4096, *args)
        assert (other == base).mean() < 0.01
    # looks shuffled: few fixed points, displacement about n/3 on average
    assert (base == np.arange(4096)).sum() < 10
    assert abs(np.abs(base - np.arange(4096)).mean() / 4096 - 1 / 3) < 0.03
    # minibatches built from it partition the batch
    mbs = base.reshape(4, 1024)
    assert len(np.unique(mbs)) == 4096


def test_done_threshold_rate():
    from oracle.ppo import done_threshold_from_inverse
    thr = done_threshold_from_inverse(1000)
    assert thr == (1 << 32) // 1000
    n = 4_000_000
    w = px.done_words(7, 5, n)
    rate = (w < np.uint32(thr)).mean()
    assert abs(rate - 1e-3) < 3 * math.sqrt(1e-3 / n)
