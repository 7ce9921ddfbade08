"""The library's reduction-strategy functions (Algorithm 1, leader rule, Table 2 time models) against the oracle:
integer / control-flow work, bit-exact; the time models to the last rounding.  Host-only: runs wherever the
library loads."""
import itertools

import numpy as np
import pytest

import paper_2206_08482_amd as g
from oracle import reduction as red

NAME = {g.REDUCE_MULTI_PROCESS: red.MPR, g.REDUCE_MULTI_RING: red.MRR, g.REDUCE_HIERARCHICAL: red.HAR}


def test_selection_on_every_small_layout():
    for n_gpus in range(0, 5):
        for counts in itertools.product(range(1, 6), repeat=n_gpus):
            ids = iter(range(1000))
            mpl = [[next(ids) for _ in range(c)] for c in counts]
            assert NAME[g.gmi_select_reduction(mpl)] == red.select_strategy(mpl), counts


def test_leaders_on_random_layouts():
    rng = np.random.default_rng(0)
    for _ in range(200):
        n_gpus = int(rng.integers(1, 6))
        mpl, nxt = [], 0
        for _p in range(n_gpus):
            c = int(rng.integers(1, 7))
            if rng.random() < 0.7:
                ids = list(range(nxt, nxt + c))
            else:
                ids = sorted(int(x) for x in rng.choice(50, size=c, replace=False))
            nxt += c
            mpl.append(ids)
        t = int(rng.integers(0, 6))
        assert g.gmi_har_leaders(mpl, t) == red.har_leaders(mpl, t), (mpl, t)


def test_time_models():
    rng = np.random.default_rng(1)
    for _ in range(100):
        gg, t = int(rng.integers(1, 9)), int(rng.integers(1, 11))
        m_p, b1, b2 = float(rng.uniform(1e5, 1e8)), float(rng.uniform(1e9, 2e10)), float(rng.uniform(1e10, 4e11))
        assert g.gmi_reduction_time(g.REDUCE_MULTI_PROCESS, gg, t, m_p, b1, b2) == pytest.approx(red.time_mpr(gg, t, m_p, b1), rel=1e-15)
        assert g.gmi_reduction_time(g.REDUCE_MULTI_RING, gg, t, m_p, b1, b2) == pytest.approx(red.time_mrr(gg, t, m_p, b2), rel=1e-15)
        assert g.gmi_reduction_time(g.REDUCE_HIERARCHICAL, gg, t, m_p, b1, b2) == pytest.approx(red.time_har(gg, t, m_p, b1, b2), rel=1e-15)


def test_error_paths():
    with pytest.raises(g.GmiError):
        g.gmi_reduction_time(7, 1, 1, 1.0, 1.0, 1.0)
    with pytest.raises(g.GmiError):
        g.gmi_reduction_time(g.REDUCE_MULTI_RING, 0, 1, 1.0, 1.0, 1.0)


def test_least_loaded_routing_matches_oracle():
    from oracle import channels as och
    rng = np.random.default_rng(2)
    for _ in range(200):
        n = int(rng.integers(1, 9))
        load = [int(x) for x in rng.integers(0, 5, size=n) * 1000]
        assert g.gmi_route_least_loaded(load) == och.route_least_loaded(load)
