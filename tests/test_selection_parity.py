"""gmi_explore (the library's Algorithm 2) against the oracle on synthetic profile tables: the chosen pair
and the exact sequence of profile() calls must be identical (integer / control-flow work: bit-exact).
No GPU work happens inside gmi_explore, so these run wherever the library loads."""
import math

import numpy as np
import pytest

import paper_2206_08482_amd as g
from oracle import selection as osel


def make_table(rng, ks, ns, p_unrunnable, saturating):
    t = {}
    for k in ks:
        cap = rng.uniform(2e3, 5e4) / k ** rng.uniform(0.3, 1.0)
        for n in ns:
            if rng.random() < p_unrunnable:
                continue
            top = cap * (1.0 - math.exp(-n / rng.uniform(300, 6000))) if saturating else cap * n * rng.uniform(0.9, 1.1)
            mem = 50.0 + n * rng.uniform(0.5, 2.0) if rng.random() > 0.1 else 50.0      # sometimes a flat footprint
            t[(k, n)] = (True, float(top), float(mem))
    return t


def run_both(t, num_gpu, alpha, ks, ns, estimate=None):
    calls_o, calls_p = [], []

    def prof(calls):
        def f(k, n):
            calls.append((k, n))
            return t.get((k, n), (False, 0.0, 0.0))
        return f
    est_o = estimate if estimate is not None else (lambda k, gpus, top: top * k * gpus)
    ref = osel.explore(prof(calls_o), est_o, num_gpu, alpha, ks, ns)
    got = g.gmi_explore(prof(calls_p), num_gpu, alpha, ks, ns, estimate)
    return ref, got, calls_o, calls_p


@pytest.mark.parametrize("seed", range(40))
def test_random_tables(seed):
    rng = np.random.default_rng(seed)
    ks = osel.GMI_PER_GPU_RANGE if seed % 2 == 0 else [8, 4, 2, 1]
    ns = osel.NUM_ENV_GRID
    t = make_table(rng, ks, ns, p_unrunnable=[0.0, 0.2, 0.6][seed % 3], saturating=seed % 4 != 3)
    alpha = [0.05, 0.1, 0.3, 0.0][seed % 4]
    estimate = None if seed % 5 else (lambda k, gpus, top: top * gpus * k ** 0.8)
    ref, got, co, cp = run_both(t, 1 + seed % 3, alpha, ks, ns, estimate)
    assert co == cp                                   # same points profiled, in the same order
    if ref is None:
        assert got is None
    else:
        assert got[:2] == ref
        est = estimate if estimate is not None else (lambda k, gpus, top: top * k * gpus)
        assert got[2] == est(ref[1], 1 + seed % 3, t[(ref[1], ref[0])][1])


def test_edge_cases():
    ks, ns = [2, 1], [128, 256, 512]
    # nothing runnable, a single runnable point, flat memory, throughput loss
    for t in ({}, {(1, 256): (True, 5.0, 1.0)},
              {(1, 128): (True, 10.0, 5.0), (1, 256): (True, 20.0, 5.0), (1, 512): (True, 20.0, 5.0)},
              {(2, 128): (True, 10.0, 5.0), (2, 256): (True, 9.0, 6.0), (2, 512): (True, 90.0, 7.0)}):
        ref, got, co, cp = run_both(t, 1, 0.1, ks, ns)
        assert co == cp
        assert (got is None and ref is None) or got[:2] == ref
    # empty value lists
    assert g.gmi_explore(lambda k, n: (True, 1.0, 1.0), 1, 0.1, [], ns) is None
    assert g.gmi_explore(lambda k, n: (True, 1.0, 1.0), 1, 0.1, ks, []) is None


def test_errors():
    with pytest.raises(g.GmiError):
        g.gmi_explore(lambda k, n: (True, 1.0, 1.0), 0, 0.1, [1], [128])            # num_gpu < 1
    with pytest.raises(ZeroDivisionError):                                           # callback failure surfaces
        g.gmi_explore(lambda k, n: (True, 1.0 / 0, 1.0), 1, 0.1, [1], [128])
