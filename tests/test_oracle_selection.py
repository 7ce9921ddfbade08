"""Pins of the Algorithm 2 oracle (the paper prints no worked example for it): hand-computed small tables,
a brute-force search for the saturation-free case, the early stop counted in profile() calls, and the
degenerate cases.  Each planted-mistake comment names the mistake the case would catch."""
import math

from oracle import selection as osel


def table_profile(table, calls=None):
    def profile(k, n):
        if calls is not None:
            calls.append((k, n))
        return table.get((k, n), (False, 0.0, 0.0))
    return profile


def linear_estimate(k, g, top):
    return top * k * g


def test_first_runnable_point_only_initialises_and_is_never_recorded():
    # one instance size, two points: the first initialises the trackers, the second is the only candidate
    t = {(1, 128): (True, 100.0, 10.0), (1, 256): (True, 150.0, 20.0)}
    assert osel.explore(table_profile(t), linear_estimate, 1, 0.1, [1], [128, 256]) == (256, 1)
    # a single runnable point can never be chosen (it only initialises) -> None
    assert osel.explore(table_profile({(1, 128): (True, 100.0, 10.0)}), linear_estimate, 1, 0.1, [1], [128]) is None
    assert osel.explore(table_profile({}), linear_estimate, 1, 0.1) is None


def test_hand_computed_saturation_stop():
    # throughput 100 -> 190 -> 200 -> 400, memory doubles each time (R_mem = 1):
    #   256: R_top 0.9 (>= 0.1, recorded); 512: R_top 0.0526 < 0.1 -> break; 1024 is never profiled
    t = {(2, 128): (True, 100.0, 1.0), (2, 256): (True, 190.0, 2.0), (2, 512): (True, 200.0, 4.0),
         (2, 1024): (True, 400.0, 8.0)}
    calls = []
    got = osel.explore(table_profile(t, calls), linear_estimate, 1, 0.1, [2], [128, 256, 512, 1024])
    assert got == (256, 2)                                   # the saturated point itself is not recorded
    assert calls == [(2, 128), (2, 256), (2, 512)]           # early stop (a missing break profiles 1024 and picks it)


def test_trackers_advance_to_every_runnable_point():
    # throughput 100 -> 200 -> 226 -> 248.6, memory doubling (R_mem = 1), alpha = 0.12.  Against the LAST
    # profiled point 1024 gains 0.1 < 0.12 and stops the search; with trackers left at an earlier point
    # (updated only when a point is recorded, or never) it would read 0.243 or 1.486, go on, and pick 1024.
    t = {(1, 128): (True, 100.0, 1.0), (1, 256): (True, 200.0, 2.0), (1, 512): (True, 226.0, 4.0),
         (1, 1024): (True, 248.6, 8.0)}
    # 512: R_top = 0.13 >= 0.12 recorded; 1024: 248.6/226 - 1 = 0.1 < 0.12 -> stop
    assert osel.explore(table_profile(t), linear_estimate, 1, 0.12, [1], [128, 256, 512, 1024]) == (512, 1)


def test_non_runnable_points_are_skipped_without_touching_the_trackers():
    # 128 not runnable -> 256 initialises; 512 not runnable; 1024 compared with 256
    t = {(4, 256): (True, 50.0, 2.0), (4, 1024): (True, 100.0, 8.0)}
    calls = []
    got = osel.explore(table_profile(t, calls), linear_estimate, 2, 0.1, [4], [128, 256, 512, 1024])
    assert got == (1024, 4)                                  # R_top = 1, R_mem = 3, Sat = 1/3
    assert len(calls) == 4
    # with alpha above 1/3 the same point counts as saturated
    assert osel.explore(table_profile(t), linear_estimate, 2, 0.34, [4], [128, 256, 512, 1024]) is None


def test_argmax_is_over_the_projected_system_throughput_and_ties_keep_the_first():
    # per-instance throughput falls with more instances per GPU, the projection multiplies it back
    t = {}
    for k, per in ((4, 30.0), (2, 55.0), (1, 100.0)):
        for i, n in enumerate([128, 256, 512]):
            t[(k, n)] = (True, per * (i + 1), float(n))
    # projections at 512: k=4 -> 360, k=2 -> 330, k=1 -> 300
    assert osel.explore(table_profile(t), linear_estimate, 1, 0.05, [4, 2, 1], [128, 256, 512]) == (512, 4)
    # order of the outer loop decides ties: equal projections keep the earlier (larger GMIperGPU) one
    t2 = {(2, 128): (True, 10.0, 1.0), (2, 256): (True, 50.0, 2.0), (1, 128): (True, 10.0, 1.0), (1, 256): (True, 100.0, 2.0)}
    assert osel.explore(table_profile(t2), linear_estimate, 1, 0.05, [2, 1], [128, 256]) == (256, 2)
    # a custom estimate is honoured (here: only one instance per GPU counts)
    assert osel.explore(table_profile(t), lambda k, g, top: top if k == 1 else 0.0, 1, 0.05, [4, 2, 1],
                        [128, 256, 512]) == (512, 1)


def test_equals_brute_force_when_nothing_saturates():
    # throughput and memory both proportional to num_env -> Sat = 1 everywhere -> plain arg-max over all
    # points but the first of each instance size
    grid = osel.NUM_ENV_GRID
    t = {(k, n): (True, n * (1.0 + 0.3 / k), float(n)) for k in osel.GMI_PER_GPU_RANGE for n in grid}
    best, best_v = None, -math.inf
    for k in osel.GMI_PER_GPU_RANGE:
        for n in grid[1:]:
            v = linear_estimate(k, 3, t[(k, n)][1])
            if v > best_v:
                best, best_v = (n, k), v
    assert osel.explore(table_profile(t), linear_estimate, 3, 0.09) == best == (16384, 10)


def test_division_readings():
    # unchanged memory with a throughput gain: Sat = +inf -> recorded; unchanged both: NaN -> not "< alpha"
    t = {(1, 128): (True, 10.0, 5.0), (1, 256): (True, 20.0, 5.0), (1, 512): (True, 20.0, 5.0)}
    assert osel.explore(table_profile(t), linear_estimate, 1, 0.1, [1], [128, 256, 512]) == (256, 1)
    # a throughput loss with growing memory: negative Sat -> stop
    t = {(1, 128): (True, 10.0, 5.0), (1, 256): (True, 9.0, 6.0), (1, 512): (True, 90.0, 7.0)}
    assert osel.explore(table_profile(t), linear_estimate, 1, 0.1, [1], [128, 256, 512]) is None
    # defaults follow the listing: instance counts 10 .. 1, environments 128 .. 16384 doubling
    assert osel.GMI_PER_GPU_RANGE == [10, 9, 8, 7, 6, 5, 4, 3, 2, 1]
    assert osel.NUM_ENV_GRID == [128 << i for i in range(8)]
