"""Pins of the oracle for Algorithm 1 (communication strategy selection), the leader rule and the time models
of the three reduction strategies (Section 4.1, Table 2)."""
import itertools

import pytest

from oracle import reduction as red


def test_paper_example_layout_selects_multi_ring():
    # the listing's own input: three GPUs with three instances each -> neither exit fires
    assert red.select_strategy([[0, 1, 2], [3, 4, 5], [6, 7, 8]]) == red.MRR


@pytest.mark.parametrize("mpl,want", [
    ([[0, 1, 2, 3]], red.MPR),                                  # all instances on one GPU
    ([], red.MPR),
    ([[0, 1], [2, 3, 4]], red.HAR),                             # different numbers per GPU
    ([[0, 1, 2], [3, 4, 5]], red.HAR),                          # 3 per GPU > 2 GPUs
    ([[0, 1], [2, 3]], red.MRR),                                # 2 per GPU == 2 GPUs
    ([[0], [1], [2], [3]], red.MRR),                            # one process per GPU
    ([[0, 1, 2, 3], [4, 5, 6, 7], [8, 9, 10, 11], [12, 13, 14, 15]], red.MRR),
])
def test_each_exit_of_the_selection(mpl, want):
    assert red.select_strategy(mpl) == want


def test_selection_equals_the_rule_stated_in_the_text_by_brute_force():
    """Section 4.1 in words: one GPU -> MPR; rings need equal counts per GPU and at most as many instances per
    GPU as GPUs; everything else -> HAR.  All layouts of up to 4 GPUs with 1..5 instances each."""
    for g in range(1, 5):
        for counts in itertools.product(range(1, 6), repeat=g):
            ids = iter(range(100))
            mpl = [[next(ids) for _ in range(c)] for c in counts]
            if g == 1:
                want = red.MPR
            elif len(set(counts)) == 1 and counts[0] <= g:
                want = red.MRR
            else:
                want = red.HAR
            assert red.select_strategy(mpl) == want, counts


def test_leaders_one_per_gpu_with_consecutive_ids():
    mpl = [[0, 1, 2], [3, 4, 5], [6, 7, 8]]
    assert red.har_leaders(mpl, 0) == [0, 3, 6]
    assert red.har_leaders(mpl, 1) == [1, 4, 7]
    assert red.har_leaders(mpl, 2) == [2, 5, 8]
    assert red.har_leaders([[0, 2], [1, 3, 5]], 1) == [None, 1]      # no id with that residue on GPU 0


def test_time_models_special_cases():
    m_p, b1, b2 = 1e6, 2e9, 5e10
    # one instance per GPU: the hierarchical form has no intra-GPU term and is the plain ring all-reduce
    assert red.time_har(8, 1, m_p, b1, b2) == pytest.approx(2 * 7 * m_p / (8 * b2))
    # one GPU: no inter-GPU term; equals the multi-process form on the same t instances
    assert red.time_har(1, 4, m_p, b1, b2) == pytest.approx(red.time_mpr(1, 4, m_p, b1))
    # the ring form with t rings plus the final ring: (t + 1) ring all-reduces
    assert red.time_mrr(4, 3, m_p, b2) == pytest.approx(4 * (2 * 3 * m_p / (4 * b2)))
    # a single instance in total needs no time under MPR
    assert red.time_mpr(1, 1, m_p, b1) == 0.0
    # hand-computed: g = 2, t = 3, M_p = 12, B1 = 2, B2 = 4
    assert red.time_mpr(2, 3, 12.0, 2.0) == pytest.approx(2 * 5 * 12 / (6 * 2))
    assert red.time_mrr(2, 3, 12.0, 4.0) == pytest.approx(2 * 1 * 4 * 12 / (2 * 4))
    assert red.time_har(2, 3, 12.0, 2.0, 4.0) == pytest.approx(2 * 1 * 12 / (2 * 4) + 2 * 2 * 12 / (3 * 2))
