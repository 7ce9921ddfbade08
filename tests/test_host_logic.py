"""Host-side logic that needs no GPU: the one-GPU contract of bench.py and the CU-mask builder."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.parametrize("style", ["contiguous", "interleaved"])
@pytest.mark.parametrize("counts", [[64, 64, 64, 64], [48, 48, 48, 48, 64], [128, 128], [8, 8, 8, 8, 224], [256]])
def test_cu_masks_partition_the_device(style, counts):
    from paper_2206_08482_amd.instances import cu_masks
    masks = cu_masks(256, counts, style)
    ints = [sum(w << (32 * i) for i, w in enumerate(m)) for m in masks]
    assert [bin(x).count("1") for x in ints] == counts
    for i in range(len(ints)):
        for j in range(i):
            assert ints[i] & ints[j] == 0                      # disjoint
    assert sum(ints) == (1 << sum(counts)) - 1 if style == "contiguous" else True
    for x in ints:      # every instance keeps compute units on each of the 8 dies (bit index mod 8 = die)
        per_die = [sum((x >> b) & 1 for b in range(d, 256, 8)) for d in range(8)]
        assert min(per_die) >= 1 and max(per_die) - min(per_die) == 0      # and the same number on every die


def test_cu_masks_reject_counts_that_are_not_whole_rows():
    from paper_2206_08482_amd.instances import cu_masks
    with pytest.raises(ValueError):
        cu_masks(256, [60, 60], "contiguous")                  # not a multiple of 8: some die would get fewer CUs
    with pytest.raises(ValueError):
        cu_masks(256, [128, 136], "contiguous")                # more than the device has
