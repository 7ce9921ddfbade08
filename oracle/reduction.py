"""Oracle for the layout-aware gradient reduction choice (Section 4.1: Algorithm 1, the leader rule of the
hierarchical reduction, and the time models of Table 2).

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing in the product).  Plain Python in the paper's
notation.  MPL is the GMI-to-GPU mapping list: MPL[p] = ids of the trainer instances on GPU p.

Readings where the paper is silent:
  * an empty MPL counts as "all instances on one GPU" (the listing's first test, len(MPL) <= 1);
  * the leader of a GPU for a given t is the instance whose id satisfies id % M == t, M = instances per GPU;
    a GPU whose ids contain no such residue has no leader (None) -- with consecutive ids per GPU, as in the
    paper's example, every GPU has exactly one;
  * the time models are evaluated as printed (t instances per GPU, g GPUs, M_p parameter bytes, B1 / B2
    bandwidths); they are real-valued formulas, no rounding.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

MPR = "Multi-Process Reduction"
MRR = "Multi-Ring Reduction"
HAR = "Hierarchical Reduction"


def select_strategy(mpl: Sequence[Sequence[int]]) -> str:
    """Algorithm 1 (Communication Strategy Selection)."""
    gmi_per_gpu_set = set()
    if len(mpl) <= 1:                       # all instances on the same GPU
        return MPR
    for gmi_li in mpl:                      # traverse all instances on all GPUs
        gmi_per_gpu_set.add(len(gmi_li))
    if len(gmi_per_gpu_set) > 1:            # GPUs host different numbers of instances
        return HAR
    if gmi_per_gpu_set.pop() > len(mpl):    # more instances per GPU than GPUs
        return HAR
    return MRR


def har_leaders(mpl: Sequence[Sequence[int]], t: int) -> List[Optional[int]]:
    """Leader instance of every GPU for step 2 of the hierarchical reduction: id % M == t."""
    out = []
    for gmi_li in mpl:
        m = len(gmi_li)
        lead = [i for i in gmi_li if m > 0 and i % m == t]
        out.append(lead[0] if lead else None)
    return out


def time_mpr(g: int, t: int, m_p: float, b1: float) -> float:
    return 2.0 * (g * t - 1) * m_p / (g * t * b1)


def time_mrr(g: int, t: int, m_p: float, b2: float) -> float:
    return 2.0 * (g - 1) * (t + 1) * m_p / (g * b2)


def time_har(g: int, t: int, m_p: float, b1: float, b2: float) -> float:
    return 2.0 * (g - 1) * m_p / (g * b2) + 2.0 * (t - 1) * m_p / (t * b1)
