"""Oracle for the machine-grouping heuristic of selective logging (paper, section "Selective
Logging").  TEST INFRASTRUCTURE ONLY, like the rest of this package: plain Python floats (IEEE
binary64), the algorithm's steps in the paper's order and notation, no shortcuts.

Setting: N machines host consecutive pipeline stages.  Logging records the messages between
groups of machines but not inside a group; a failure rolls the whole group of the failed machine
back.  R(G) is the per-iteration computation time of group G, M(G_i, G_{i+1}) the bytes sent per
iteration between adjacent groups, T the checkpoint interval in iterations, B the network
bandwidth, M_max the storage limit for logging data.

  M(grouping) = T * sum of M over adjacent groups
  merging G_i and G_{i+1}:  R(G_i, G_{i+1}) = R(G_i) + R(G_{i+1}) + M(G_i, G_{i+1}) / B
  dR = R(G_i, G_{i+1}) (|G_i| + |G_{i+1}|)/N - R(G_i) |G_i|/N - R(G_{i+1}) |G_{i+1}|/N
  dM = M(G_i, G_{i+1}) T
Start with every machine a group of its own; while M(grouping) > M_max merge the adjacent pair
with the smallest dR/dM.  With parallel recovery every R(G) that enters dR is divided by
floor(N/|G|).

Readings where the text is silent: ties go to the pair with the lowest index; a pair with
M(G_i, G_{i+1}) = 0 frees no storage and is never merged while a pair with dM > 0 exists (its
ratio is +infinity; if every remaining pair has dM = 0 the storage is 0 and the loop has ended
unless M_max < 0, in which case the lowest-index pair is merged); the expected recovery time of a
grouping is sum over groups of R(G) |G| / N, which is what the dR formula differences.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple


def group_machines(R: Sequence[float], M: Sequence[float], T: float, B: float, M_max: float,
                   parallel_recovery: bool = False) -> Tuple[List[List[int]], float, float, list]:
    """Returns (groups, storage, expected_recovery, log).  groups: lists of machine ranks in
    pipeline order; log: one (left_group_index, dR, dM) per merge, in order."""
    N = len(R)
    if N < 1 or len(M) != N - 1:
        raise ValueError("need N >= 1 compute times and N - 1 message sizes")
    groups = [[i] for i in range(N)]
    Rg = [float(r) for r in R]                 # R(G) of each current group (undivided)
    Mg = [float(m) for m in M]                 # M(G_i, G_{i+1}) for each adjacent pair of current groups

    def eff(r: float, size: int) -> float:
        return r / (N // size) if parallel_recovery else r

    def storage() -> float:
        s = 0.0
        for m in Mg:
            s += m
        return T * s

    log = []
    while len(groups) > 1 and storage() > M_max:
        best, best_ratio, best_d = None, None, None
        for i in range(len(groups) - 1):
            a, b = len(groups[i]), len(groups[i + 1])
            merged = Rg[i] + Rg[i + 1] + Mg[i] / B
            dR = eff(merged, a + b) * (a + b) / N - eff(Rg[i], a) * a / N - eff(Rg[i + 1], b) * b / N
            dM = Mg[i] * T
            ratio = dR / dM if dM > 0 else math.inf
            if best is None or ratio < best_ratio:
                best, best_ratio, best_d = i, ratio, (dR, dM)
        i = best
        log.append((i, best_d[0], best_d[1]))
        Rg[i] = Rg[i] + Rg[i + 1] + Mg[i] / B
        groups[i] = groups[i] + groups[i + 1]
        del groups[i + 1], Rg[i + 1], Mg[i]
    expected = 0.0
    for g, r in zip(groups, Rg):
        expected += eff(r, len(g)) * len(g) / N
    return groups, storage(), expected, log
