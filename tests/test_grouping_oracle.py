"""Pins for the oracle of the machine-grouping heuristic (section "Selective Logging"): a hand-worked
example, the closed forms the merge rule implies, brute force over every contiguous grouping of
tiny pipelines, and the cases that reduce to something obvious.  CPU only."""
import itertools
import math
import random

import pytest

from golden_io import read_grouping_example
from oracle.grouping import group_machines


def _group_of(groups):
    out = {}
    for k, g in enumerate(groups):
        for r in g:
            out[r] = k
    return [out[r] for r in sorted(out)]


def _closed_form(groups, R, M, T, B, parallel):
    """Storage and expected recovery of a grouping straight from the definitions, no merging:
    R(G) = sum of its machines' R + (bytes on its internal links)/B; storage = T * bytes on cut links."""
    N = len(R)
    cut = sum(M[g[-1]] for g in groups[:-1])
    exp = 0.0
    for g in groups:
        r = sum(R[i] for i in g) + sum(M[i] for i in g[:-1]) / B
        if parallel:
            r /= N // len(g)
        exp += r * len(g) / N
    return T * cut, exp


def test_hand_worked_example():
    R, M, T, B, cases = read_grouping_example()
    for limit, parallel, want_groups, want_storage, want_recovery in cases:
        groups, storage, recovery, _ = group_machines([float(r) for r in R], [float(m) for m in M], float(T), float(B),
                                                      float(limit), parallel)
        assert _group_of(groups) == want_groups, (limit, parallel)
        assert storage == float(want_storage) and recovery == pytest.approx(float(want_recovery), rel=1e-15)


@pytest.mark.parametrize("parallel", [False, True])
def test_result_matches_the_definitions_and_the_limit(parallel):
    rng = random.Random(5)
    for trial in range(300):
        N = rng.randint(1, 12)
        R = [rng.uniform(0.1, 5.0) for _ in range(N)]
        M = [rng.choice([0.0, rng.uniform(1.0, 100.0)]) if trial % 7 == 0 else rng.uniform(1.0, 100.0) for _ in range(N - 1)]
        T, B = rng.choice([1.0, 10.0, 100.0]), rng.uniform(1.0, 50.0)
        total = T * sum(M)
        limit = rng.uniform(-0.1, 1.1) * total
        groups, storage, recovery, log = group_machines(R, M, T, B, limit, parallel)
        assert [r for g in groups for r in g] == list(range(N))                    # contiguous, in pipeline order
        s, e = _closed_form(groups, R, M, T, B, parallel)
        assert storage == pytest.approx(s, rel=1e-12, abs=1e-12) and recovery == pytest.approx(e, rel=1e-12)
        assert storage <= limit or len(groups) == 1                                # the loop's exit condition
        assert len(log) == N - len(groups)
        # the path adds up: recovery = initial + sum dR, storage = initial - sum dM
        s0, e0 = _closed_form([[i] for i in range(N)], R, M, T, B, parallel)
        assert recovery == pytest.approx(e0 + sum(d[1] for d in log), rel=1e-11)
        assert storage == pytest.approx(s0 - sum(d[2] for d in log), rel=1e-11, abs=1e-9)
        if not parallel:
            assert all(d[1] > 0 for d in log)                                      # the paper: dR is always positive
        # undoing the last merge would have violated the limit (the loop merges only while it must)
        if log:
            assert storage + log[-1][2] > limit


def test_every_merge_takes_the_smallest_ratio_brute_force():
    """Tiny pipelines: replay the log and compare each step with the ratios of ALL adjacent pairs
    computed from the definitions (closed form of both groupings), not with the merge formulas."""
    rng = random.Random(11)
    for _ in range(200):
        N = rng.randint(2, 7)
        R = [rng.uniform(0.1, 5.0) for _ in range(N)]
        M = [rng.uniform(1.0, 100.0) for _ in range(N - 1)]
        T, B = 3.0, rng.uniform(1.0, 50.0)
        parallel = rng.random() < 0.5
        groups, _, _, log = group_machines(R, M, T, B, -1.0, parallel)             # merge all the way
        assert len(groups) == 1 and len(log) == N - 1
        cur = [[i] for i in range(N)]
        for (i, dR, dM) in log:
            s0, e0 = _closed_form(cur, R, M, T, B, parallel)
            ratios = []
            for k in range(len(cur) - 1):
                nxt = cur[:k] + [cur[k] + cur[k + 1]] + cur[k + 2:]
                s1, e1 = _closed_form(nxt, R, M, T, B, parallel)
                ratios.append((e1 - e0) / (s0 - s1))
            assert ratios[i] <= min(ratios) * (1 + 1e-9) + 1e-15
            assert dR / dM == pytest.approx(ratios[i], rel=1e-7)
            cur = cur[:i] + [cur[i] + cur[i + 1]] + cur[i + 2:]


def test_special_cases():
    R, M = [1.0, 2.0, 3.0, 4.0, 5.0], [8.0, 4.0, 2.0, 1.0]
    # enough storage: nothing merges (the paper's "each machine forms a group")
    g, s, e, log = group_machines(R, M, 10.0, 2.0, 150.0)
    assert g == [[0], [1], [2], [3], [4]] and s == 150.0 and e == pytest.approx(3.0) and log == []
    # no storage at all: one group, no logging
    g, s, e, _ = group_machines(R, M, 10.0, 2.0, 0.0)
    assert g == [[0, 1, 2, 3, 4]] and s == 0.0 and e == pytest.approx(15.0 + 15.0 / 2.0)
    # one machine
    assert group_machines([2.5], [], 10.0, 1.0, 0.0)[:3] == ([[0]], 0.0, 2.5)
    # a lower limit only coarsens the grouping: the merge sequence does not depend on the limit
    prev = None
    for limit in (150, 120, 90, 60, 30, 10, 0):
        g = group_machines(R, M, 10.0, 2.0, float(limit))[0]
        if prev is not None:
            assert all(any(set(a) <= set(b) for b in g) for a in prev)
        prev = g
    # identical machines and links, infinite bandwidth: dR of merging sizes a and b is 2ab r/N, dM the same
    # for every pair, so singles pair up from the left before anything larger forms
    g = group_machines([1.0] * 8, [5.0] * 7, 1.0, math.inf, 5.0 * 3)[0]
    assert g == [[0, 1], [2, 3], [4, 5], [6, 7]]
    # a tie goes to the pair with the lowest index (a reading: the paper does not say)
    assert group_machines([1.0] * 4, [5.0] * 3, 1.0, math.inf, 10.0)[0] == [[0, 1], [2], [3]]
    # a link that carries nothing is never merged while merging elsewhere still frees storage
    g = group_machines([1.0, 1.0, 1.0], [0.0, 9.0], 1.0, 1.0, 1.0)[0]
    assert g == [[0], [1, 2]]
    with pytest.raises(ValueError):
        group_machines([1.0, 2.0], [], 1.0, 1.0, 0.0)
