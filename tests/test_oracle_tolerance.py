"""Pins for the oracle of the appendix's third post-balancing algorithm (tolerance comparator)."""
import heapq
import os

import numpy as np
import pytest

import oracle
import workloads as wl
from test_oracle_dispatch import check_layout

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg3_tolerance.txt")


def _cases():
    cases, cur = [], None
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if tok[0] == "case":
            cur = {"name": tok[1]}
        elif tok[0] == "end":
            cases.append(cur)
        elif tok[0] == "batches":
            cur["batches"] = [[int(x) for x in grp.split()] for grp in " ".join(tok[1:]).split("|")]
        elif tok[0] in ("D", "v"):
            cur[tok[0]] = int(tok[1])
        else:
            cur[tok[0]] = [int(x) for x in tok[1:]]
    return cases


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"])
def test_golden(case):
    L = np.array(case["lengths"], np.int32)
    D = case["D"]
    asg = oracle.balance_tolerance(L, D, case["v"], 3, 7)
    check_layout(L, D, asg)
    assert [[int(L[s]) for s in asg.seqs_of(i)] for i in range(D)] == case["batches"]
    for i in range(D):
        assert int(asg.loads[i]) == 3 * case["squares"][i] + 7 * case["sums"][i]


def heap_replay(L, D, key_of):
    """A real priority queue works whenever the comparison is a total order: key_of(sum, sq, i)."""
    order = sorted(range(len(L)), key=lambda s: (-int(L[s]), s))
    heap = [(key_of(0, 0, i), 0, 0, i) for i in range(D)]
    heapq.heapify(heap)
    inst = np.zeros(len(L), np.int32)
    for s in order:
        _, sm, sq, i = heapq.heappop(heap)
        inst[s] = i
        sm, sq = sm + int(L[s]), sq + int(L[s]) ** 2
        heapq.heappush(heap, (key_of(sm, sq, i), sm, sq, i))
    return inst


@pytest.mark.parametrize("seed", range(20))
def test_extremes_reduce_to_a_priority_queue(seed):
    n = 1 + int(wl.uniform01(seed, 5, 1)[0] * 300)
    D = 1 + int(wl.uniform01(seed, 6, 1)[0] * 20)
    L = wl.random_lengths(700 + seed, n, 0 if seed % 2 else 1, [4, 60, 5000][seed % 3], zero_frac=0.1 * (seed % 2))
    # v <= 1: order by (length sum, squares, index)
    for v in (0, 1):
        asg = oracle.balance_tolerance(L, D, v, 1, 1)
        assert np.array_equal(asg.inst, heap_replay(L, D, lambda sm, sq, i: (sm, sq, i)))
    # v above the total length: order by (squares, index)
    asg = oracle.balance_tolerance(L, D, int(L.sum()) + 1, 1, 1)
    assert np.array_equal(asg.inst, heap_replay(L, D, lambda sm, sq, i: (sq, i)))
    check_layout(L, D, asg)


def cmp_listing(a, b, v):
    """CMP of the listing on (sum, squares) pairs."""
    if abs(a[0] - b[0]) < v:
        return a[1] < b[1]
    return a[0] < b[0]


@pytest.mark.parametrize("seed", range(20))
def test_choice_against_the_comparator(seed):
    """Step by step: the batch chosen is inside the window, nobody inside the window precedes it
    under the listing's CMP, everybody outside is at least v heavier than the lightest, and it is
    the lowest index among equals."""
    n = 5 + int(wl.uniform01(seed, 7, 1)[0] * 120)
    D = 2 + int(wl.uniform01(seed, 8, 1)[0] * 9)
    L = wl.random_lengths(800 + seed, n, 1, 40)
    v = 2 + int(wl.uniform01(seed, 9, 1)[0] * 60)
    asg = oracle.balance_tolerance(L, D, v, 1, 1)
    state = [(0, 0)] * D
    for s in sorted(range(n), key=lambda s: (-int(L[s]), s)):
        i = int(asg.inst[s])
        m = min(x[0] for x in state)
        assert state[i][0] - m < v
        for j in range(D):
            if state[j][0] - m < v:
                assert not cmp_listing(state[j], state[i], v)
                assert not (state[j][1] == state[i][1] and j < i)
            else:
                assert state[j][0] >= m + v
        state[i] = (state[i][0] + int(L[s]), state[i][1] + int(L[s]) ** 2)
    sums = [x[0] for x in state]
    for i in range(D):
        assert int(asg.tok_off[i + 1] - asg.tok_off[i]) == sums[i]
        assert int(asg.loads[i]) == state[i][1] + sums[i]


def test_trade_off_and_special_cases():
    w = wl.WORKLOADS[4]
    L = wl.draw_lengths(w)
    D = w.D

    def spread(asg):
        sums = np.diff(asg.tok_off).astype(np.float64)
        sq = np.array([np.sum(L[asg.seqs_of(i)].astype(np.float64) ** 2) for i in range(D)])
        return sums.max() / sums.mean(), sq.max() / sq.mean()

    tight, wide = oracle.balance_tolerance(L, D, 1, 1, 1), oracle.balance_tolerance(L, D, int(L.sum()) + 1, 1, 1)
    mid = oracle.balance_tolerance(L, D, 2048, 1, 1)
    # the tolerance trades token balance against balance of the quadratic term
    assert spread(tight)[0] <= spread(mid)[0] <= spread(wide)[0]
    assert spread(wide)[1] <= spread(mid)[1] <= spread(tight)[1]
    # every length sum stays within about v of the lightest while batches still compete
    sums = np.diff(mid.tok_off)
    assert sums.max() - sums.min() < 2048 + int(L.max())
    # all equal -> round robin; D = 1; n = 0; errors
    asg = oracle.balance_tolerance(np.full(10, 5, np.int32), 4, 3, 1, 1)
    assert np.array_equal(asg.inst, np.arange(10) % 4)
    asg = oracle.balance_tolerance(wl.random_lengths(1, 9, 1, 9), 1, 5, 1, 1)
    assert (asg.inst == 0).all()
    asg = oracle.balance_tolerance(np.zeros(0, np.int32), 3, 5, 1, 1)
    assert np.array_equal(asg.seq_off, [0, 0, 0, 0])
    with pytest.raises(oracle.OracleError):
        oracle.balance_tolerance(np.array([1, -2], np.int32), 2, 1, 1, 1)
    with pytest.raises(oracle.OracleError):
        oracle.balance_tolerance(np.array([1], np.int32), 0, 1, 1, 1)
    with pytest.raises(oracle.OracleError):  # squares overflow 2^63
        oracle.balance_tolerance(np.full(4, 2**31 - 1, np.int32), 1, 1, 1, 0)
