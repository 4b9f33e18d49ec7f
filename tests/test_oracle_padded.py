"""Pins for the oracle of Algorithm 2 (Post-Balancing with paddings, Sec. 5.1): hand-worked
fixtures, a literal list-of-lists replay with a LINEAR search of the bound, the brute-force optimum
over all contiguous cuts and over all assignments, closed forms."""
import itertools
import os

import numpy as np
import pytest

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg2_padded.txt")


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
        elif tok[0] in ("D", "bound"):
            cur[tok[0]] = int(tok[1])
        else:
            cur[tok[0]] = [int(x) for x in tok[1:]]
    return cases


def batches_py(sorted_len, b):
    """Algorithm 2's batch-counting helper with Python lists, as the listing states it."""
    ret = [[]]
    for l in sorted_len:
        if (len(ret[-1]) + 1) * l > b:
            ret.append([])
        ret[-1].append(l)
    return ret


def padded_len(batch):
    return len(batch) * max(batch) if batch else 0


def check_padded_layout(L, D, asg):
    n = len(L)
    assert sorted(asg.order.tolist()) == list(range(n))
    key = [(int(L[s]), int(s)) for s in asg.order]
    assert key == sorted(key)  # ascending length, ties by index, instance-major
    assert asg.seq_off[0] == 0 and asg.seq_off[D] == n and asg.tok_off[0] == 0
    for i in range(D):
        seqs, cu = asg.seqs_of(i), asg.cu_of(i)
        mx = int(L[seqs].max()) if len(seqs) else 0
        assert np.array_equal(cu, np.arange(len(seqs) + 1) * mx)
        assert np.all(asg.inst[seqs] == i)
        assert asg.tok_off[i + 1] - asg.tok_off[i] == len(seqs) * mx
    return [padded_len([int(L[s]) for s in asg.seqs_of(i)]) for i in range(D)]


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"])
def test_golden(case):
    L = np.array(case["lengths"], np.int32)
    D = case["D"]
    asg, bound = oracle.balance_padded(L, D, 3, 5)
    assert bound == case["bound"]
    got = [[int(L[s]) for s in asg.seqs_of(i)] for i in range(D)]
    want = case["batches"] + [[] for _ in range(D - len(case["batches"]))]
    assert got == want
    assert check_padded_layout(L, D, asg)[: len(case["padded"])] == case["padded"]
    srt = oracle.sort_asc(L)
    for b in case["fails"]:
        assert oracle.least_batches(L, srt, b)[0] > D
    assert oracle.least_batches(L, srt, bound)[0] <= D
    # Eq. 2, padding branch: a*L^2/cnt + b*L with L = cnt*max
    for i in range(D):
        seqs = asg.seqs_of(i)
        if len(seqs):
            Li = len(seqs) * int(L[seqs].max())
            assert int(asg.loads[i]) * len(seqs) == 3 * Li * Li + 5 * Li * len(seqs)
        else:
            assert asg.loads[i] == 0


@pytest.mark.parametrize("seed", range(40))
def test_linear_search_replay(seed):
    """Smallest feasible bound by trying b = left, left+1, ... with the list-of-lists replay."""
    n = 1 + int(wl.uniform01(seed, 1, 1)[0] * 40)
    D = 1 + int(wl.uniform01(seed, 2, 1)[0] * 7)
    L = wl.random_lengths(500 + seed, n, 0, 30, zero_frac=0.15 if seed % 3 == 0 else 0.0)
    srt = sorted(L.tolist())
    b = srt[0]
    while len(batches_py(srt, b)) > D:
        b += 1
    asg, bound = oracle.balance_padded(L, D, 1, 1)
    assert bound == b
    got = [[int(L[s]) for s in asg.seqs_of(i)] for i in range(D)]
    want = batches_py(srt, b)
    assert got == want + [[] for _ in range(D - len(want))]
    check_padded_layout(L, D, asg)
    assert np.array_equal(oracle.sort_asc(L), np.lexsort((np.arange(n), L)))
    # batch counts never grow with the bound (what makes the binary search valid)
    cnts = [oracle.least_batches(L, oracle.sort_asc(L), x)[0] for x in range(srt[0], b + 40)]
    assert all(c0 >= c1 for c0, c1 in zip(cnts, cnts[1:]))


def best_contiguous(srt, D):
    n = len(srt)
    best = None
    for k in range(1, min(D, n) + 1):
        for cuts in itertools.combinations(range(1, n), k - 1):
            edges = (0,) + cuts + (n,)
            m = max((e1 - e0) * srt[e1 - 1] for e0, e1 in zip(edges, edges[1:]))
            best = m if best is None else min(best, m)
    return best


def best_any(L, D):
    best = None
    for assign in itertools.product(range(D), repeat=len(L)):
        cnt, mx = [0] * D, [0] * D
        for l, i in zip(L, assign):
            cnt[i] += 1
            mx[i] = max(mx[i], l)
        m = max(c * x for c, x in zip(cnt, mx))
        best = m if best is None else min(best, m)
    return best


@pytest.mark.parametrize("seed", range(30))
def test_result_is_the_minimax_optimum(seed):
    """The largest padded batch length the algorithm returns equals the optimum over every cut of
    the ascending list into at most D runs, and (tiny cases) over every assignment whatsoever."""
    n = 2 + int(wl.uniform01(seed, 3, 1)[0] * 7)
    D = 1 + int(wl.uniform01(seed, 4, 1)[0] * 3)
    L = wl.random_lengths(900 + seed, n, 1, 12)
    asg, bound = oracle.balance_padded(L, D, 1, 1)
    achieved = max(check_padded_layout(L, D, asg))
    assert achieved == best_contiguous(sorted(L.tolist()), D)
    assert achieved == max(bound, int(L.max()))
    if n <= 7:
        assert achieved == best_any(L.tolist(), D)


def test_closed_forms_and_errors():
    # all equal: ceil(n/D) sequences per batch
    for n, D, l in [(10, 4, 7), (64, 8, 3), (5, 5, 11), (3, 8, 2)]:
        asg, bound = oracle.balance_padded(np.full(n, l, np.int32), D, 0, 1)
        per = -(-n // D)
        assert bound == (per * l if n > D else l)
        assert max(check_padded_layout(np.full(n, l, np.int32), D, asg)) == bound
    # D = 1: one batch, n * max
    L = wl.random_lengths(7, 33, 1, 50)
    asg, bound = oracle.balance_padded(L, 1, 2, 3)
    assert bound == 33 * int(L.max()) and asg.tok_off[1] == bound
    assert int(asg.loads[0]) == 33 * (2 * int(L.max()) ** 2 + 3 * int(L.max()))
    # n = 0
    asg, bound = oracle.balance_padded(np.zeros(0, np.int32), 3, 1, 1)
    assert bound == 0 and np.array_equal(asg.seq_off, [0, 0, 0, 0]) and np.array_equal(asg.cu_seqlens, [0, 0, 0])
    # all zero lengths: one batch of n empty slots
    asg, bound = oracle.balance_padded(np.zeros(6, np.int32), 3, 1, 1)
    assert bound == 0 and np.array_equal(asg.seq_off, [0, 6, 6, 6]) and asg.tok_off[3] == 0
    with pytest.raises(oracle.OracleError):
        oracle.balance_padded(np.array([3, -1], np.int32), 2, 1, 1)
    with pytest.raises(oracle.OracleError):
        oracle.balance_padded(np.array([3], np.int32), 0, 1, 1)
    # a padded batch of more than 2^31 - 1 rows cannot be described by int32 cu_seqlens
    with pytest.raises(oracle.OracleError):
        oracle.balance_padded(np.full(3, 2**30, np.int32), 1, 0, 1)


def test_padding_waste_shrinks_on_the_audio_workload():
    """Sec. 5.1's side benefit: fewer redundant paddings than batching each instance's own block."""
    w = wl.WORKLOADS[3]
    L = wl.draw_lengths(w)
    asg, bound = oracle.balance_padded(L, w.D, w.a, w.b)
    after = check_padded_layout(L, w.D, asg)
    per = w.n // w.D
    before = [per * int(L[i * per: (i + 1) * per].max()) for i in range(w.D)]
    assert max(after) <= bound and max(after) < 0.5 * max(before)
    assert sum(after) < 0.6 * sum(before)


def test_composition_from_a_padded_encoder_batch():
    """Rows of a padded encoder batch (Sec. 7: audio is batched with paddings) composed into the
    unpadded LLM batch: the first sub_len rows of every padded slot are the example's."""
    w = wl.WORKLOADS[1]
    L = wl.draw_lengths(w)
    split = wl.draw_modality_split(w, L)
    sub_off = wl.draw_interleave_offsets(split, 3)
    sub = np.ascontiguousarray(split[:, 2])
    H = 12
    easg, _ = oracle.balance_padded(sub, 3, 1, 1)
    masg = oracle.balance(L, w.D, w.a, w.b)
    rows = np.full((int(easg.tok_off[3]), H), 0xDEAD, dtype=np.uint16)
    cu0 = np.concatenate([[0], np.cumsum(sub, dtype=np.int64)])
    for i in range(3):
        cu = easg.cu_of(i)
        for j, s in enumerate(easg.seqs_of(i)):
            r0 = int(easg.tok_off[i]) + int(cu[j])
            rows[r0: r0 + sub[s]] = wl.token_tag_np(np.arange(cu0[s], cu0[s + 1]), H)
    T = int(L.sum())
    got = np.zeros((T, H), dtype=np.uint16)
    oracle.pack_composed(rows, got, sub, sub_off[:, 2], easg, masg)
    want = np.zeros((T, H), dtype=np.uint16)
    oracle.pack_composed(wl.token_tag_np(np.arange(cu0[-1]), H), want, sub, sub_off[:, 2], None, masg)
    assert np.array_equal(got, want) and not (got == 0xDEAD).any()
