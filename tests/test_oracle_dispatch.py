"""Pins for the dispatch oracle: every check here is something other than the
oracle's own code path (closed forms, a library sort, a heap-based replay of
Algorithm 1, brute-force optima, Graham's bound, hand-worked fixtures)."""
import heapq
import itertools
import os

import numpy as np
import pytest

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "lpt_textbook.txt")


def _golden_cases():
    cases, cur = [], None
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if tok[0] == "case":
            cur = {"name": tok[1], "cu": {}}
        elif tok[0] == "end":
            cases.append(cur)
        elif tok[0] == "cu":
            cur["cu"][int(tok[1].rstrip(":"))] = [int(x) for x in tok[2:]]
        elif tok[0] in ("D", "opt"):
            cur[tok[0]] = int(tok[1])
        else:
            cur[tok[0]] = [int(x) for x in tok[1:]]
    return cases


def heap_lpt(costs, D):
    """Algorithm 1 with a real priority queue keyed (load, instance index)."""
    order = sorted(range(len(costs)), key=lambda s: (-int(costs[s]), s))
    heap = [(0, i) for i in range(D)]
    heapq.heapify(heap)
    inst = [0] * len(costs)
    bins = [[] for _ in range(D)]
    for s in order:
        load, i = heapq.heappop(heap)
        inst[s] = i
        bins[i].append(s)
        heapq.heappush(heap, (load + int(costs[s]), i))
    loads = [sum(int(costs[s]) for s in b) for b in bins]
    return inst, bins, loads


def brute_opt(costs, D):
    best = None
    n = len(costs)
    for assign in itertools.product(range(D), repeat=n):
        loads = [0] * D
        for s, i in enumerate(assign):
            loads[i] += costs[s]
        m = max(loads)
        if best is None or m < best:
            best = m
    return best


def check_layout(L, D, asg):
    n = len(L)
    assert sorted(asg.order.tolist()) == list(range(n))
    assert asg.seq_off[0] == 0 and asg.seq_off[D] == n
    assert asg.tok_off[0] == 0 and asg.tok_off[D] == int(np.sum(L, dtype=np.int64))
    for i in range(D):
        seqs = asg.seqs_of(i)
        cu = asg.cu_of(i)
        assert cu[0] == 0
        assert np.array_equal(np.diff(cu), L[seqs])
        assert np.all(asg.inst[seqs] == i)
        assert asg.tok_off[i + 1] - asg.tok_off[i] == cu[-1]


@pytest.mark.parametrize("case", _golden_cases(), ids=lambda c: c["name"])
def test_golden_lpt(case):
    L = np.array(case["L"], dtype=np.int32)
    asg = oracle.balance(L, case["D"], 0, 1)
    assert asg.inst.tolist() == case["inst"]
    assert asg.loads.tolist() == case["loads"]
    for i, cu in case["cu"].items():
        assert asg.cu_of(i).tolist() == cu
    assert brute_opt(case["L"], case["D"]) == case["opt"]
    if case["name"].startswith("graham"):
        D = case["D"]
        # the tight family reaches the bound exactly: 3D*LPT == (4D-1)*OPT
        assert 3 * D * max(case["loads"]) == (4 * D - 1) * case["opt"]


def test_cost_closed_form_and_errors():
    L = np.array([0, 1, 7, 512, 8192, 32768], dtype=np.int32)
    for a, b in [(1, 512), (0, 1), (3, 0), (1, 98304)]:
        c = oracle.cost(L, a, b)
        assert c.tolist() == [a * int(l) * int(l) + b * int(l) for l in L]
    # Sec. 5.1: with beta << alpha the objective is the token count itself
    assert oracle.cost(L, 0, 1).tolist() == L.tolist()
    with pytest.raises(oracle.OracleError) as e:
        oracle.cost(np.array([3, -1], dtype=np.int32), 1, 1)
    assert e.value.code == -5
    with pytest.raises(oracle.OracleError) as e:
        oracle.cost(np.array([2 ** 31 - 1] * 4, dtype=np.int32), 2 ** 40, 0)
    assert e.value.code == -5


@pytest.mark.parametrize("seed", range(6))
def test_sort_against_library_sort(seed):
    n = [0, 1, 2, 97, 1000, 4099][seed]
    L = wl.random_lengths(seed, n, 0, 40, zero_frac=0.2)  # many ties
    c = oracle.cost(L, 1, 3)
    got = oracle.sort_desc(c)
    want = sorted(range(n), key=lambda s: (-int(c[s]), s))
    assert got.tolist() == want


@pytest.mark.parametrize("seed", range(12))
def test_greedy_matches_heap_replay(seed):
    n = [1, 5, 64, 333, 1024, 2000][seed % 6]
    D = [1, 2, 3, 8, 16, 37, 64, 256][seed % 8]
    L = wl.random_lengths(100 + seed, n, 0 if seed % 2 else 1, 50 if seed % 3 else 4000,
                          zero_frac=0.15 if seed % 2 else 0.0)
    a, b = [(1, 512), (0, 1), (1, 0), (2, 7)][seed % 4]
    asg = oracle.balance(L, D, a, b)
    c = oracle.cost(L, a, b)
    inst, bins, loads = heap_lpt(c, D)
    assert asg.inst.tolist() == inst
    assert asg.loads.tolist() == loads
    for i in range(D):
        assert asg.seqs_of(i).tolist() == bins[i]
    check_layout(L, D, asg)
    assert int(asg.loads.sum()) == int(c.sum())


def test_bruteforce_optimum_and_graham_bound():
    rng_seed = 0
    for n in range(1, 10):
        for D in (1, 2, 3):
            for rep in range(3 if n < 9 else 1):
                rng_seed += 1
                L = wl.random_lengths(rng_seed, n, 1, 30)
                a, b = [(0, 1), (1, 2), (1, 512)][rep % 3]
                c = [int(x) for x in oracle.cost(L, a, b)]
                asg = oracle.balance(L, D, a, b)
                lpt = int(asg.loads.max())
                opt = brute_opt(c, D)
                assert lpt >= opt
                # Graham: LPT <= (4/3 - 1/(3D)) OPT  <=>  3D*LPT <= (4D-1)*OPT
                assert 3 * D * lpt <= (4 * D - 1) * opt


def test_special_cases():
    # all equal -> round robin
    L = np.full(23, 100, dtype=np.int32)
    asg = oracle.balance(L, 5, 1, 512)
    assert asg.inst.tolist() == [s % 5 for s in range(23)]
    # D = 1 -> order is the stable descending sort
    L = wl.random_lengths(5, 200, 0, 30)
    asg = oracle.balance(L, 1, 1, 1)
    assert asg.order.tolist() == sorted(range(200), key=lambda s: (-int(L[s]), s))
    assert asg.cu_of(0).tolist() == [0] + np.cumsum(L[asg.order]).tolist()
    # n <= D -> one per instance in sorted order, rest empty
    L = np.array([5, 9, 7], dtype=np.int32)
    asg = oracle.balance(L, 6, 1, 0)
    assert asg.inst.tolist() == [2, 0, 1]
    assert asg.seq_off.tolist() == [0, 1, 2, 3, 3, 3, 3]
    assert asg.cu_seqlens.tolist() == [0, 9, 0, 7, 0, 5, 0, 0, 0]
    # n = 0
    asg = oracle.balance(np.zeros(0, np.int32), 3, 1, 1)
    assert asg.seq_off.tolist() == [0, 0, 0, 0] and asg.cu_seqlens.tolist() == [0, 0, 0]
    assert asg.tok_off.tolist() == [0, 0, 0, 0]
    with pytest.raises(oracle.OracleError):
        oracle.balance(np.array([1], np.int32), 0, 1, 1)


@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_pack_tag_and_inverse(cid):
    w = wl.WORKLOADS[cid]
    L = wl.draw_lengths(w)
    if cid == 4:
        L = L[:300] // 16  # keep the host copy small; the law's shape is kept
    H = min(w.H, 64)
    asg = oracle.balance(L, w.D, w.a, w.b)
    check_layout(L, w.D, asg)
    T = int(L.sum())
    tokens = wl.token_tag_np(np.arange(T), H)
    packed = oracle.pack(tokens, L, asg)
    rmap = oracle.row_map(L, asg)
    # permutation invariant: every source row exactly once
    assert np.array_equal(np.sort(rmap), np.arange(T))
    # tag test: each packed row equals g(source row)
    assert np.array_equal(packed, wl.token_tag_np(rmap, H))
    # rows of a sequence are contiguous and in order
    src_cu = np.concatenate([[0], np.cumsum(L)])
    for i in range(w.D):
        cu = asg.cu_of(i)
        for j, s in enumerate(asg.seqs_of(i)):
            lo = int(asg.tok_off[i]) + int(cu[j])
            assert np.array_equal(rmap[lo: lo + L[s]], np.arange(src_cu[s], src_cu[s] + L[s]))
    # inverse: scattering back reproduces the source
    back = np.empty_like(tokens)
    back[rmap] = packed
    assert np.array_equal(back, tokens)
    # a sub-range of instances is the matching slice
    part = oracle.pack(tokens, L, asg, 1, 3)
    assert np.array_equal(part, packed[int(asg.tok_off[1]): int(asg.tok_off[3])])


def test_balancing_beats_contiguous_split():
    for cid in (2, 3, 4):
        w = wl.WORKLOADS[cid]
        L = wl.draw_lengths(w)
        asg = oracle.balance(L, w.D, w.a, w.b)
        before = oracle.load_ratio(L, (np.arange(w.n) * w.D) // w.n, w.D, w.a, w.b)
        after = oracle.load_ratio(L, asg.inst, w.D, w.a, w.b)
        assert after <= before and after < 1.05
        assert abs(after - float(asg.loads.max() / asg.loads.mean())) < 1e-12


def test_workload_laws():
    for cid, w in wl.WORKLOADS.items():
        L = wl.draw_lengths(w)
        assert L.dtype == np.int32 and len(L) == w.n
        assert np.array_equal(L, wl.draw_lengths(w))  # seeded
    L2 = wl.draw_lengths(wl.WORKLOADS[2])
    assert set(np.unique(L2)) <= {0, 256, 576, 1024, 2304}
    assert 0.1 < np.mean(L2 == 0) < 0.3
    L3 = wl.draw_lengths(wl.WORKLOADS[3])
    assert 0.12 < np.mean(L3 == 0) < 0.28 and L3[L3 > 0].min() >= 25 and L3.max() <= 1500
    L4 = wl.draw_lengths(wl.WORKLOADS[4])
    assert L4.min() >= 64 and L4.max() <= 8192 and 1500 < np.median(L4) < 2700
    split = wl.draw_modality_split(wl.WORKLOADS[4], L4)
    assert np.array_equal(split.sum(axis=1), L4) and split.min() >= 0
    # Dirichlet(0.3,..): compositions are spiky (one modality usually dominates)
    assert np.mean(split.max(axis=1) / L4 > 0.6) > 0.5
    L5 = wl.draw_lengths(wl.WORKLOADS[5])
    assert L5.max() <= 32768 and L5.min() >= 64


# ----------------------------------------------------------------------------
# Rearrangement composition (Sec. 5.3): Pi_M o Pi_E^-1 in one pass
# ----------------------------------------------------------------------------
def modality_case(cid, shrink=1, keep=None, seed=0):
    """Lengths, three-way modality split and the row offset of every modality inside the
    example's interleaved sequence (modalities ordered per example by a seeded draw)."""
    w = wl.WORKLOADS[cid]
    L = wl.draw_lengths(w)
    if keep is not None:
        L = L[:keep]
    L = (L // shrink).astype(np.int32)
    split = wl.draw_modality_split(w, L)
    sub_off = wl.draw_interleave_offsets(split, 1000 + seed)
    return w, L, split, sub_off


def dst_starts(asg, D):
    """Row of the first token of every example in the packed LLM batch, from the
    assignment's fields alone."""
    start = np.zeros(len(asg.order), dtype=np.int64)
    for i in range(D):
        cu = asg.cu_of(i)
        for j, s in enumerate(asg.seqs_of(i)):
            start[s] = int(asg.tok_off[i]) + int(cu[j])
    return start


def encoder_rows(sub, easg, De, H, salt):
    """The encoder phase's output in ITS packed order: row r of example s carries the tag of
    (salt + original-order row).  Built without the oracle's pack."""
    cu0 = np.concatenate([[0], np.cumsum(sub, dtype=np.int64)])
    src = np.empty(int(cu0[-1]), dtype=np.int64)
    if easg is None:
        src[:] = np.arange(cu0[-1])
    else:
        st = dst_starts(easg, De)
        for s in range(len(sub)):
            src[st[s]: st[s] + sub[s]] = np.arange(cu0[s], cu0[s + 1])
    return wl.token_tag_np(salt + src, H), cu0


@pytest.mark.parametrize("cid,shrink,keep", [(1, 1, None), (4, 16, 400), (2, 4, 600)])
def test_pack_composed_tag(cid, shrink, keep):
    w, L, split, sub_off = modality_case(cid, shrink, keep)
    H, Dm, De = 24, w.D, max(2, w.D // 2)
    masg = oracle.balance(L, Dm, w.a, w.b)
    start = dst_starts(masg, Dm)
    T = int(L.sum())
    packed = np.full((T, H), 0xFFFF, dtype=np.uint16)
    want = np.empty((T, H), dtype=np.uint16)
    for m in range(3):
        sub = split[:, m].copy()
        # text (m = 0) never left its instance: original order; encoders have their own dispatch
        easg = None if m == 0 else oracle.balance(sub, De, 1, 4 + m)
        salt = m * (1 << 30)
        rows, cu0 = encoder_rows(sub, easg, De, H, salt)
        oracle.pack_composed(rows, packed, sub, sub_off[:, m], easg, masg)
        for s in range(len(L)):
            d0 = start[s] + sub_off[s, m]
            want[d0: d0 + sub[s]] = wl.token_tag_np(salt + np.arange(cu0[s], cu0[s + 1]), H)
    # the three modalities tile every destination row exactly once and carry the right rows
    assert np.array_equal(packed, want)


def test_pack_composed_equals_reset_interleave_pack():
    """Two-step definition: undo Pi_E, interleave in original order, then apply Pi_M with the
    plain pack; one composed pass per modality must give the same buffer."""
    w, L, split, sub_off = modality_case(3, 2, 500, seed=3)
    H, Dm, De = 16, w.D, 5
    masg = oracle.balance(L, Dm, w.a, w.b)
    T = int(L.sum())
    src_cu = np.concatenate([[0], np.cumsum(L, dtype=np.int64)])
    inter = np.empty((T, H), dtype=np.uint16)
    packed = np.zeros((T, H), dtype=np.uint16)
    for m in range(3):
        sub = split[:, m].copy()
        easg = oracle.balance(sub, De, 2, 1) if m else None
        rows, cu0 = encoder_rows(sub, easg, De, H, 7 * m)
        for s in range(len(L)):
            a = src_cu[s] + sub_off[s, m]
            inter[a: a + sub[s]] = wl.token_tag_np(7 * m + np.arange(cu0[s], cu0[s + 1]), H)
        oracle.pack_composed(rows, packed, sub, sub_off[:, m], easg, masg)
    assert np.array_equal(packed, oracle.pack(inter, L, masg))
    # an instance sub-range is the matching slice and leaves nothing else touched
    part = np.zeros((int(masg.tok_off[4] - masg.tok_off[2]), H), dtype=np.uint16)
    for m in range(3):
        sub = split[:, m].copy()
        easg = oracle.balance(sub, De, 2, 1) if m else None
        rows, _ = encoder_rows(sub, easg, De, H, 7 * m)
        oracle.pack_composed(rows, part, sub, sub_off[:, m], easg, masg, 2, 4)
    assert np.array_equal(part, packed[int(masg.tok_off[2]): int(masg.tok_off[4])])


def test_pack_composed_special_cases():
    w = wl.WORKLOADS[1]
    L = wl.draw_lengths(w)
    H = 8
    asg = oracle.balance(L, w.D, w.a, w.b)
    T = int(L.sum())
    tokens = wl.token_tag_np(np.arange(T), H)
    zero = np.zeros(len(L), dtype=np.int32)
    # identity source, whole sequences, offset 0: the plain pack
    out = np.zeros_like(tokens)
    oracle.pack_composed(tokens, out, L, zero, None, asg)
    assert np.array_equal(out, oracle.pack(tokens, L, asg))
    # source order = destination order: the composition is the identity map
    out2 = np.zeros_like(tokens)
    oracle.pack_composed(out, out2, L, zero, asg, asg)
    assert np.array_equal(out2, out)
    # empty modality: nothing is written
    sent = np.full_like(tokens, 0xABCD)
    oracle.pack_composed(tokens[:0], sent, zero, zero, None, asg)
    assert (sent == 0xABCD).all()
    # a sub-sequence that overruns its interleaved sequence is refused
    off = zero.copy()
    off[int(np.argmax(L))] = 1
    with pytest.raises(oracle.OracleError):
        oracle.pack_composed(tokens, out, L, off, None, asg)
    # an encoder segment shorter than the sub-sequence is refused (a longer one is a padded slot)
    longer = (L + 1).astype(np.int32)
    big = np.zeros((int(longer.sum()), H), dtype=tokens.dtype)
    with pytest.raises(oracle.OracleError):
        oracle.pack_composed(tokens, big, longer, zero, asg, oracle.balance(longer, w.D, w.a, w.b))
    shorter = np.maximum(L - 1, 0).astype(np.int32)
    oracle.pack_composed(tokens, big, shorter, zero, asg, asg)


# ----------------------------------------------------------------------------
# communication-volume matrix (Sec. 5.2.2)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_comm_volume(cid):
    w = wl.WORKLOADS[cid]
    L = wl.draw_lengths(w)
    asg = oracle.balance(L, w.D, w.a, w.b)
    V, inter = oracle.comm_volume(L, asg, w.D, node=4)
    src = (np.arange(w.n, dtype=np.int64) * w.D) // w.n
    # a library scatter-add gives the same matrix
    want = np.zeros((w.D, w.D), dtype=np.int64)
    np.add.at(want, (src, asg.inst), L.astype(np.int64))
    assert np.array_equal(V.astype(np.int64), want)
    # rows: what an instance sampled; columns: what an instance ends up with
    assert np.array_equal(V.sum(axis=1).astype(np.int64), np.bincount(src, weights=L, minlength=w.D).astype(np.int64))
    assert np.array_equal(V.sum(axis=0).astype(np.int64), np.diff(asg.tok_off))
    off_node = (np.arange(w.D)[:, None] // 4) != (np.arange(w.D)[None, :] // 4)
    assert np.array_equal(inter.astype(np.int64), (want * off_node).sum(axis=1))
    # explicit source instances; nothing moves when every sequence stays where it was sampled
    perm = (np.arange(w.n) * 7 + 3) % w.D
    V2, _ = oracle.comm_volume(L, asg, w.D, src_inst=perm)
    want2 = np.zeros((w.D, w.D), dtype=np.int64)
    np.add.at(want2, (perm, asg.inst), L.astype(np.int64))
    assert np.array_equal(V2.astype(np.int64), want2)
    V3, inter3 = oracle.comm_volume(L, asg, w.D, src_inst=asg.inst, node=1)
    assert np.array_equal(V3.astype(np.int64), np.diag(np.diff(asg.tok_off))) and not inter3.any()
    with pytest.raises(oracle.OracleError):
        oracle.comm_volume(L, asg, w.D, src_inst=np.full(w.n, w.D, np.int32))
