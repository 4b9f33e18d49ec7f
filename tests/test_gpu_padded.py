"""HIP orch_balance_padded (Algorithm 2, Sec. 5.1) vs the CPU oracle: every output bit-exact; rows
moved into the padded layout and out of it by orch_pack_composed."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_23830_amd as orch
import workloads as wl
from gpu_common import assert_assignment_equal, bits

pytestmark = pytest.mark.gpu

GUARD = 0x7C7C


def run_padded(L, D, a, b, dev):
    Ld = torch.from_numpy(np.ascontiguousarray(L, dtype=np.int32)).to(dev)
    bound = torch.full((1,), -1, dtype=torch.int64, device=dev)
    asg = orch.balance_padded(Ld, D, a, b, bound=bound)
    torch.cuda.synchronize()
    return Ld, asg, int(bound.item())


def check(L, D, a, b, dev):
    _, asg, bound = run_padded(L, D, a, b, dev)
    ref, rbound = oracle.balance_padded(L, D, a, b)
    assert bound == rbound
    assert_assignment_equal(asg, ref)
    return asg, ref


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_configs(gpu_device, cid):
    w = wl.WORKLOADS[cid]
    check(wl.draw_lengths(w), w.D, w.a, w.b, gpu_device)


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes(gpu_device, seed):
    u = wl.uniform01(300 + seed, 1, 4)
    n = 1 + int(u[0] * 3000)
    D = 1 + int(u[1] * (300 if seed % 4 else 4096))
    hi = [3, 40, 1500, 100000][seed % 4]
    L = wl.random_lengths(310 + seed, n, 0 if seed % 2 else 1, hi, zero_frac=0.2 if seed % 3 == 0 else 0.0)
    check(L, D, 1 + seed, 7, gpu_device)


def test_edge_cases(gpu_device):
    dev = gpu_device
    check(np.zeros(0, np.int32), 3, 1, 1, dev)                       # n = 0
    check(np.zeros(10, np.int32), 3, 1, 1, dev)                      # all empty
    check(np.array([300], np.int32), 1, 1, 1, dev)                   # one sequence, one instance
    check(np.array([9, 3], np.int32), 4, 1, 1, dev)                  # n < D
    check(np.full(1000, 17, np.int32), 7, 2, 3, dev)                 # all equal
    check(np.arange(1, 2049, dtype=np.int32)[::-1].copy(), 64, 1, 1, dev)
    check(np.array([1, 100, 1, 1], np.int32), 2, 1, 1, dev)          # bound below the longest
    check(wl.random_lengths(5, 4096, 1, 9), 4096, 1, 1, dev)         # D = n = 4096
    L = wl.random_lengths(6, 40000, 0, 2000, zero_frac=0.1)          # n above the LDS-resident limit
    check(L, 50, 1, 1, dev)
    # large lengths: bound range of 2^46, costs near the u64 limit
    check(np.array([2**31 - 1, 2**30, 5, 2**31 - 1], np.int32), 4, 0, 1, dev)


def test_data_errors_on_device(gpu_device):
    dev = gpu_device
    _, asg, _ = run_padded(np.array([5, -1, 7], np.int32), 2, 1, 1, dev)
    assert int(asg.dev_status.item()) == -5
    # a padded batch of more than 2^31 - 1 rows
    _, asg, _ = run_padded(np.full(3, 2**30, np.int32), 1, 0, 1, dev)
    assert int(asg.dev_status.item()) == -5
    # cost overflow: a * max^2 beyond u64
    _, asg, _ = run_padded(np.array([2**31 - 1], np.int32), 1, 2**40, 1, dev)
    assert int(asg.dev_status.item()) == -5
    # and a following good call clears the status
    _, asg, _ = run_padded(np.array([5, 1, 7], np.int32), 2, 1, 1, dev)
    assert int(asg.dev_status.item()) == 0


def test_rows_into_and_out_of_the_padded_batch(gpu_device):
    """C3 (audio): rows in original order go into the padded encoder batches, and from there,
    composed, into the unpadded LLM-phase batch of another assignment."""
    dev = gpu_device
    w = wl.WORKLOADS[3]
    L = wl.draw_lengths(w)
    T, H = int(L.sum()), 128
    Ld, pasg, _ = run_padded(L, w.D, w.a, w.b, dev)
    pref, _ = oracle.balance_padded(L, w.D, w.a, w.b)
    zero = torch.zeros(len(L), dtype=torch.int32, device=dev)
    tokens = wl.token_tag_torch(0, T, H, dev)
    tok_np = wl.token_tag_np(np.arange(T), H)
    prow = int(pref.tok_off[w.D])
    padded = torch.full((prow, H), GUARD, dtype=torch.int16, device=dev)
    orch.pack_composed(tokens, padded, Ld, zero, None, pasg)
    torch.cuda.synchronize()
    assert int(pasg.dev_status.item()) == 0
    want = np.full((prow, H), GUARD, dtype=np.uint16)
    oracle.pack_composed(tok_np, want, L, np.zeros(len(L), np.int32), None, pref)
    assert np.array_equal(bits(padded), want)
    assert (want == GUARD).all(axis=1).sum() == prow - T  # the pad rows, untouched
    # the plain pack refuses a padded assignment
    out = torch.full((prow, H), GUARD, dtype=torch.int16, device=dev)
    orch.pack(tokens, Ld, pasg, out=out)
    torch.cuda.synchronize()
    assert int(pasg.dev_status.item()) == -5 and bool((out == GUARD).all())
    pasg.dev_status.zero_()
    # padded encoder batch -> LLM batch (here: the same lengths under Algorithm 1, D = 5)
    masg = orch.balance(Ld, 5, 1, 64)
    mref = oracle.balance(L, 5, 1, 64)
    llm = torch.full((T, H), GUARD, dtype=torch.int16, device=dev)
    orch.pack_composed(padded, llm, Ld, zero, pasg, masg)
    torch.cuda.synchronize()
    assert int(masg.dev_status.item()) == 0
    assert np.array_equal(bits(llm), oracle.pack(tok_np, L, mref))
