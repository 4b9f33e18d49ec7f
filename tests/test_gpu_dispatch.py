"""HIP orch_balance vs the CPU oracle: bit-exact assignment and layout."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_23830_amd as orch
import workloads as wl
from gpu_common import assert_assignment_equal, run_balance

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_workload_configs(gpu_device, cid):
    w = wl.WORKLOADS[cid]
    L = wl.draw_lengths(w)
    _, asg = run_balance(L, w.D, w.a, w.b, gpu_device)
    assert_assignment_equal(asg, oracle.balance(L, w.D, w.a, w.b))


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes(gpu_device, seed):
    n = [0, 1, 2, 63, 64, 65, 1000, 1025, 4097, 20000, 333, 777, 5000, 128, 2048, 9][seed]
    D = [1, 2, 3, 7, 64, 65, 128, 200, 256, 257, 512, 1000, 1024, 5, 33, 16][(seed * 5) % 16]
    a, b = [(1, 512), (0, 1), (1, 0), (3, 11)][seed % 4]
    L = wl.random_lengths(900 + seed, n, 0, [8, 100, 5000, 40000][seed % 4], zero_frac=0.2 if seed % 3 == 0 else 0.0)
    _, asg = run_balance(L, D, a, b, gpu_device)
    assert_assignment_equal(asg, oracle.balance(L, D, a, b))


def test_many_ties_and_equal_lengths(gpu_device):
    L = np.full(1000, 77, dtype=np.int32)
    _, asg = run_balance(L, 13, 1, 512, gpu_device)
    ref = oracle.balance(L, 13, 1, 512)
    assert_assignment_equal(asg, ref)
    assert asg.inst.cpu().numpy().tolist() == [s % 13 for s in range(1000)]
    L = wl.random_lengths(5, 6000, 0, 3, zero_frac=0.3)
    _, asg = run_balance(L, 48, 0, 1, gpu_device)
    assert_assignment_equal(asg, oracle.balance(L, 48, 0, 1))


@pytest.mark.parametrize("D", [8, 32, 64, 100, 256, 700])
def test_mixed_round_lengths(gpu_device, D):
    """Costs spanning many orders of magnitude: some rounds hand an item to every
    instance, others stop after one or two, and a zero-cost tail ends the batch."""
    rng = np.random.default_rng(1000 + D)
    n = 6 * D + 37
    L = np.exp(rng.normal(5.0, 2.5, n)).astype(np.int64).clip(0, 200000).astype(np.int32)
    L[rng.random(n) < 0.05] = 0
    for a, b in ((1, 0), (1, 4096), (0, 1)):
        _, asg = run_balance(L, D, a, b, gpu_device)
        assert_assignment_equal(asg, oracle.balance(L, D, a, b))


def test_large_instance_counts_use_the_lds_kernel(gpu_device):
    for D in (1025, 2560, 4096):
        L = wl.random_lengths(D, 9000, 1, 3000)
        _, asg = run_balance(L, D, 1, 100, gpu_device)
        assert_assignment_equal(asg, oracle.balance(L, D, 1, 100))


def test_wide_keys(gpu_device):
    # costs up to ~2^50 (sum < 2^63): seven radix passes
    L = wl.random_lengths(3, 3000, 1, 2 ** 20)
    a, b = 2 ** 10, 12345
    _, asg = run_balance(L, 32, a, b, gpu_device)
    assert_assignment_equal(asg, oracle.balance(L, 32, a, b))


def test_data_errors_set_dev_status(gpu_device):
    L = np.array([5, -3, 7], dtype=np.int32)
    _, asg = run_balance(L, 2, 1, 1, gpu_device)
    assert int(asg.dev_status.item()) == -5
    with pytest.raises(oracle.OracleError):
        oracle.balance(L, 2, 1, 1)
    L = np.array([2 ** 31 - 1] * 4, dtype=np.int32)
    _, asg = run_balance(L, 2, 2 ** 40, 0, gpu_device)
    assert int(asg.dev_status.item()) == -5
    # the flag is cleared by the next good call on the same buffers
    Lg = torch.from_numpy(np.array([4, 2, 9], dtype=np.int32)).to(gpu_device)
    orch.balance(Lg, 2, 1, 1, out=asg)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == 0


def test_deterministic_rerun(gpu_device):
    w = wl.WORKLOADS[4]
    L = wl.draw_lengths(w)
    _, a1 = run_balance(L, w.D, w.a, w.b, gpu_device)
    _, a2 = run_balance(L, w.D, w.a, w.b, gpu_device)
    for f in ("inst", "order", "seq_off", "tok_off", "cu_seqlens", "loads"):
        assert torch.equal(getattr(a1, f), getattr(a2, f))


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_comm_volume(gpu_device, cid):
    """orch_comm_volume (Sec. 5.2.2) vs the oracle: every cell and the inter-node sums, bit-exact."""
    import torch

    w = wl.WORKLOADS[cid]
    L = wl.draw_lengths(w)
    Ld, asg = run_balance(L, w.D, w.a, w.b, gpu_device)
    ref = oracle.balance(L, w.D, w.a, w.b)
    V, inter = orch.comm_volume(Ld, asg, w.D, node=8)
    torch.cuda.synchronize()
    Vr, ir = oracle.comm_volume(L, ref, w.D, node=8)
    assert np.array_equal(V.cpu().numpy().view(np.uint64), Vr)
    assert np.array_equal(inter.cpu().numpy().view(np.uint64), ir)
    # explicit source instances, another source count, no node output asked for
    src = ((np.arange(w.n) * 5 + 1) % 3).astype(np.int32)
    V2, _ = orch.comm_volume(Ld, asg, 3, src_inst=torch.from_numpy(src).to(gpu_device))
    torch.cuda.synchronize()
    assert np.array_equal(V2.cpu().numpy().view(np.uint64), oracle.comm_volume(L, ref, 3, src_inst=src)[0])
    assert int(asg.dev_status.item()) == 0
    # a source instance outside its range is a data error
    bad = torch.from_numpy(np.full(w.n, 3, np.int32)).to(gpu_device)
    orch.comm_volume(Ld, asg, 3, src_inst=bad)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == -5
