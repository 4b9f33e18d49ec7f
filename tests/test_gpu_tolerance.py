"""HIP orch_balance_tolerance (Appendix A, third algorithm) vs the CPU oracle: bit-exact outputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_23830_amd as orch
import workloads as wl
from gpu_common import assert_assignment_equal, bits

pytestmark = pytest.mark.gpu


def check(L, D, v, a, b, dev):
    Ld = torch.from_numpy(np.ascontiguousarray(L, dtype=np.int32)).to(dev)
    asg = orch.balance_tolerance(Ld, D, v, a, b)
    torch.cuda.synchronize()
    assert_assignment_equal(asg, oracle.balance_tolerance(L, D, v, a, b))
    return Ld, asg


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("v", [0, 64, 2048, 1 << 40])
def test_configs(gpu_device, cid, v):
    w = wl.WORKLOADS[cid]
    check(wl.draw_lengths(w), w.D, v, w.a, w.b, gpu_device)


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes(gpu_device, seed):
    u = wl.uniform01(400 + seed, 1, 4)
    n = 1 + int(u[0] * 3000)
    D = 1 + int(u[1] * [60, 128, 600, 1024][seed % 4])
    hi = [3, 40, 1500, 100000][seed % 4]
    L = wl.random_lengths(410 + seed, n, 0 if seed % 2 else 1, hi, zero_frac=0.2 if seed % 3 == 0 else 0.0)
    v = int(u[2] * 3 * hi)
    check(L, D, v, 1 + seed, 7, gpu_device)


def test_edge_cases(gpu_device):
    dev = gpu_device
    check(np.zeros(0, np.int32), 3, 5, 1, 1, dev)
    check(np.zeros(10, np.int32), 3, 5, 1, 1, dev)
    check(np.array([300], np.int32), 1, 5, 1, 1, dev)
    check(np.array([9, 3], np.int32), 4, 5, 1, 1, dev)
    check(np.full(1000, 17, np.int32), 7, 20, 2, 3, dev)
    for D in (63, 64, 65, 128, 129, 256, 257, 512, 513, 1024):  # every register-count variant, ragged
        check(wl.random_lengths(D, 2500, 1, 300), D, 150, 1, 1, dev)
    check(np.array([2**31 - 1, 2**30, 5], np.int32), 3, 1 << 20, 1, 1, dev)
    # just inside the 32-bit form (longest < 2^30, all together < 2^32): squares near 2^61, the
    # comparison by leading bits drops 30 of them, near-equal squares go to the exact comparison
    near = np.array([2**29 + 3, 2**29 + 1, 2**29, 2**29, 2**29 - 1, 2**29 - 5, 2**29 - 9, 77, 5, 5, 1], np.int32)
    for D, v in ((2, 1000), (3, 0), (3, 1 << 31), (5, 1 << 29), (40, 7), (100, 1 << 33)):
        check(near, D, v, 0, 1, dev)
    # many equal lengths: equal squares all the time (the exact comparison decides nearly every step)
    for D in (4, 31, 32, 33, 64, 200):
        check(np.repeat(np.array([900, 411, 411, 30, 7], np.int32), 120), D, 500, 1, 1, dev)
    # more than 2^32 tokens in total: the 64-bit form of the kernel
    big = np.concatenate([np.full(5, 2**30, np.int32), wl.random_lengths(9, 300, 1, 5000)])
    for D, v in ((5, 3000), (70, 1 << 29), (300, 0)):
        check(big, D, v, 0, 1, dev)


def test_data_errors_on_device(gpu_device):
    dev = gpu_device
    for L, D, a in ((np.array([5, -1, 7], np.int32), 2, 1),          # negative length
                    (np.full(4, 2**31 - 1, np.int32), 1, 0),         # squares reach 2^63
                    (np.array([2**31 - 1], np.int32), 1, 2**40)):    # load overflows
        asg = orch.balance_tolerance(torch.from_numpy(L).to(dev), D, 3, a, 1)
        torch.cuda.synchronize()
        assert int(asg.dev_status.item()) == -5
    asg = orch.balance_tolerance(torch.from_numpy(np.array([5, 1, 7], np.int32)).to(dev), 2, 3, 1, 1)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == 0


def test_assignment_drives_pack(gpu_device):
    w = wl.WORKLOADS[3]
    L = wl.draw_lengths(w)
    Ld, asg = check(L, w.D, 256, w.a, w.b, gpu_device)
    T, H = int(L.sum()), 64
    packed = orch.pack(wl.token_tag_torch(0, T, H, gpu_device), Ld, asg)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == 0
    ref = oracle.balance_tolerance(L, w.D, 256, w.a, w.b)
    assert np.array_equal(bits(packed), oracle.pack(wl.token_tag_np(np.arange(T), H), L, ref))
