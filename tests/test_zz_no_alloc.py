"""orch_balance_static (the entry point that allocates nothing) against orch_balance:
bit-exact outputs on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_23830_amd as orch
import workloads as wl
from gpu_common import assert_assignment_equal

pytestmark = pytest.mark.gpu


def _fields(a):
    n, D = a.n, a.D
    size = {"inst": n, "order": n, "seq_off": D + 1, "tok_off": D + 1, "cu_seqlens": n + D, "loads": D,
            "dev_status": 1}
    return [getattr(a, f).cpu().numpy()[:m] for f, m in size.items()]


def _compare(L, D, a, b, dev):
    Ld = torch.from_numpy(np.ascontiguousarray(L, dtype=np.int32)).to(dev)
    n = Ld.numel()
    got = orch.Assignment.empty(n, D, dev)
    before = torch.cuda.memory_allocated(dev)
    orch.balance_static(Ld, D, a, b, got)
    assert torch.cuda.memory_allocated(dev) == before   # the binding allocated nothing either
    torch.cuda.synchronize()
    want = orch.balance(Ld, D, a, b)
    torch.cuda.synchronize()
    for g, w_ in zip(_fields(got), _fields(want)):
        assert np.array_equal(g, w_)
    assert_assignment_equal(got, oracle.balance(L, D, a, b))


def test_two_calls_second_smaller(gpu_device):
    w5, w3 = wl.WORKLOADS[5], wl.WORKLOADS[3]
    _compare(wl.draw_lengths(w5), w5.D, w5.a, w5.b, gpu_device)     # 32768 sequences, 256 instances
    _compare(wl.draw_lengths(w3), w3.D, w3.a, w3.b, gpu_device)     # 1024 sequences: stale scratch beyond it
    _compare(wl.random_lengths(77, 9, 0, 50), 4, 0, 1, gpu_device)
    _compare(np.zeros(0, dtype=np.int32), 3, 1, 1, gpu_device)


def test_size_limit_is_an_error(gpu_device):
    nmax = orch.balance_static_max_n()
    assert nmax >= 32768
    L = torch.ones(nmax + 1, dtype=torch.int32, device=gpu_device)
    out = orch.Assignment.empty(nmax + 1, 8, gpu_device)
    with pytest.raises(orch.OrchError) as e:
        orch.balance_static(L, 8, 0, 1, out)
    assert e.value.code == -3 and "scratch" in str(e.value)
    # the largest accepted size still runs and matches
    Lmax = wl.random_lengths(5, nmax, 1, 4000)
    _compare(Lmax, 64, 1, 100, gpu_device)
