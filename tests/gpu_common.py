"""Shared helpers of the GPU parity tests (HIP path vs CPU oracle)."""
import numpy as np
import torch

import oracle
import paper_2503_23830_amd as orch
import workloads as wl


def bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def run_balance(L: np.ndarray, D: int, a: int, b: int, dev):
    Ld = torch.from_numpy(np.ascontiguousarray(L, dtype=np.int32)).to(dev)
    asg = orch.balance(Ld, D, a, b)
    torch.cuda.synchronize()
    return Ld, asg


def assert_assignment_equal(asg, ref):
    assert int(asg.dev_status.item()) == 0
    n, D = asg.n, asg.D
    assert np.array_equal(asg.inst.cpu().numpy()[:n], ref.inst)
    assert np.array_equal(asg.order.cpu().numpy()[:n], ref.order)
    assert np.array_equal(asg.seq_off.cpu().numpy(), ref.seq_off)
    assert np.array_equal(asg.tok_off.cpu().numpy(), ref.tok_off)
    assert np.array_equal(asg.cu_seqlens.cpu().numpy()[: n + D], ref.cu_seqlens)
    assert np.array_equal(asg.loads.cpu().numpy().view(np.uint64), ref.loads)


def attn_tolerance_check(out_gpu: np.ndarray, want: np.ndarray):
    """bf16 inputs, fp32 accumulation vs the fp64 oracle on the same inputs:
    max-abs <= 2e-2 and mean-abs <= 2e-3 over all compared elements."""
    err = np.abs(out_gpu.astype(np.float64) - want)
    assert np.isfinite(out_gpu).all()
    assert err.max() <= 2e-2, err.max()
    assert err.mean() <= 2e-3, err.mean()
    return float(err.max()), float(err.mean())
