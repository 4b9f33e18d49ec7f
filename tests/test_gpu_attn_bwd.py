"""HIP orch_varlen_attn_bwd vs the fp64 CPU oracle.

Tolerance (derived, not from the paper): every term of a gradient passes bf16 roundings (P or dS
before the second product, at head_dim 128 both of them for dk, and the output), each at most 2^-9
relative to the TERM; a gradient
element is a sum of many such terms that partly cancel, so its error scales with the size of the
gradients of the tensor, not with the element: max |got - want| <= 1e-2 + 2^-7 max|want| over the
compared tensor, mean-abs <= 2e-3, and the rms error is at most 5e-3 of the rms gradient (the
discriminating bound: a dropped or wrong term shows as a relative rms error of order 1)."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2503_23830_amd as orch
import workloads as wl
from gpu_common import bits

pytestmark = pytest.mark.gpu
NT = min(16, os.cpu_count() or 1)


def grad_check(got: np.ndarray, want: np.ndarray):
    assert np.isfinite(got).all()
    err = np.abs(got.astype(np.float64) - want)
    assert err.max() <= 1e-2 + 2.0 ** -7 * np.abs(want).max(), float(err.max())
    assert err.mean() <= 2e-3, float(err.mean())
    rms = np.sqrt((want ** 2).mean())
    if rms > 0:
        assert np.sqrt((err ** 2).mean()) <= 5e-3 * rms


def make(seed, T, Hq, Hkv, d, dev):
    return (wl.normal_bf16_torch((T, Hq, d), seed, 1, dev), wl.normal_bf16_torch((T, Hkv, d), seed, 2, dev),
            wl.normal_bf16_torch((T, Hkv, d), seed, 3, dev), wl.normal_bf16_torch((T, Hq, d), seed, 4, dev))


def fwd_bwd(q, k, v, do, cud, causal, scale=0.0, fill=True):
    T, Hq, d = q.shape
    lse = torch.zeros((Hq, T), dtype=torch.float32, device=q.device)
    out = orch.varlen_attn_fwd(q, k, v, cud, causal, scale=scale, lse=lse)
    nan = float("nan")
    dq = torch.full_like(q, nan) if fill else None
    dk = torch.full_like(k, nan) if fill else None
    dv = torch.full_like(v, nan) if fill else None
    dq, dk, dv = orch.varlen_attn_bwd(q, k, v, out, lse, do, cud, causal, scale=scale, dq=dq, dk=dk, dv=dv)
    torch.cuda.synchronize()
    return dq, dk, dv


def run_full(cu, Hq, Hkv, d, causal, dev, seed=1, scale=0.0, total=None):
    cu = np.ascontiguousarray(cu, dtype=np.int32)
    T = int(cu[-1]) if total is None else total
    q, k, v, do = make(seed, T, Hq, Hkv, d, dev)
    dq, dk, dv = fwd_bwd(q, k, v, do, torch.from_numpy(cu).to(dev), causal, scale)
    wq, wk, wv = oracle.attn_bwd(bits(q), bits(k), bits(v), bits(do), cu, causal, scale=scale, nthreads=NT)
    rows = np.zeros(T, dtype=bool)
    for t in range(len(cu) - 1):
        rows[cu[t]: cu[t + 1]] = True
    for got, want in ((dq, wq), (dk, wk), (dv, wv)):
        g = got.float().cpu().numpy()
        grad_check(g[rows], want[rows])
        assert np.isnan(g[~rows]).all()  # rows outside every sequence are never written


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("Hq,Hkv,d", [(4, 4, 64), (4, 1, 128), (8, 8, 128), (6, 2, 64)])
def test_small_ragged(gpu_device, causal, Hq, Hkv, d):
    L = [1, 0, 37, 128, 129, 64, 63, 65, 300, 0, 2, 513]
    run_full(np.concatenate([[0], np.cumsum(L)]), Hq, Hkv, d, causal, gpu_device)


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 8, 128), (4, 2, 64)])
def test_tile_boundaries(gpu_device, causal, Hq, Hkv, d):
    """Lengths around 32-row blocks, 64-row streamed tiles and the 128 rows a workgroup owns."""
    L = [1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 320, 511, 512, 767]
    run_full(np.concatenate([[0], np.cumsum(L)]), Hq, Hkv, d, causal, gpu_device, seed=7)


@pytest.mark.parametrize("causal", [True, False])
def test_long_rows_wide_group(gpu_device, causal):
    """Eight q-heads per kv-head and sequences of many 64-row tiles: the key-stationary kernels walk
    heads x tiles through their LDS stages many times over."""
    run_full(np.array([0, 1500, 1500 + 257]), 16, 2, 128, causal, gpu_device, seed=11)


def test_explicit_scale_and_padding_rows(gpu_device):
    cu = np.array([0, 200, 200, 431], dtype=np.int32)
    run_full(cu, 4, 2, 128, True, gpu_device, scale=0.05, total=500)
    run_full(cu, 4, 2, 64, False, gpu_device, scale=0.2, total=500)


def test_c1_all_instances(gpu_device):
    w = wl.WORKLOADS[1]
    ref = oracle.balance(wl.draw_lengths(w), w.D, w.a, w.b)
    for i in range(w.D):
        run_full(ref.cu_of(i), w.Hq, w.Hkv, w.d, w.causal, gpu_device, seed=10 + i)


def test_closed_forms_on_device(gpu_device):
    dev = gpu_device
    Hq, Hkv, d = 4, 2, 128
    cu = np.array([0, 1, 150, 400], dtype=np.int32)
    q, k, v, do = make(5, 400, Hq, Hkv, d, dev)
    cud = torch.from_numpy(cu).to(dev)
    dq, dk, dv = fwd_bwd(q, k, v, do, cud, True)
    # L = 1: p = 1 and ds = 0 up to the rounding of lse and delta; dv is the sum of the group's dout rows
    assert dq[0].float().abs().max() <= 1e-4 and dk[0].float().abs().max() <= 1e-4
    want = do[0].float().reshape(Hkv, Hq // Hkv, d).sum(dim=1)
    assert (dv[0].float() - want).abs().max() <= 2.0 ** -7 * want.abs().max()
    # deterministic
    dq2, dk2, dv2 = fwd_bwd(q, k, v, do, cud, True)
    assert torch.equal(dq, dq2) and torch.equal(dk, dk2) and torch.equal(dv, dv2)
    # sequence independence: a sequence run alone gives the same gradients, bit for bit
    a, b, c = fwd_bwd(q[150:400].contiguous(), k[150:400].contiguous(), v[150:400].contiguous(),
                      do[150:400].contiguous(), torch.tensor([0, 250], dtype=torch.int32, device=dev), True)
    assert torch.equal(a, dq[150:400]) and torch.equal(b, dk[150:400]) and torch.equal(c, dv[150:400])
    # GQA = explicit head repetition: same dq; key / value gradients of the copies add up
    kr, vr = k.repeat_interleave(2, dim=1).contiguous(), v.repeat_interleave(2, dim=1).contiguous()
    dqr, dkr, dvr = fwd_bwd(q, kr, vr, do, cud, True)
    assert torch.equal(dqr, dq)
    for full, rep in ((dk, dkr), (dv, dvr)):
        s = rep.float().reshape(400, Hkv, 2, d).sum(dim=2)
        assert (s - full.float()).abs().max() <= 1e-2 + 2.0 ** -6 * full.float().abs().max()
    # all value rows of a sequence equal: out does not depend on p there, so dq = dk = 0 up to rounding
    v2 = v.clone()
    v2[150:400] = v2[150]
    dq3, dk3, _ = fwd_bwd(q, k, v2, do, cud, True)
    assert dq3[150:400].float().abs().max() <= 2e-2 and dk3[150:400].float().abs().max() <= 2e-2


def pick_units(cu, Hkv, cap):
    """(sequence, kv-head) units the oracle can afford: the shortest, the longest below `cap`
    rows and one in between, on the first, a middle and the last kv-head."""
    lens = np.diff(cu)
    ok = np.nonzero((lens > 0) & (lens <= cap))[0]
    srt = ok[np.argsort(lens[ok], kind="stable")]
    seqs = [int(srt[0]), int(srt[len(srt) // 2]), int(srt[-1])]
    heads = [0, Hkv // 2, Hkv - 1]
    return list(zip(seqs, heads))


@pytest.mark.parametrize("cid", [2, 3, 4, 5])
def test_config_units_and_invariants(gpu_device, cid):
    """One instance's share at full shape (the most loaded instance): the oracle computes whole
    (sequence, kv-head) units; every sequence is checked through the invariants that hold at any
    size: key gradients of a sequence sum to zero, value gradients sum to the summed dout."""
    dev = gpu_device
    w = wl.WORKLOADS[cid]
    L = wl.draw_lengths(w)
    ref = oracle.balance(L, w.D, w.a, w.b)
    i = int(np.argmax(ref.loads))
    cu = np.ascontiguousarray(ref.cu_of(i))
    T = int(cu[-1])
    q, k, v, do = make(100 + cid, T, w.Hq, w.Hkv, w.d, dev)
    dq, dk, dv = fwd_bwd(q, k, v, do, torch.from_numpy(cu).to(dev), w.causal, fill=False)
    group = w.Hq // w.Hkv
    qb, kb, vb, db = bits(q), bits(k), bits(v), bits(do)
    for t, g in pick_units(cu, w.Hkv, 2600 if cid >= 4 else 4096):
        r0, r1 = int(cu[t]), int(cu[t + 1])
        wq, wk, wv = oracle.attn_bwd_unit(qb, kb, vb, db, r0, r1, g, w.causal, nthreads=NT)
        grad_check(dq[r0:r1, g * group: (g + 1) * group].float().cpu().numpy(), wq)
        grad_check(dk[r0:r1, g].float().cpu().numpy(), wk)
        grad_check(dv[r0:r1, g].float().cpu().numpy(), wv)
    # invariants over every sequence and kv-head, sums in fp64 on the device
    cud = torch.from_numpy(cu.astype(np.int64)).to(dev)
    seg = torch.repeat_interleave(torch.arange(len(cu) - 1, device=dev), cud[1:] - cud[:-1])
    nseq = len(cu) - 1
    dk_sum = torch.zeros((nseq, w.Hkv, w.d), dtype=torch.float64, device=dev).index_add_(0, seg, dk.double())
    dk_abs = torch.zeros((nseq, w.Hkv, w.d), dtype=torch.float64, device=dev).index_add_(0, seg, dk.double().abs())
    # each of the L summands carries a bf16 rounding of at most 2^-9 of its size
    assert bool((dk_sum.abs() <= 2.0 ** -8 * dk_abs + 1e-3).all())
    dv_sum = torch.zeros((nseq, w.Hkv, w.d), dtype=torch.float64, device=dev).index_add_(0, seg, dv.double())
    do_sum = torch.zeros((nseq, w.Hq, w.d), dtype=torch.float64, device=dev).index_add_(0, seg, do.double())
    do_sum = do_sum.reshape(nseq, w.Hkv, group, w.d).sum(dim=2)
    dv_abs = torch.zeros((nseq, w.Hkv, w.d), dtype=torch.float64, device=dev).index_add_(0, seg, dv.double().abs())
    assert bool(((dv_sum - do_sum).abs() <= 2.0 ** -7 * dv_abs + 1e-2).all())
    assert bool(torch.isfinite(dq.float()).all())
