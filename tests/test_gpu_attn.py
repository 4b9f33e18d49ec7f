"""HIP orch_varlen_attn_fwd vs the fp64 CPU oracle (max-abs <= 2e-2, mean-abs <= 2e-3)."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2503_23830_amd as orch
import workloads as wl
from gpu_common import attn_tolerance_check, bits

pytestmark = pytest.mark.gpu
NT = min(16, os.cpu_count() or 1)


def make_qkv(seed, T, Hq, Hkv, d, dev):
    return (wl.normal_bf16_torch((T, Hq, d), seed, 1, dev), wl.normal_bf16_torch((T, Hkv, d), seed, 2, dev),
            wl.normal_bf16_torch((T, Hkv, d), seed, 3, dev))


def run_full(cu, Hq, Hkv, d, causal, dev, seed=1, scale=0.0, with_lse=True, total=None):
    cu = np.ascontiguousarray(cu, dtype=np.int32)
    T = int(cu[-1]) if total is None else total
    q, k, v = make_qkv(seed, T, Hq, Hkv, d, dev)
    lse = torch.full((Hq, T), float("nan"), dtype=torch.float32, device=dev) if with_lse else None
    out = torch.full((T, Hq, d), float("nan"), dtype=torch.bfloat16, device=dev)
    orch.varlen_attn_fwd(q, k, v, torch.from_numpy(cu).to(dev), causal, scale=scale, out=out, lse=lse)
    torch.cuda.synchronize()
    want, wlse = oracle.attn_fwd(bits(q), bits(k), bits(v), cu, causal, scale=scale, nthreads=NT, want_lse=True)
    got = out.float().cpu().numpy()
    rows = np.zeros(T, dtype=bool)
    for t in range(len(cu) - 1):
        rows[cu[t]: cu[t + 1]] = True
    stats = attn_tolerance_check(got[rows], want[rows])
    # rows outside every sequence are never written
    assert np.isnan(got[~rows]).all()
    if with_lse:
        gl = lse.cpu().numpy()
        assert np.max(np.abs(gl[:, rows] - wlse[:, rows])) <= 1e-3
    return stats


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("Hq,Hkv,d", [(4, 4, 64), (4, 1, 128), (8, 8, 128), (6, 2, 64)])
def test_small_ragged(gpu_device, causal, Hq, Hkv, d):
    # several q tiles and k tiles, ragged tails, empty and length-1 sequences
    L = [1, 0, 37, 128, 129, 64, 63, 65, 300, 0, 2, 513]
    cu = np.concatenate([[0], np.cumsum(L)])
    run_full(cu, Hq, Hkv, d, causal, gpu_device)


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (4, 2)])
def test_head_dim_128_ring_boundaries(gpu_device, causal, Hq, Hkv):
    """Lengths around every boundary of the head_dim-128 kernel: 32-key blocks, 64-key tiles, the
    four-stage K/V rings (1 to 17 tiles per sequence) and 256-row query tiles; Hkv = 8 takes the
    per-XCD head mapping, Hkv = 2 the plain one."""
    L = [1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 320, 511, 512, 767, 1025]
    cu = np.concatenate([[0], np.cumsum(L)])
    run_full(cu, Hq, Hkv, 128, causal, gpu_device, seed=7)


def test_c1_all_instances(gpu_device):
    w = wl.WORKLOADS[1]
    L = wl.draw_lengths(w)
    ref = oracle.balance(L, w.D, w.a, w.b)
    for i in range(w.D):
        run_full(ref.cu_of(i), w.Hq, w.Hkv, w.d, w.causal, gpu_device, seed=10 + i)


def test_explicit_scale_and_padding_rows(gpu_device):
    cu = np.array([0, 200, 200, 431], dtype=np.int32)
    run_full(cu, 4, 2, 128, True, gpu_device, scale=0.05, total=500)
    run_full(cu, 4, 2, 64, False, gpu_device, scale=0.2, total=500)


def test_closed_forms_on_device(gpu_device):
    dev = gpu_device
    Hq, Hkv, d = 4, 2, 128
    cu = np.array([0, 1, 150, 400], dtype=np.int32)
    q, k, v = make_qkv(5, 400, Hq, Hkv, d, dev)
    cud = torch.from_numpy(cu).to(dev)
    out = orch.varlen_attn_fwd(q, k, v, cud, True)
    torch.cuda.synchronize()
    # L = 1: out = v exactly (bit-exact through the bf16 round trip)
    for h in range(Hq):
        assert torch.equal(out[0, h], v[0, h // 2])
    # all V rows of a sequence equal -> out is that row (p sums to 1 up to rounding)
    v2 = v.clone()
    v2[150:400] = v2[150]
    out2 = orch.varlen_attn_fwd(q, k, v2, cud, True)
    torch.cuda.synchronize()
    ref = v2[150].float()[None].repeat_interleave(2, dim=1)
    assert (out2[150:400].float() - ref).abs().max() <= 2e-2
    # sequence independence: a sequence run alone gives the same rows, bit for bit
    alone = orch.varlen_attn_fwd(q[150:400].contiguous(), k[150:400].contiguous(), v[150:400].contiguous(),
                                 torch.tensor([0, 250], dtype=torch.int32, device=dev), True)
    torch.cuda.synchronize()
    assert torch.equal(alone, out[150:400])
    # GQA = explicit head repetition
    rep = orch.varlen_attn_fwd(q, k.repeat_interleave(2, dim=1).contiguous(),
                               v.repeat_interleave(2, dim=1).contiguous(), cud, True)
    torch.cuda.synchronize()
    assert torch.equal(rep, out)
    # deterministic
    again = orch.varlen_attn_fwd(q, k, v, cud, True)
    torch.cuda.synchronize()
    assert torch.equal(again, out)


def sample_triples(cu, Hq, group, count, seed):
    """(sequence, head, row) samples: first/last rows, rows around tile edges,
    the longest and shortest non-empty sequences, each kv group's first and last
    q-head, plus seeded random triples."""
    lens = np.diff(cu)
    nz = np.nonzero(lens)[0]
    longest, shortest = nz[np.argmax(lens[nz])], nz[np.argmin(lens[nz])]
    trip = []
    heads_edge = sorted({0, group - 1, Hq - group, Hq - 1})
    for t in (longest, shortest, nz[0], nz[-1]):
        Lt = int(lens[t])
        rows = {0, Lt - 1}
        for e in (16, 32, 64, 128, 256, 1024):
            for dlt in (-1, 0, 1):
                if 0 <= e + dlt < Lt:
                    rows.add(e + dlt)
                if 0 <= Lt - e + dlt < Lt:
                    rows.add(Lt - e + dlt)
        for r in sorted(rows):
            for h in heads_edge:
                trip.append((t, h, int(cu[t]) + r))
    u = wl.uniform01(seed, 9, 3 * count).reshape(3, count)
    for j in range(count):
        t = nz[int(u[0, j] * len(nz))]
        trip.append((int(t), int(u[1, j] * Hq), int(cu[t]) + int(u[2, j] * lens[t])))
    a = np.array(trip, dtype=np.int32)
    return a[:, 0], a[:, 1], a[:, 2]


@pytest.mark.parametrize("cid", [2, 3, 4, 5])
def test_config_row_sampled(gpu_device, cid):
    """One instance's share at full shape (the most loaded instance after
    balancing); the fp64 oracle computes sampled rows one by one."""
    w = wl.WORKLOADS[cid]
    L = wl.draw_lengths(w)
    ref = oracle.balance(L, w.D, w.a, w.b)
    i = int(np.argmax(ref.loads))
    cu = np.ascontiguousarray(ref.cu_of(i))
    T = int(cu[-1])
    dev = gpu_device
    q, k, v = make_qkv(100 + cid, T, w.Hq, w.Hkv, w.d, dev)
    lse = torch.full((w.Hq, T), float("nan"), dtype=torch.float32, device=dev)
    status = torch.full((1,), 77, dtype=torch.int32, device=dev)
    out = orch.varlen_attn_fwd(q, k, v, torch.from_numpy(cu).to(dev), w.causal, lse=lse,
                               max_seqlen=int(np.diff(cu).max()), dev_status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    count = 4096 if cid < 5 else 1024
    seq, head, row = sample_triples(cu, w.Hq, w.Hq // w.Hkv, count, cid)
    want, wlse = oracle.attn_rows(bits(q), bits(k), bits(v), cu, w.causal, seq, head, row, nthreads=NT,
                                  want_lse=True)
    rt = torch.from_numpy(row.astype(np.int64)).to(dev)
    ht = torch.from_numpy(head.astype(np.int64)).to(dev)
    got = out[rt, ht].float().cpu().numpy()
    attn_tolerance_check(got, want)
    assert np.max(np.abs(lse[ht, rt].cpu().numpy().astype(np.float64) - wlse)) <= 1e-3
    assert torch.isfinite(out.float()).all()
    assert torch.isfinite(lse).all()   # every row of the instance belongs to a sequence


@pytest.mark.parametrize("d", [64, 128])
def test_invalid_cu_seqlens_is_reported_and_writes_nothing(gpu_device, d):
    """Data errors only the device can see: dev_status = ORCH_EDATA and out / lse untouched."""
    dev = gpu_device
    Hq, Hkv, T = 4, 2, 600
    q, k, v = make_qkv(3, T, Hq, Hkv, d, dev)
    good = np.array([0, 100, 100, 600], dtype=np.int32)
    cases = {
        "decreasing": (np.array([0, 300, 200, 600], dtype=np.int32), 0),
        "beyond total_tokens": (np.array([0, 100, 300, 601], dtype=np.int32), 0),
        "negative": (np.array([-1, 100, 300, 600], dtype=np.int32), 0),
        "longer than max_seqlen": (good, 499),
    }
    for name, (cu, max_seqlen) in cases.items():
        out = torch.full((T, Hq, d), float("nan"), dtype=torch.bfloat16, device=dev)
        lse = torch.full((Hq, T), float("nan"), dtype=torch.float32, device=dev)
        status = torch.zeros(1, dtype=torch.int32, device=dev)
        orch.varlen_attn_fwd(q, k, v, torch.from_numpy(cu).to(dev), True, out=out, lse=lse,
                             max_seqlen=max_seqlen, dev_status=status)
        torch.cuda.synchronize()
        assert int(status.item()) == -5, name
        assert torch.isnan(out.float()).all() and torch.isnan(lse).all(), name
        dq, dk, dv = (torch.full_like(t, float("nan")) for t in (q, k, v))
        status.zero_()
        orch.varlen_attn_bwd(q, k, v, q, torch.zeros((Hq, T), dtype=torch.float32, device=dev), q,
                             torch.from_numpy(cu).to(dev), True, max_seqlen=max_seqlen, dq=dq, dk=dk, dv=dv,
                             dev_status=status)
        torch.cuda.synchronize()
        assert int(status.item()) == -5, name
        assert all(torch.isnan(t.float()).all() for t in (dq, dk, dv)), name
    # a valid call with the exact bound: status OK, same result as without the bound
    status = torch.full((1,), 77, dtype=torch.int32, device=dev)
    a = orch.varlen_attn_fwd(q, k, v, torch.from_numpy(good).to(dev), True, max_seqlen=500, dev_status=status)
    b = orch.varlen_attn_fwd(q, k, v, torch.from_numpy(good).to(dev), True)
    torch.cuda.synchronize()
    assert int(status.item()) == 0 and torch.equal(a, b)


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("d", [64, 128])
def test_reference_far_above_the_first_block(gpu_device, causal, d):
    """The kernels take every probability against the row maximum of the FIRST 32-key block.
    Here later keys score hundreds of units above it (the exponentials would overflow), so the
    marked tiles must come from the moving-reference pass; other sequences of the same call
    (ordinary data) keep the fast pass.  Both against the fp64 oracle."""
    dev = gpu_device
    Hq, Hkv = 4, 2
    L = [300, 700, 40, 513]
    cu = np.concatenate([[0], np.cumsum(L)]).astype(np.int32)
    T = int(cu[-1])
    q, k, v = make_qkv(21, T, Hq, Hkv, d, dev)
    # sequence 1 (rows 300..999): queries all +4, keys 0..31 all -4, keys from 320 on all +4 scaled up
    q[300:1000] = 4.0
    k[300:332] = -4.0
    k[620:1000] = 4.0 + 0.25 * k[620:1000].sign()
    # sequence 3: one huge late key for half of the heads only
    k[1040 + 400, 0] = 24.0 * q[1040 + 400, 0].sign()
    lse = torch.full((Hq, T), float("nan"), dtype=torch.float32, device=dev)
    out = torch.full((T, Hq, d), float("nan"), dtype=torch.bfloat16, device=dev)
    orch.varlen_attn_fwd(q, k, v, torch.from_numpy(cu).to(dev), causal, out=out, lse=lse)
    torch.cuda.synchronize()
    want, wlse = oracle.attn_fwd(bits(q), bits(k), bits(v), cu, causal, nthreads=NT, want_lse=True)
    attn_tolerance_check(out.float().cpu().numpy(), want)
    gl, wl_ = lse.cpu().numpy().astype(np.float64), wlse
    assert np.max(np.abs(gl - wl_) / np.maximum(1.0, np.abs(wl_))) <= 1e-3
