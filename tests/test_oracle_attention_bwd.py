"""Pins for the attention-backward oracle: torch's fp64 autograd through its own
scaled_dot_product_attention (independent library routine), invariants of the softmax Jacobian
and closed forms."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from test_oracle_attention import bf16_bits, make_qkv


def autograd_reference(q, k, v, dout, cu, causal, scale=None):
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    qd = q.double().clone().requires_grad_(True)
    kd = k.double().clone().requires_grad_(True)
    vd = v.double().clone().requires_grad_(True)
    loss = 0.0
    for t in range(len(cu) - 1):
        lo, hi = int(cu[t]), int(cu[t + 1])
        if hi == lo:
            continue
        qq = qd[lo:hi].permute(1, 0, 2)[None]
        kk = kd[lo:hi].repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)[None]
        vv = vd[lo:hi].repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)[None]
        o = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv, is_causal=causal, scale=scale)
        loss = loss + (o[0].permute(1, 0, 2) * dout[lo:hi].double()).sum()
    loss.backward()
    return qd.grad.numpy(), kd.grad.numpy(), vd.grad.numpy()


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Hq,Hkv,d", [(4, 4, 64), (8, 2, 128), (3, 1, 16)])
def test_against_library_autograd(causal, Hq, Hkv, d):
    cu = np.array([0, 1, 1, 38, 40, 97], dtype=np.int32)  # L = 1, 0, 37, 2, 57
    T = int(cu[-1]) + 3  # trailing rows outside every sequence
    q, k, v = make_qkv(11, T, Hq, Hkv, d)
    dout = wl.normal_bf16_torch((T, Hq, d), 11, 4, "cpu")
    dq, dk, dv = oracle.attn_bwd(bf16_bits(q), bf16_bits(k), bf16_bits(v), bf16_bits(dout), cu, causal, nthreads=3)
    wq, wk, wv = autograd_reference(q, k, v, dout, cu, causal)
    for got, want in ((dq, wq), (dk, wk), (dv, wv)):
        assert np.max(np.abs(got - want)) < 1e-11
    # explicit scale
    dq2, dk2, dv2 = oracle.attn_bwd(bf16_bits(q), bf16_bits(k), bf16_bits(v), bf16_bits(dout), cu, causal, scale=0.07)
    wq, wk, wv = autograd_reference(q, k, v, dout, cu, causal, scale=0.07)
    for got, want in ((dq2, wq), (dk2, wk), (dv2, wv)):
        assert np.max(np.abs(got - want)) < 1e-11


def test_invariants_and_closed_forms():
    Hq, Hkv, d = 6, 2, 32
    cu = np.array([0, 50, 51, 120], dtype=np.int32)
    T = 120
    q, k, v = make_qkv(12, T, Hq, Hkv, d)
    dout = wl.normal_bf16_torch((T, Hq, d), 12, 4, "cpu")
    qb, kb, vb, db = bf16_bits(q), bf16_bits(k), bf16_bits(v), bf16_bits(dout)
    for causal in (False, True):
        dq, dk, dv = oracle.attn_bwd(qb, kb, vb, db, cu, causal, nthreads=2)
        for t in range(3):
            lo, hi = int(cu[t]), int(cu[t + 1])
            # rows of ds sum to zero: the key gradients of a sequence sum to zero ...
            assert np.max(np.abs(dk[lo:hi].sum(axis=0))) < 1e-10
            # ... and rows of p sum to one: the value gradients sum to the summed dout of the group
            want = dout[lo:hi].double().numpy().reshape(hi - lo, Hkv, Hq // Hkv, d).sum(axis=(0, 2))
            assert np.max(np.abs(dv[lo:hi].sum(axis=0) - want)) < 1e-10
        # L = 1: p = 1, ds = 0
        assert not dq[50].any() and not dk[50].any()
        assert np.max(np.abs(dv[50] - dout[50].double().numpy().reshape(Hkv, Hq // Hkv, d).sum(axis=1))) < 1e-12
        # thread-count independence (up to fp64 summation order)
        dq1, dk1, dv1 = oracle.attn_bwd(qb, kb, vb, db, cu, causal, nthreads=1)
        assert np.max(np.abs(dq1 - dq)) < 1e-12 and np.max(np.abs(dk1 - dk)) < 1e-12 and np.max(np.abs(dv1 - dv)) < 1e-12
    # all key rows of a sequence equal: the scores do not depend on j, so dq = 0 there
    k2 = k.clone()
    k2[51:120] = k2[51]
    dq, _, _ = oracle.attn_bwd(qb, bf16_bits(k2), vb, db, cu, False)
    assert np.max(np.abs(dq[51:120])) < 1e-12
    # all value rows equal: out does not depend on p, so dq = dk = 0 there
    v2 = v.clone()
    v2[51:120] = v2[51]
    dq, dk, _ = oracle.attn_bwd(qb, kb, bf16_bits(v2), db, cu, True)
    assert np.max(np.abs(dq[51:120])) < 1e-12 and np.max(np.abs(dk[51:120])) < 1e-12
    # sequence independence: a sequence run alone gives the same gradients
    dqa, dka, dva = oracle.attn_bwd(qb, kb, vb, db, cu, True)
    dqs, dks, dvs = oracle.attn_bwd(qb[51:120], kb[51:120], vb[51:120], db[51:120], np.array([0, 69], np.int32), True)
    assert np.array_equal(dqs, dqa[51:120]) and np.array_equal(dks, dka[51:120]) and np.array_equal(dvs, dva[51:120])
    # GQA = explicit head repetition followed by summing the repeated heads' key/value gradients
    kr = k.repeat_interleave(Hq // Hkv, dim=1)
    vr = v.repeat_interleave(Hq // Hkv, dim=1)
    dqr, dkr, dvr = oracle.attn_bwd(qb, bf16_bits(kr), bf16_bits(vr), db, cu, True)
    assert np.max(np.abs(dqr - dqa)) < 1e-12
    assert np.max(np.abs(dkr.reshape(T, Hkv, Hq // Hkv, d).sum(axis=2) - dka)) < 1e-11
    assert np.max(np.abs(dvr.reshape(T, Hkv, Hq // Hkv, d).sum(axis=2) - dva)) < 1e-11
