"""Pins for the attention oracle: closed forms, invariances and an independent
library routine (torch's fp64 scaled_dot_product_attention on the CPU)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl


def bf16_bits(x: torch.Tensor) -> np.ndarray:
    return x.to(torch.bfloat16).contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_f64(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def make_qkv(seed, T, Hq, Hkv, d):
    q = wl.normal_bf16_torch((T, Hq, d), seed, 1, "cpu")
    k = wl.normal_bf16_torch((T, Hkv, d), seed, 2, "cpu")
    v = wl.normal_bf16_torch((T, Hkv, d), seed, 3, "cpu")
    return q, k, v


def sdpa_reference(q, k, v, cu, causal, scale=None):
    """Per sequence: torch SDPA in fp64 with heads repeated for GQA."""
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    out = torch.zeros(T, Hq, d, dtype=torch.float64)
    for t in range(len(cu) - 1):
        lo, hi = int(cu[t]), int(cu[t + 1])
        if hi == lo:
            continue
        qq = q[lo:hi].double().permute(1, 0, 2)[None]
        kk = k[lo:hi].double().repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)[None]
        vv = v[lo:hi].double().repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)[None]
        o = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv, is_causal=causal, scale=scale)
        out[lo:hi] = o[0].permute(1, 0, 2)
    return out.numpy()


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Hq,Hkv,d", [(4, 4, 64), (8, 2, 128), (3, 1, 16)])
def test_against_library_sdpa(causal, Hq, Hkv, d):
    cu = np.array([0, 1, 1, 38, 40, 97], dtype=np.int32)  # L = 1, 0, 37, 2, 57
    q, k, v = make_qkv(7, int(cu[-1]), Hq, Hkv, d)
    got, lse = oracle.attn_fwd(bf16_bits(q), bf16_bits(k), bf16_bits(v), cu, causal, want_lse=True,
                               nthreads=2)
    want = sdpa_reference(q, k, v, cu, causal)
    assert np.max(np.abs(got - want)) < 1e-12
    # lse against scipy's logsumexp on explicitly formed scores
    from scipy.special import logsumexp
    lo, hi = 1, 38
    h = Hq - 1
    g = h // (Hq // Hkv)
    S = (q[lo:hi, h].double() @ k[lo:hi, g].double().T).numpy() / np.sqrt(d)
    if causal:
        S = np.where(np.tril(np.ones_like(S)) > 0, S, -np.inf)
    assert np.max(np.abs(lse[h, lo:hi] - logsumexp(S, axis=1))) < 1e-12
    # explicit scale argument
    got2 = oracle.attn_fwd(bf16_bits(q), bf16_bits(k), bf16_bits(v), cu, causal, scale=0.37)
    assert np.max(np.abs(got2 - sdpa_reference(q, k, v, cu, causal, scale=0.37))) < 1e-12


def test_closed_forms():
    Hq, Hkv, d = 4, 2, 32
    cu = np.array([0, 1, 20, 20, 45], dtype=np.int32)
    T = 45
    q, k, v = make_qkv(3, T, Hq, Hkv, d)
    qb, kb, vb = bf16_bits(q), bf16_bits(k), bf16_bits(v)
    vf = bits_to_f64(vb)
    # L = 1: out = v exactly
    out = oracle.attn_fwd(qb, kb, vb, cu, True)
    for h in range(Hq):
        assert np.array_equal(out[0, h], vf[0, h // 2])
    # all K rows of a sequence equal -> uniform weights
    k2 = k.clone()
    k2[1:20] = k2[1]
    k2[20:45] = k2[20]
    k2b = bf16_bits(k2)
    ob = oracle.attn_fwd(qb, k2b, vb, cu, False)
    oc = oracle.attn_fwd(qb, k2b, vb, cu, True)
    for h in range(Hq):
        g = h // 2
        assert np.allclose(ob[1:20, h], vf[1:20, g].mean(axis=0)[None], atol=1e-13)
        assert np.allclose(ob[20:45, h], vf[20:45, g].mean(axis=0)[None], atol=1e-13)
        pref = np.cumsum(vf[20:45, g], axis=0) / np.arange(1, 26)[:, None]
        assert np.allclose(oc[20:45, h], pref, atol=1e-13)
    # all V rows equal -> out is that row
    v2 = v.clone()
    v2[20:45] = v2[20]
    o = oracle.attn_fwd(qb, kb, bf16_bits(v2), cu, True)
    for h in range(Hq):
        assert np.allclose(o[20:45, h], bits_to_f64(bf16_bits(v2))[20, h // 2][None], atol=1e-13)


def test_invariances():
    Hq, Hkv, d = 4, 2, 32
    cu = np.array([0, 9, 40, 64], dtype=np.int32)
    q, k, v = make_qkv(11, 64, Hq, Hkv, d)
    qb, kb, vb = bf16_bits(q), bf16_bits(k), bf16_bits(v)
    base_b = oracle.attn_fwd(qb, kb, vb, cu, False)
    base_c = oracle.attn_fwd(qb, kb, vb, cu, True)
    # bidirectional: permuting (k, v) rows inside a sequence changes nothing
    perm = np.arange(64)
    perm[9:40] = 9 + np.array(wl.bits64(5, 1, 31).argsort())
    o = oracle.attn_fwd(qb, kb[perm], vb[perm], cu, False)
    assert np.max(np.abs(o - base_b)) < 1e-13
    # sequence independence (the paper's consequence-invariance, Sec. 3.3)
    alone = oracle.attn_fwd(qb[9:40], kb[9:40], vb[9:40], np.array([0, 31], np.int32), True)
    assert np.array_equal(alone, base_c[9:40])
    # GQA = explicit head repetition
    rep = oracle.attn_fwd(qb, np.repeat(kb, 2, axis=1), np.repeat(vb, 2, axis=1), cu, True)
    assert np.array_equal(rep, base_c)
    # causal row i only sees rows <= i: changing later k/v leaves it untouched
    k3, v3 = kb.copy(), vb.copy()
    k3[30:40] = kb[0:10]
    v3[30:40] = vb[0:10]
    o3 = oracle.attn_fwd(qb, k3, v3, cu, True)
    assert np.array_equal(o3[9:30], base_c[9:30]) and not np.array_equal(o3[30:40], base_c[30:40])
    # last causal row = last bidirectional row
    assert np.allclose(base_c[39], base_b[39], atol=1e-13)
    # sampled rows = rows of the full run
    seq = np.array([0, 1, 1, 2, 2], np.int32)
    head = np.array([0, 3, 1, 2, 0], np.int32)
    row = np.array([8, 9, 39, 40, 63], np.int32)
    r, l = oracle.attn_rows(qb, kb, vb, cu, True, seq, head, row, want_lse=True, nthreads=2)
    full, lse = oracle.attn_fwd(qb, kb, vb, cu, True, want_lse=True)
    for m in range(5):
        assert np.array_equal(r[m], full[row[m], head[m]])
        assert l[m] == lse[head[m], row[m]]


def test_threads_do_not_change_results():
    cu = np.array([0, 33, 64], dtype=np.int32)
    q, k, v = make_qkv(2, 64, 2, 2, 16)
    a = oracle.attn_fwd(bf16_bits(q), bf16_bits(k), bf16_bits(v), cu, True, nthreads=1)
    b = oracle.attn_fwd(bf16_bits(q), bf16_bits(k), bf16_bits(v), cu, True, nthreads=4)
    assert np.array_equal(a, b)
