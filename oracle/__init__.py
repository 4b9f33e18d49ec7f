"""Python face of the CPU oracle (plain C in this directory, built with gcc).

TEST INFRASTRUCTURE.  Only tests, ``__graft_entry__.smoke()`` and the bench's
``cpu_baseline`` leg may import this package.  It shares no code with the HIP
library, never imports it, and is never a fallback for it.

Functions mirror the dispatcher's problem statement (OrchMLLM Sec. 5.1:
inputs are the instance count and the list of sequence lengths, the output is
the list of new batches) and the attention definition; all arrays are numpy,
host memory.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "dispatch_oracle.c"), os.path.join(_HERE, "attention_oracle.c")]
_LIB_PATH = os.path.join(_HERE, "liborch_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64 arithmetic kept strict: no fast-math)."""
    stale = force or not os.path.exists(_LIB_PATH) or any(
        os.path.getmtime(s) > os.path.getmtime(_LIB_PATH) for s in _SRCS)
    if stale:
        tmp = _LIB_PATH + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-ffp-contract=off", "-o", tmp] + _SRCS + ["-lm"])
        os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        for name in ("orc_cost", "orc_sort_desc", "orc_greedy", "orc_balance", "orc_pack",
                     "orc_row_map", "orc_pack_composed", "orc_sort_asc", "orc_balance_padded", "orc_balance_tolerance", "orc_comm_volume", "orc_attn_fwd",
                     "orc_attn_rows", "orc_attn_bwd_unit"):
            getattr(_lib, name).restype = C.c_int
        _lib.orc_least_batches.restype = C.c_int64
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__("oracle status %d" % code)
        self.code = code


def _check(rc):
    if rc != 0:
        raise OracleError(rc)


def _i32(x):
    return np.ascontiguousarray(x, dtype=np.int32)


def cost(lengths, a: int, b: int) -> np.ndarray:
    L = _i32(lengths)
    out = np.empty(len(L), dtype=np.uint64)
    _check(lib().orc_cost(_p(L), C.c_int32(len(L)), C.c_uint64(a), C.c_uint64(b), _p(out)))
    return out


def sort_desc(cost_arr) -> np.ndarray:
    c = np.ascontiguousarray(cost_arr, dtype=np.uint64)
    out = np.empty(len(c), dtype=np.int32)
    _check(lib().orc_sort_desc(_p(c), C.c_int32(len(c)), _p(out)))
    return out


@dataclass
class Assignment:
    inst: np.ndarray        # int32[n]
    order: np.ndarray       # int32[n]
    seq_off: np.ndarray     # int32[D+1]
    tok_off: np.ndarray     # int64[D+1]
    cu_seqlens: np.ndarray  # int32[n+D]
    loads: np.ndarray       # uint64[D]

    def cu_of(self, i: int) -> np.ndarray:
        lo = int(self.seq_off[i]) + i
        return self.cu_seqlens[lo: lo + int(self.seq_off[i + 1] - self.seq_off[i]) + 1]

    def seqs_of(self, i: int) -> np.ndarray:
        return self.order[int(self.seq_off[i]): int(self.seq_off[i + 1])]


def balance(lengths, D: int, a: int, b: int) -> Assignment:
    L = _i32(lengths)
    n = len(L)
    if D < 1:
        raise OracleError(-1)
    out = Assignment(np.empty(n, np.int32), np.empty(n, np.int32), np.empty(D + 1, np.int32),
                     np.empty(D + 1, np.int64), np.empty(n + D, np.int32), np.empty(D, np.uint64))
    _check(lib().orc_balance(_p(L), C.c_int32(n), C.c_int32(D), C.c_uint64(a), C.c_uint64(b),
                             _p(out.inst), _p(out.order), _p(out.seq_off), _p(out.tok_off),
                             _p(out.cu_seqlens), _p(out.loads)))
    return out


def sort_asc(lengths) -> np.ndarray:
    L = _i32(lengths)
    out = np.empty(len(L), np.int32)
    _check(lib().orc_sort_asc(_p(L), C.c_int32(len(L)), _p(out)))
    return out


def least_batches(lengths, sorted_idx, bound: int):
    """The batch-counting helper of Algorithm 2 at a bound: (number of batches, batch of every sorted position)."""
    L, srt = _i32(lengths), _i32(sorted_idx)
    batch_of = np.empty(len(L), np.int32)
    cnt = lib().orc_least_batches(_p(L), _p(srt), C.c_int32(len(L)), C.c_uint64(bound), _p(batch_of))
    return int(cnt), batch_of


def balance_padded(lengths, D: int, a: int, b: int):
    """Algorithm 2 (Sec. 5.1, batching with paddings): returns (Assignment, bound).  The
    assignment's cu_seqlens are the padded slots j * max_i and tok_off the padded batch lengths."""
    L = _i32(lengths)
    n = len(L)
    if D < 1:
        raise OracleError(-1)
    out = Assignment(np.empty(n, np.int32), np.empty(n, np.int32), np.empty(D + 1, np.int32),
                     np.empty(D + 1, np.int64), np.empty(n + D, np.int32), np.empty(D, np.uint64))
    bound = C.c_uint64(0)
    _check(lib().orc_balance_padded(_p(L), C.c_int32(n), C.c_int32(D), C.c_uint64(a), C.c_uint64(b),
                                    _p(out.inst), _p(out.order), _p(out.seq_off), _p(out.tok_off),
                                    _p(out.cu_seqlens), _p(out.loads), C.byref(bound)))
    return out, int(bound.value)


def balance_tolerance(lengths, D: int, v: int, a: int, b: int) -> Assignment:
    """The appendix's third algorithm: longest-first greedy whose "lightest batch" is, among the
    batches within the tolerance interval v of the smallest length sum, the one with the
    smallest sum of squared lengths."""
    L = _i32(lengths)
    n = len(L)
    if D < 1:
        raise OracleError(-1)
    out = Assignment(np.empty(n, np.int32), np.empty(n, np.int32), np.empty(D + 1, np.int32),
                     np.empty(D + 1, np.int64), np.empty(n + D, np.int32), np.empty(D, np.uint64))
    _check(lib().orc_balance_tolerance(_p(L), C.c_int32(n), C.c_int32(D), C.c_uint64(v), C.c_uint64(a),
                                       C.c_uint64(b), _p(out.inst), _p(out.order), _p(out.seq_off),
                                       _p(out.tok_off), _p(out.cu_seqlens), _p(out.loads)))
    return out


def comm_volume(lengths, asg: Assignment, D_src: int, src_inst=None, node: int = 0):
    """V[from][to] in tokens (Sec. 5.2.2, the cost matrix of the node-wise rearrangement), and, for
    node > 0, per source instance the tokens sent to instances on other nodes of `node` instances."""
    L = _i32(lengths)
    D = len(asg.loads)
    V = np.empty((D_src, D), dtype=np.uint64)
    inter = np.zeros(D_src, dtype=np.uint64)
    f = None if src_inst is None else _i32(src_inst)
    _check(lib().orc_comm_volume(_p(L), C.c_int32(len(L)), C.c_int32(D_src), _p(f) if f is not None else None,
                                 C.c_int32(D), _p(asg.order), _p(asg.seq_off), _p(V), C.c_int32(node), _p(inter)))
    return V, inter


def pack(tokens: np.ndarray, lengths, asg: Assignment, inst_begin: int = 0, inst_end: int | None = None):
    """tokens: 2-D array [T, H] of any 2-byte dtype; returns the packed rows of
    instances [inst_begin, inst_end)."""
    L = _i32(lengths)
    D = len(asg.loads)
    if inst_end is None:
        inst_end = D
    tokens = np.ascontiguousarray(tokens)
    rows = int(asg.tok_off[inst_end] - asg.tok_off[inst_begin])
    out = np.empty((rows, tokens.shape[1]), dtype=tokens.dtype)
    rb = tokens.shape[1] * tokens.dtype.itemsize
    _check(lib().orc_pack(_p(tokens), _p(out), _p(L), C.c_int32(len(L)), C.c_int32(D), C.c_int64(rb),
                          _p(asg.order), _p(asg.seq_off), _p(asg.tok_off), _p(asg.cu_seqlens),
                          C.c_int32(inst_begin), C.c_int32(inst_end)))
    return out


def pack_composed(enc_rows: np.ndarray, packed: np.ndarray, sub_len, sub_off, enc_asg, llm_asg: Assignment,
                  inst_begin: int = 0, inst_end: int | None = None) -> np.ndarray:
    """Rearrangement composition (Sec. 5.3): rows in the encoder phase's packed order
    (`enc_asg`, or None for original example order) are placed inside the interleaved
    sequences of the LLM-phase assignment `llm_asg`, example s at row `sub_off[s]` of its
    sequence.  Writes into `packed` (rows of instances [inst_begin, inst_end)) in place and
    returns it; rows of other modalities are left as they are."""
    sl, so = _i32(sub_len), _i32(sub_off)
    Dm = len(llm_asg.loads)
    if inst_end is None:
        inst_end = Dm
    enc_rows = np.ascontiguousarray(enc_rows)
    assert packed.flags.c_contiguous and packed.dtype == enc_rows.dtype
    rb = enc_rows.shape[1] * enc_rows.dtype.itemsize
    if enc_asg is None:
        e = (0, None, None, None, None)
    else:
        e = (len(enc_asg.loads), _p(enc_asg.order), _p(enc_asg.seq_off), _p(enc_asg.tok_off), _p(enc_asg.cu_seqlens))
    _check(lib().orc_pack_composed(_p(enc_rows), _p(packed), _p(sl), _p(so), C.c_int32(len(sl)), C.c_int64(rb),
                                   C.c_int32(e[0]), e[1], e[2], e[3], e[4], C.c_int32(Dm), _p(llm_asg.order),
                                   _p(llm_asg.seq_off), _p(llm_asg.tok_off), _p(llm_asg.cu_seqlens),
                                   C.c_int32(inst_begin), C.c_int32(inst_end)))
    return packed


def pack_composed_pieces(enc_rows: np.ndarray, packed: np.ndarray, piece_ptr, piece_off, piece_len, enc_asg,
                         llm_asg: Assignment, inst_begin: int = 0, inst_end: int | None = None) -> np.ndarray:
    """Rearrangement composition with several sub-sequences per example (Sec. 6): example s's rows of
    this modality (one run in the encoder's packed order `enc_asg`, or in original order when None) are
    cut into the pieces piece_ptr[s] .. piece_ptr[s+1]-1; piece p goes to row piece_off[p] of the
    example's interleaved sequence.  Writes into `packed` in place and returns it."""
    pp, po, pl = _i32(piece_ptr), _i32(piece_off), _i32(piece_len)
    n = len(pp) - 1
    Dm = len(llm_asg.loads)
    if inst_end is None:
        inst_end = Dm
    enc_rows = np.ascontiguousarray(enc_rows)
    assert packed.flags.c_contiguous and packed.dtype == enc_rows.dtype
    rb = enc_rows.shape[1] * enc_rows.dtype.itemsize
    if enc_asg is None:
        e = (0, None, None, None, None)
    else:
        e = (len(enc_asg.loads), _p(enc_asg.order), _p(enc_asg.seq_off), _p(enc_asg.tok_off), _p(enc_asg.cu_seqlens))
    _check(lib().orc_pack_composed_pieces(_p(enc_rows), _p(packed), _p(pp), _p(po), _p(pl), C.c_int32(n),
                                          C.c_int64(rb), C.c_int32(e[0]), e[1], e[2], e[3], e[4], C.c_int32(Dm),
                                          _p(llm_asg.order), _p(llm_asg.seq_off), _p(llm_asg.tok_off),
                                          _p(llm_asg.cu_seqlens), C.c_int32(inst_begin), C.c_int32(inst_end)))
    return packed


def row_map(lengths, asg: Assignment) -> np.ndarray:
    L = _i32(lengths)
    D = len(asg.loads)
    out = np.empty(int(asg.tok_off[D]), dtype=np.int64)
    _check(lib().orc_row_map(_p(L), C.c_int32(len(L)), C.c_int32(D), _p(asg.order), _p(asg.seq_off),
                             _p(asg.tok_off), _p(asg.cu_seqlens), _p(out)))
    return out


def _u16(x):
    x = np.ascontiguousarray(x)
    assert x.dtype.itemsize == 2
    return x.view(np.uint16)


def attn_fwd(q, k, v, cu_seqlens, causal: bool, scale: float = 0.0, nthreads: int = 1,
             want_lse: bool = False):
    """q [T,Hq,d], k,v [T,Hkv,d] as bf16 bit patterns (any 2-byte dtype).
    Returns fp64 out [T,Hq,d] (and lse [Hq,T]); also the thread count used."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    cu = _i32(cu_seqlens)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    out = np.zeros((T, Hq, d), dtype=np.float64)
    lse = np.zeros((Hq, T), dtype=np.float64) if want_lse else None
    used = C.c_int(0)
    _check(lib().orc_attn_fwd(_p(q), _p(k), _p(v), _p(out), _p(lse), _p(cu), C.c_int32(len(cu) - 1),
                              C.c_int64(T), C.c_int32(Hq), C.c_int32(Hkv), C.c_int32(d), C.c_double(scale),
                              C.c_int(1 if causal else 0), C.c_int(nthreads), C.byref(used)))
    attn_fwd.last_threads = used.value
    return (out, lse) if want_lse else out


def attn_rows(q, k, v, cu_seqlens, causal: bool, seq, head, abs_row, scale: float = 0.0,
              nthreads: int = 1, want_lse: bool = False):
    """Selected output rows only: out fp64 [M, d] for (seq[m], head[m], abs_row[m])."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    cu = _i32(cu_seqlens)
    seq, head, abs_row = _i32(seq), _i32(head), _i32(abs_row)
    _, Hq, d = q.shape
    Hkv = k.shape[1]
    M = len(seq)
    out = np.zeros((M, d), dtype=np.float64)
    lse = np.zeros(M, dtype=np.float64) if want_lse else None
    _check(lib().orc_attn_rows(_p(q), _p(k), _p(v), _p(cu), C.c_int32(len(cu) - 1), C.c_int32(Hq),
                               C.c_int32(Hkv), C.c_int32(d), C.c_double(scale),
                               C.c_int(1 if causal else 0), _p(seq), _p(head), _p(abs_row),
                               C.c_int32(M), _p(out), _p(lse), C.c_int(nthreads)))
    return (out, lse) if want_lse else out


def attn_bwd_unit(q, k, v, dout, r0: int, r1: int, g: int, causal: bool, scale: float = 0.0, nthreads: int = 1):
    """Gradients of one (sequence rows [r0, r1), kv-head g) unit: dq fp64 [L, group, d] for the
    q-heads of g's group, dk and dv fp64 [L, d]."""
    q, k, v, dout = _u16(q), _u16(k), _u16(v), _u16(dout)
    _, Hq, d = q.shape
    Hkv = k.shape[1]
    L = r1 - r0
    dq = np.zeros((L, Hq // Hkv, d), dtype=np.float64)
    dk = np.zeros((L, d), dtype=np.float64)
    dv = np.zeros((L, d), dtype=np.float64)
    _check(lib().orc_attn_bwd_unit(_p(q), _p(k), _p(v), _p(dout), C.c_int64(r0), C.c_int64(r1), C.c_int32(g),
                                   C.c_int32(Hq), C.c_int32(Hkv), C.c_int32(d), C.c_double(scale),
                                   C.c_int(1 if causal else 0), _p(dq), _p(dk), _p(dv), C.c_int(nthreads)))
    return dq, dk, dv


def attn_bwd(q, k, v, dout, cu_seqlens, causal: bool, scale: float = 0.0, nthreads: int = 1):
    """Full backward: dq fp64 [T,Hq,d], dk, dv fp64 [T,Hkv,d] (rows outside every sequence stay 0)."""
    qa = _u16(q)
    T, Hq, d = qa.shape
    Hkv = _u16(k).shape[1]
    group = Hq // Hkv
    cu = _i32(cu_seqlens)
    dq = np.zeros((T, Hq, d)), np.zeros((T, Hkv, d)), np.zeros((T, Hkv, d))
    dq, dk, dv = dq
    for t in range(len(cu) - 1):
        r0, r1 = int(cu[t]), int(cu[t + 1])
        for g in range(Hkv):
            a, b, c = attn_bwd_unit(q, k, v, dout, r0, r1, g, causal, scale, nthreads)
            dq[r0:r1, g * group: (g + 1) * group] = a
            dk[r0:r1, g] = b
            dv[r0:r1, g] = c
    return dq, dk, dv


def load_ratio(lengths, inst, D: int, a: int, b: int) -> float:
    """max_i load / mean_i load of an arbitrary assignment, with Eq. 2's cost."""
    c = cost(lengths, a, b).astype(np.float64)
    loads = np.zeros(D)
    np.add.at(loads, np.asarray(inst), c)
    return float(loads.max() / loads.mean()) if loads.mean() > 0 else 1.0
