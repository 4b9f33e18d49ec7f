"""Thin ctypes binding over liborch.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels.  torch supplies
device memory (``torch.empty``), raw pointers (``data_ptr()``) and the current
HIP stream; nothing here computes.  There is no CPU fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "liborch.so")
_lib = None

EXPORTS = ("orch_balance_workspace", "orch_balance", "orch_pack_workspace", "orch_pack",
           "orch_balance_padded", "orch_balance_tolerance", "orch_balance_static", "orch_balance_static_max_n", "orch_balance_stages",
           "orch_pack_composed_workspace", "orch_pack_composed", "orch_comm_volume",
           "orch_pack_composed_pieces_workspace", "orch_pack_composed_pieces",
           "orch_varlen_attn_workspace", "orch_varlen_attn_fwd", "orch_varlen_attn_bwd_workspace",
           "orch_varlen_attn_bwd", "orch_last_error",
           "orch_attn_variant")


class OrchError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("liborch status %d: %s" % (code, msg))
        self.code = code


class _Phase(C.Structure):
    _fields_ = [("a", C.c_uint64), ("b", C.c_uint64)]


class _Assignment(C.Structure):
    _fields_ = [("inst", C.c_void_p), ("order", C.c_void_p), ("seq_off", C.c_void_p),
                ("tok_off", C.c_void_p), ("cu_seqlens", C.c_void_p), ("loads", C.c_void_p),
                ("dev_status", C.c_void_p)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """dlopen liborch.so (built in-tree by build.py); raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise OrchError(-4, "liborch.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(_LIB_PATH)
    lib.orch_balance_workspace.restype = C.c_size_t
    lib.orch_balance_workspace.argtypes = [C.c_int32, C.c_int32]
    lib.orch_pack_workspace.restype = C.c_size_t
    lib.orch_pack_workspace.argtypes = [C.c_int32, C.c_int32]
    lib.orch_varlen_attn_workspace.restype = C.c_size_t
    lib.orch_varlen_attn_workspace.argtypes = [C.c_int32, C.c_int32, C.c_int32]
    lib.orch_balance.restype = C.c_int
    lib.orch_balance.argtypes = [C.c_void_p, C.c_int32, C.c_int32, _Phase, _Assignment, C.c_void_p,
                                 C.c_size_t, C.c_void_p]
    lib.orch_balance_stages.restype = C.c_int
    lib.orch_balance_stages.argtypes = [C.c_void_p, C.c_int32, C.c_int32, _Phase, _Assignment, C.c_void_p,
                                        C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]
    lib.orch_balance_static.restype = C.c_int
    lib.orch_balance_static.argtypes = [C.c_void_p, C.c_int32, C.c_int32, _Phase, _Assignment, C.c_void_p]
    lib.orch_balance_static_max_n.restype = C.c_int32
    lib.orch_balance_static_max_n.argtypes = []
    lib.orch_balance_padded.restype = C.c_int
    lib.orch_balance_padded.argtypes = [C.c_void_p, C.c_int32, C.c_int32, _Phase, _Assignment, C.c_void_p,
                                        C.c_void_p, C.c_size_t, C.c_void_p]
    lib.orch_balance_tolerance.restype = C.c_int
    lib.orch_balance_tolerance.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_uint64, _Phase, _Assignment,
                                           C.c_void_p, C.c_size_t, C.c_void_p]
    lib.orch_pack.restype = C.c_int
    lib.orch_pack.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int64,
                              C.c_int32, C.c_int64, _Assignment, C.c_int32, C.c_int32, C.c_void_p,
                              C.c_size_t, C.c_void_p]
    lib.orch_pack_composed_workspace.restype = C.c_size_t
    lib.orch_pack_composed_workspace.argtypes = [C.c_int32]
    lib.orch_pack_composed.restype = C.c_int
    lib.orch_pack_composed.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                       C.POINTER(_Assignment), C.c_int32, _Assignment, C.c_int64, C.c_int32,
                                       C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.orch_pack_composed_pieces_workspace.restype = C.c_size_t
    lib.orch_pack_composed_pieces_workspace.argtypes = [C.c_int32, C.c_int32]
    lib.orch_pack_composed_pieces.restype = C.c_int
    lib.orch_pack_composed_pieces.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                              C.c_int32, C.c_int32, C.POINTER(_Assignment), C.c_int32, _Assignment,
                                              C.c_int64, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_void_p,
                                              C.c_size_t, C.c_void_p]
    lib.orch_comm_volume.restype = C.c_int
    lib.orch_comm_volume.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, _Assignment,
                                     C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.orch_varlen_attn_fwd.restype = C.c_int
    lib.orch_varlen_attn_fwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                         C.c_int32, C.c_int32, C.c_float, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_size_t, C.c_void_p]
    lib.orch_varlen_attn_bwd_workspace.restype = C.c_size_t
    lib.orch_varlen_attn_bwd_workspace.argtypes = [C.c_int32, C.c_int32, C.c_int32]
    lib.orch_varlen_attn_bwd.restype = C.c_int
    lib.orch_varlen_attn_bwd.argtypes = [C.c_void_p] * 10 + [C.c_int32] * 6 + [C.c_float, C.c_int32, C.c_void_p,
                                                                                C.c_void_p, C.c_size_t, C.c_void_p]
    lib.orch_last_error.restype = C.c_char_p
    lib.orch_attn_variant.restype = C.c_char_p
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise OrchError(rc, load_library().orch_last_error().decode())


def _stream(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


@dataclass
class Assignment:
    """Device tensors written by balance (see orch_assignment in include/orch.h)."""
    inst: torch.Tensor
    order: torch.Tensor
    seq_off: torch.Tensor
    tok_off: torch.Tensor
    cu_seqlens: torch.Tensor
    loads: torch.Tensor       # int64 storage holding u64 values
    dev_status: torch.Tensor
    n: int
    D: int

    def _c(self) -> _Assignment:
        return _Assignment(self.inst.data_ptr(), self.order.data_ptr(), self.seq_off.data_ptr(),
                           self.tok_off.data_ptr(), self.cu_seqlens.data_ptr(), self.loads.data_ptr(),
                           self.dev_status.data_ptr())

    @staticmethod
    def empty(n: int, D: int, device) -> "Assignment":
        e = lambda m, dt: torch.empty(max(m, 1), dtype=dt, device=device)
        return Assignment(e(n, torch.int32), e(n, torch.int32), e(D + 1, torch.int32),
                          e(D + 1, torch.int64), e(n + D, torch.int32), e(D, torch.int64),
                          torch.zeros(1, dtype=torch.int32, device=device), n, D)


def balance_workspace(n: int, D: int) -> int:
    return load_library().orch_balance_workspace(n, D)


def pack_workspace(n: int, D: int) -> int:
    return load_library().orch_pack_workspace(n, D)


def pack_composed_workspace(n: int) -> int:
    return load_library().orch_pack_composed_workspace(n)


def varlen_attn_workspace(batch: int, total_tokens: int, Hq: int) -> int:
    return load_library().orch_varlen_attn_workspace(batch, total_tokens, Hq)


def balance(lengths: torch.Tensor, D: int, a: int, b: int, out: Assignment | None = None,
            ws: torch.Tensor | None = None) -> Assignment:
    """orch_balance: lengths int32[n] on the GPU -> Assignment (Sec. 5.1, Alg. 1)."""
    lib = load_library()
    assert lengths.dtype == torch.int32 and lengths.is_cuda and lengths.is_contiguous()
    n = lengths.numel()
    dev = lengths.device
    if out is None:
        out = Assignment.empty(n, D, dev)
    if ws is None:
        ws = _workspace(lib.orch_balance_workspace(n, max(D, 1)), dev)
    _check(lib.orch_balance(_ptr(lengths), n, D, _Phase(a, b), out._c(), _ptr(ws), ws.numel(),
                            C.c_void_p(_stream(dev))))
    return out


def balance_stages(lengths: torch.Tensor, D: int, a: int, b: int, out: Assignment, ws: torch.Tensor, events):
    """orch_balance_stages: orch_balance that records the caller's four torch.cuda.Event objects
    (created with enable_timing=True and recorded once before, so that their handles exist)
    before the sort, after it, after the greedy and after the layout kernel."""
    lib = load_library()
    assert lengths.dtype == torch.int32 and lengths.is_cuda and lengths.is_contiguous() and len(events) == 4
    arr = (C.c_void_p * 4)(*[C.c_void_p(e.cuda_event) for e in events])
    _check(lib.orch_balance_stages(_ptr(lengths), lengths.numel(), D, _Phase(a, b), out._c(), _ptr(ws), ws.numel(),
                                   C.c_void_p(_stream(lengths.device)), arr))
    return out


def balance_static(lengths: torch.Tensor, D: int, a: int, b: int, out: Assignment) -> Assignment:
    """orch_balance_static: orch_balance on the library's built-in scratch; allocates nothing, so
    `out` must be given."""
    lib = load_library()
    assert lengths.dtype == torch.int32 and lengths.is_cuda and lengths.is_contiguous()
    _check(lib.orch_balance_static(_ptr(lengths), lengths.numel(), D, _Phase(a, b), out._c(),
                                   C.c_void_p(_stream(lengths.device))))
    return out


def balance_static_max_n() -> int:
    return load_library().orch_balance_static_max_n()


def balance_padded(lengths: torch.Tensor, D: int, a: int, b: int, out: Assignment | None = None,
                   bound: torch.Tensor | None = None, ws: torch.Tensor | None = None) -> Assignment:
    """orch_balance_padded: Algorithm 2 (Sec. 5.1, batching with paddings).  `bound`, if given, is an
    int64 device tensor of one element that receives the bound found."""
    lib = load_library()
    assert lengths.dtype == torch.int32 and lengths.is_cuda and lengths.is_contiguous()
    assert bound is None or (bound.dtype == torch.int64 and bound.is_cuda and bound.numel() == 1)
    n = lengths.numel()
    dev = lengths.device
    if out is None:
        out = Assignment.empty(n, D, dev)
    if ws is None:
        ws = _workspace(lib.orch_balance_workspace(n, max(D, 1)), dev)
    _check(lib.orch_balance_padded(_ptr(lengths), n, D, _Phase(a, b), out._c(), _ptr(bound), _ptr(ws),
                                   ws.numel(), C.c_void_p(_stream(dev))))
    return out


def balance_tolerance(lengths: torch.Tensor, D: int, v: int, a: int, b: int, out: Assignment | None = None,
                      ws: torch.Tensor | None = None) -> Assignment:
    """orch_balance_tolerance: the appendix's third algorithm with tolerance interval v."""
    lib = load_library()
    assert lengths.dtype == torch.int32 and lengths.is_cuda and lengths.is_contiguous()
    n = lengths.numel()
    dev = lengths.device
    if out is None:
        out = Assignment.empty(n, D, dev)
    if ws is None:
        ws = _workspace(lib.orch_balance_workspace(n, max(D, 1)), dev)
    _check(lib.orch_balance_tolerance(_ptr(lengths), n, D, v, _Phase(a, b), out._c(), _ptr(ws), ws.numel(),
                                      C.c_void_p(_stream(dev))))
    return out


def pack(tokens: torch.Tensor, lengths: torch.Tensor, asg: Assignment, inst_begin: int = 0,
         inst_end: int | None = None, out: torch.Tensor | None = None, packed_rows: int | None = None,
         ws: torch.Tensor | None = None) -> torch.Tensor:
    """orch_pack: tokens [T,H] (any 2-byte dtype) -> packed rows of the chosen instances
    (Sec. 5.2.1).  Without `out`, packed_rows rows are allocated (default T)."""
    lib = load_library()
    assert tokens.is_cuda and tokens.is_contiguous() and tokens.element_size() == 2 and tokens.dim() == 2
    T, H = tokens.shape
    dev = tokens.device
    if inst_end is None:
        inst_end = asg.D
    if out is None:
        out = torch.empty((T if packed_rows is None else packed_rows, H), dtype=tokens.dtype, device=dev)
    assert out.is_contiguous() and out.dtype == tokens.dtype and out.shape[1] == H
    if ws is None:
        ws = _workspace(lib.orch_pack_workspace(asg.n, asg.D), dev)
    _check(lib.orch_pack(_ptr(tokens), _ptr(out), _ptr(lengths), asg.n, asg.D, T, H, out.shape[0],
                         asg._c(), inst_begin, inst_end, _ptr(ws), ws.numel(), C.c_void_p(_stream(dev))))
    return out


def pack_composed(enc_rows: torch.Tensor, out: torch.Tensor, sub_len: torch.Tensor, sub_off: torch.Tensor,
                  src: Assignment | None, dst: Assignment, inst_begin: int = 0, inst_end: int | None = None,
                  ws: torch.Tensor | None = None) -> torch.Tensor:
    """orch_pack_composed (Sec. 5.3): one modality's rows, in the order of the encoder-phase
    assignment `src` (None = original example order), written in place into `out`, the packed
    LLM batch of assignment `dst`, at row `sub_off[s]` of every example's sequence."""
    lib = load_library()
    assert enc_rows.is_cuda and enc_rows.is_contiguous() and enc_rows.element_size() == 2 and enc_rows.dim() == 2
    assert out.is_contiguous() and out.dtype == enc_rows.dtype and out.dim() == 2 and out.shape[1] == enc_rows.shape[1]
    for t in (sub_len, sub_off):
        assert t.dtype == torch.int32 and t.is_cuda and t.is_contiguous() and t.numel() == dst.n
    assert src is None or src.n == dst.n
    dev = enc_rows.device
    if inst_end is None:
        inst_end = dst.D
    if ws is None:
        ws = _workspace(lib.orch_pack_composed_workspace(dst.n), dev)
    src_c = src._c() if src is not None else None
    _check(lib.orch_pack_composed(_ptr(enc_rows), _ptr(out), _ptr(sub_len), _ptr(sub_off), dst.n,
                                  src.D if src is not None else 0, C.byref(src_c) if src_c is not None else None,
                                  dst.D, dst._c(), enc_rows.shape[0], enc_rows.shape[1], out.shape[0],
                                  inst_begin, inst_end, _ptr(ws), ws.numel(), C.c_void_p(_stream(dev))))
    return out


def pack_composed_pieces(enc_rows: torch.Tensor, out: torch.Tensor, piece_ptr: torch.Tensor, piece_off: torch.Tensor,
                         piece_len: torch.Tensor, src: Assignment | None, dst: Assignment, inst_begin: int = 0,
                         inst_end: int | None = None, ws: torch.Tensor | None = None) -> torch.Tensor:
    """orch_pack_composed_pieces (Sec. 6 on Sec. 5.3): as pack_composed, with example s's run of rows cut
    into the pieces piece_ptr[s] .. piece_ptr[s+1]-1 placed at rows piece_off of its sequence."""
    lib = load_library()
    assert enc_rows.is_cuda and enc_rows.is_contiguous() and enc_rows.element_size() == 2 and enc_rows.dim() == 2
    assert out.is_contiguous() and out.dtype == enc_rows.dtype and out.dim() == 2 and out.shape[1] == enc_rows.shape[1]
    for t in (piece_ptr, piece_off, piece_len):
        assert t.dtype == torch.int32 and t.is_cuda and t.is_contiguous()
    assert piece_ptr.numel() == dst.n + 1 and piece_off.numel() == piece_len.numel()
    assert src is None or src.n == dst.n
    dev = enc_rows.device
    P = piece_off.numel()
    if inst_end is None:
        inst_end = dst.D
    if ws is None:
        ws = _workspace(lib.orch_pack_composed_pieces_workspace(dst.n, P), dev)
    src_c = src._c() if src is not None else None
    _check(lib.orch_pack_composed_pieces(_ptr(enc_rows), _ptr(out), _ptr(piece_ptr), _ptr(piece_off), _ptr(piece_len),
                                         dst.n, P, src.D if src is not None else 0,
                                         C.byref(src_c) if src_c is not None else None, dst.D, dst._c(),
                                         enc_rows.shape[0], enc_rows.shape[1], out.shape[0], inst_begin, inst_end,
                                         _ptr(ws), ws.numel(), C.c_void_p(_stream(dev))))
    return out


def pack_composed_pieces_workspace(n: int, n_pieces: int) -> int:
    return load_library().orch_pack_composed_pieces_workspace(n, n_pieces)


def comm_volume(lengths: torch.Tensor, asg: Assignment, D_src: int, src_inst: torch.Tensor | None = None,
                node: int = 0):
    """orch_comm_volume (Sec. 5.2.2): returns (V int64[D_src, D], inter int64[D_src]) holding u64 values."""
    lib = load_library()
    assert lengths.dtype == torch.int32 and lengths.is_cuda and lengths.is_contiguous()
    assert src_inst is None or (src_inst.dtype == torch.int32 and src_inst.is_cuda and src_inst.numel() == asg.n)
    dev = lengths.device
    V = torch.empty((D_src, asg.D), dtype=torch.int64, device=dev)
    inter = torch.empty(D_src, dtype=torch.int64, device=dev)
    _check(lib.orch_comm_volume(_ptr(lengths), asg.n, D_src, _ptr(src_inst), asg.D, asg._c(), _ptr(V), node,
                                _ptr(inter), C.c_void_p(_stream(dev))))
    return V, inter


def varlen_attn_fwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens: torch.Tensor,
                    causal: bool, scale: float = 0.0, max_seqlen: int = 0, out: torch.Tensor | None = None,
                    lse: torch.Tensor | None = None, ws: torch.Tensor | None = None,
                    dev_status: torch.Tensor | None = None) -> torch.Tensor:
    """orch_varlen_attn_fwd: q [T,Hq,d], k,v [T,Hkv,d] bf16, cu_seqlens int32[batch+1];
    dev_status, if given, is an int32 device tensor of one element."""
    lib = load_library()
    for t in (q, k, v):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.bfloat16 and t.dim() == 3
    assert cu_seqlens.dtype == torch.int32 and cu_seqlens.is_cuda and cu_seqlens.is_contiguous()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    assert k.shape == v.shape == (T, Hkv, d)
    dev = q.device
    batch = cu_seqlens.numel() - 1
    if out is None:
        out = torch.empty_like(q)
    if lse is not None:
        assert lse.dtype == torch.float32 and lse.is_contiguous() and lse.numel() == Hq * T
    if ws is None:
        ws = _workspace(lib.orch_varlen_attn_workspace(batch, T, Hq), dev)
    _check(lib.orch_varlen_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(cu_seqlens),
                                    batch, T, max_seqlen, Hq, Hkv, d, float(scale), 1 if causal else 0,
                                    _ptr(dev_status), _ptr(ws), ws.numel(), C.c_void_p(_stream(dev))))
    return out


def varlen_attn_bwd_workspace(batch: int, total_tokens: int, Hq: int) -> int:
    return load_library().orch_varlen_attn_bwd_workspace(batch, total_tokens, Hq)


def varlen_attn_bwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, out: torch.Tensor, lse: torch.Tensor,
                    dout: torch.Tensor, cu_seqlens: torch.Tensor, causal: bool, scale: float = 0.0,
                    max_seqlen: int = 0, dq: torch.Tensor | None = None, dk: torch.Tensor | None = None,
                    dv: torch.Tensor | None = None, ws: torch.Tensor | None = None,
                    dev_status: torch.Tensor | None = None):
    """orch_varlen_attn_bwd: (dq, dk, dv) from the forward pass's inputs, out and lse, and dout."""
    lib = load_library()
    for t in (q, k, v, out, dout):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.bfloat16 and t.dim() == 3
    assert cu_seqlens.dtype == torch.int32 and cu_seqlens.is_cuda and cu_seqlens.is_contiguous()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    assert k.shape == v.shape == (T, Hkv, d) and out.shape == dout.shape == q.shape
    assert lse.dtype == torch.float32 and lse.is_cuda and lse.is_contiguous() and lse.numel() == Hq * T
    dev = q.device
    batch = cu_seqlens.numel() - 1
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    for t, ref in ((dq, q), (dk, k), (dv, v)):
        assert t.is_contiguous() and t.dtype == torch.bfloat16 and t.shape == ref.shape
    if ws is None:
        ws = _workspace(lib.orch_varlen_attn_bwd_workspace(batch, T, Hq), dev)
    _check(lib.orch_varlen_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(dout), _ptr(dq), _ptr(dk),
                                    _ptr(dv), _ptr(cu_seqlens), batch, T, max_seqlen, Hq, Hkv, d, float(scale),
                                    1 if causal else 0, _ptr(dev_status), _ptr(ws), ws.numel(),
                                    C.c_void_p(_stream(dev))))
    return dq, dk, dv


def attn_variant() -> str:
    return load_library().orch_attn_variant().decode()
