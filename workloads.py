"""Seeded synthetic inputs for the five dispatcher / varlen-attention workloads.

This module only *draws inputs*: sequence lengths, opaque 16-bit token rows and
N(0,1) bf16 q/k/v.  It contains none of the method's arithmetic (no cost, no
sort, no assignment, no attention) and is the one module that both the HIP
path's tests/bench and the CPU oracle's tests may import.

Random numbers come from a counter-based generator (a 64-bit mixing function
applied to seed/stream/counter), so a draw depends only on its coordinates and
not on numpy's or torch's generator versions.

The length laws stand in for the paper's production mixes (Sec. 7, "Models"
and "Datasets"): image patch counts of 224..672-pixel images at patch 14,
log-normally distributed audio frame counts, and LLM-phase sequences whose
text / image / audio composition varies per example (Sec. 3.2, Modality
Composition Incoherence).
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

BASE_SEED = 2503
_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_MIX1 = 0xBF58476D1CE4E5B9
_MIX2 = 0x94D049BB133111EB


# ----------------------------------------------------------------------------
# counter-based generator (numpy, uint64)
# ----------------------------------------------------------------------------
def _mix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on a uint64 array (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        x = (x + np.uint64(_GOLD)).astype(np.uint64)
        x = (x ^ (x >> np.uint64(30))) * np.uint64(_MIX1)
        x = (x ^ (x >> np.uint64(27))) * np.uint64(_MIX2)
        x = x ^ (x >> np.uint64(31))
    return x


def bits64(seed: int, stream: int, count: int, offset: int = 0) -> np.ndarray:
    """`count` 64-bit words of stream `stream` under `seed`, counters offset.."""
    key = _mix64(np.array([(seed * 0x100000001B3 + stream * _GOLD) & _M64], dtype=np.uint64))[0]
    ctr = np.arange(offset, offset + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix64(ctr * np.uint64(_MIX2) ^ key)


def uniform01(seed: int, stream: int, count: int, offset: int = 0) -> np.ndarray:
    """Uniform doubles in (0, 1): 53 random bits, never exactly 0 or 1."""
    u = (bits64(seed, stream, count, offset) >> np.uint64(11)).astype(np.float64)
    return (u + 0.5) * (1.0 / 9007199254740992.0)


def normal01(seed: int, stream: int, count: int) -> np.ndarray:
    """Standard normals by Box-Muller on two uniform streams."""
    u1 = uniform01(seed, stream, count, 0)
    u2 = uniform01(seed, stream ^ 0x5A5A5A5A, count, 1 << 40)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)


def gamma_small(seed: int, stream: int, count: int, shape: float, rounds: int = 12) -> np.ndarray:
    """Gamma(shape<1, 1) draws: Marsaglia-Tsang at shape+1 with a fixed number
    of vectorised rejection rounds, then the U^(1/shape) boost."""
    a1 = shape + 1.0
    dd = a1 - 1.0 / 3.0
    cc = 1.0 / math.sqrt(9.0 * dd)
    out = np.full(count, dd, dtype=np.float64)
    done = np.zeros(count, dtype=bool)
    for r in range(rounds):
        x = normal01(seed, stream + 1000 * (r + 1), count)
        u = uniform01(seed, stream + 1000 * (r + 1) + 500, count)
        v = (1.0 + cc * x) ** 3
        ok = v > 0
        lv = np.log(np.where(ok, v, 1.0))
        acc = ok & (np.log(u) < 0.5 * x * x + dd - dd * v + dd * lv)
        take = acc & ~done
        out[take] = dd * v[take]
        done |= acc
    boost = uniform01(seed, stream + 777, count) ** (1.0 / shape)
    return out * boost


# ----------------------------------------------------------------------------
# workload descriptions
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    cid: int           # 1..5
    name: str
    n: int             # sequences in the global batch
    D: int             # data-parallel instances
    a: int             # quadratic cost coefficient
    b: int             # linear cost coefficient
    H: int             # bf16 elements per token row (pack)
    Hq: int
    Hkv: int
    d: int
    causal: bool
    law: str


# Cost presets: C1's (a, b) is given with the workload; the others follow FLOP
# counting of a plain transformer layer: linear work ~24 h^2 per token,
# attention 4 h L per token bidirectional (half of that causal), so with a = 1
# the linear coefficient is 6 h (bidirectional) or 12 h (causal).
WORKLOADS = {
    1: Workload(1, "C1-tiny-text", 64, 4, 1, 512, 256, 4, 4, 64, True, "uniform16_512"),
    2: Workload(2, "C2-vision", 512, 8, 1, 6144, 1024, 16, 16, 64, False, "image_patches"),
    3: Workload(3, "C3-audio", 1024, 16, 1, 7680, 1280, 16, 16, 64, False, "audio_frames"),
    4: Workload(4, "C4-llm-mci", 4096, 32, 1, 49152, 4096, 32, 8, 128, True, "llm_8192"),
    5: Workload(5, "C5-llm-84b", 32768, 256, 1, 98304, 8192, 64, 8, 128, True, "llm_32768"),
}


def seed_for(cid: int, base_seed: int = BASE_SEED) -> int:
    return base_seed * 16 + cid


def _lognormal_int(seed, stream, n, median, sigma, lo, hi):
    z = normal01(seed, stream, n)
    x = np.rint(np.exp(math.log(median) + sigma * z))
    return np.clip(x, lo, hi).astype(np.int32)


def draw_lengths(w: Workload, base_seed: int = BASE_SEED) -> np.ndarray:
    """int32[n] sequence lengths of workload `w` (what the phase balances on)."""
    s = seed_for(w.cid, base_seed)
    if w.law == "uniform16_512":
        u = uniform01(s, 1, w.n)
        return (16 + np.floor(u * 497.0)).astype(np.int32)
    if w.law == "image_patches":
        u = uniform01(s, 1, w.n)
        edges = np.cumsum([0.2, 0.3, 0.25, 0.15, 0.1])
        vals = np.array([0, 256, 576, 1024, 2304], dtype=np.int32)
        return vals[np.minimum(np.searchsorted(edges, u, side="right"), 4)]
    if w.law == "audio_frames":
        L = _lognormal_int(s, 1, w.n, 300.0, 0.8, 25, 1500)
        none = uniform01(s, 2, w.n) < 0.2
        L[none] = 0
        return L
    if w.law == "llm_8192":
        return _lognormal_int(s, 1, w.n, 2048.0, 0.9, 64, 8192)
    if w.law == "llm_32768":
        return _lognormal_int(s, 1, w.n, 2048.0, 0.9, 64, 32768)
    raise ValueError(w.law)


def draw_modality_split(w: Workload, lengths: np.ndarray, base_seed: int = BASE_SEED) -> np.ndarray:
    """int32[n,3] (text, image, audio) token counts per example, summing to the
    example's length: total * Dirichlet(0.3,0.3,0.3), largest-remainder rounding."""
    s = seed_for(w.cid, base_seed)
    n = len(lengths)
    g = np.stack([gamma_small(s, 100 + 10 * j, n, 0.3) for j in range(3)], axis=1)
    g = np.maximum(g, 1e-300)
    p = g / g.sum(axis=1, keepdims=True)
    raw = p * lengths[:, None].astype(np.float64)
    base = np.floor(raw).astype(np.int64)
    rem = lengths.astype(np.int64) - base.sum(axis=1)
    frac = raw - base
    rank = np.argsort(np.argsort(-frac, axis=1, kind="stable"), axis=1, kind="stable")
    base += (rank < rem[:, None]).astype(np.int64)
    return base.astype(np.int32)


def draw_interleave_offsets(split: np.ndarray, seed: int) -> np.ndarray:
    """int32[n,3]: the row at which each modality's sub-sequence starts inside its example's
    interleaved sequence.  Every example orders its three modalities by a seeded permutation
    and lays them out back to back (Sec. 3.1: sub-sequences are interleaved per example)."""
    n = split.shape[0]
    perms = np.array([[0, 1, 2], [0, 2, 1], [1, 0, 2], [1, 2, 0], [2, 0, 1], [2, 1, 0]], dtype=np.int64)
    slot_mod = perms[(uniform01(seed, 21, n) * 6).astype(np.int64)]  # [n,3]: slot -> modality
    lens = np.take_along_axis(split.astype(np.int64), slot_mod, axis=1)
    starts = np.cumsum(lens, axis=1) - lens
    off = np.empty((n, 3), dtype=np.int32)
    np.put_along_axis(off, slot_mod, starts.astype(np.int32), axis=1)
    return off


def draw_piece_layout(split: np.ndarray, seed: int, max_pieces: int = 4):
    """Several sub-sequences per (example, modality) (Sec. 6: an example's subsequences are interleaved
    in a predefined order; e.g. several images between pieces of text).  Every modality's token count
    of an example is cut into 1..max_pieces pieces (0 pieces when the count is 0) at seeded cut points,
    and the pieces of the three modalities are laid out back to back in a seeded order that keeps each
    modality's own pieces in sequence.  Returns one (piece_ptr int32[n+1], piece_off int32[P],
    piece_len int32[P]) triple per modality; offsets are rows inside the example's interleaved
    sequence."""
    n, M = split.shape
    ptr = [np.zeros(n + 1, dtype=np.int64) for _ in range(M)]
    offs = [[] for _ in range(M)]
    lens = [[] for _ in range(M)]
    u_cnt = uniform01(seed, 31, n * M).reshape(n, M)
    u_cut = uniform01(seed, 32, n * M * max_pieces).reshape(n, M, max_pieces)
    u_ord = uniform01(seed, 33, n * M * max_pieces).reshape(n, M, max_pieces)
    for s in range(n):
        pieces = []   # (order key, modality, index within modality, length)
        for m in range(M):
            tot = int(split[s, m])
            k = 0 if tot == 0 else min(tot, 1 + int(u_cnt[s, m] * max_pieces))
            cuts = np.sort((u_cut[s, m, : max(k - 1, 0)] * (tot + 1)).astype(np.int64)) if k > 1 else np.zeros(0, np.int64)
            edges = np.concatenate([[0], cuts, [tot]])
            keys = np.sort(u_ord[s, m, :k])   # ascending keys keep the modality's pieces in order
            for t in range(k):
                pieces.append((float(keys[t]), m, t, int(edges[t + 1] - edges[t])))
            ptr[m][s + 1] = ptr[m][s] + k
        pieces.sort(key=lambda x: (x[0], x[1], x[2]))
        row = 0
        place = {}
        for _, m, t, ln in pieces:
            place[(m, t)] = (row, ln)
            row += ln
        for m in range(M):
            for t in range(int(ptr[m][s + 1] - ptr[m][s])):
                offs[m].append(place[(m, t)][0])
                lens[m].append(place[(m, t)][1])
    return [(ptr[m].astype(np.int32), np.array(offs[m], dtype=np.int32), np.array(lens[m], dtype=np.int32))
            for m in range(M)]


def random_lengths(seed: int, n: int, lo: int, hi: int, zero_frac: float = 0.0) -> np.ndarray:
    """Generic test helper: uniform ints in [lo, hi], a fraction forced to 0."""
    u = uniform01(seed, 11, n)
    L = (lo + np.floor(u * (hi - lo + 1))).astype(np.int32)
    if zero_frac > 0:
        L[uniform01(seed, 12, n) < zero_frac] = 0
    return L


# ----------------------------------------------------------------------------
# payloads
# ----------------------------------------------------------------------------
def token_tag_np(rows: np.ndarray, H: int) -> np.ndarray:
    """uint16[len(rows), H]: the opaque 16-bit word of element (row, column) of
    the source token buffer, a pure function of the *global source row*."""
    r = np.asarray(rows, dtype=np.uint64)[:, None]
    c = np.arange(H, dtype=np.uint64)[None, :]
    with np.errstate(over="ignore"):
        x = (r * np.uint64(H) + c) * np.uint64(_GOLD)
        x = (x ^ (x >> np.uint64(29))) * np.uint64(_MIX1)
    return ((x >> np.uint64(40)) & np.uint64(0xFFFF)).astype(np.uint16)


def _s64(v: int) -> int:
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


def token_tag_torch(row_begin: int, row_end: int, H: int, device, out=None):
    """Same words as token_tag_np for rows [row_begin,row_end), produced with
    torch integer ops on `device`; returns (or fills) an int16 tensor viewed as
    the bf16 bit pattern."""
    import torch

    nrow = row_end - row_begin
    if out is None:
        out = torch.empty((nrow, H), dtype=torch.int16, device=device)
    step = max(1, (1 << 25) // H)
    c = torch.arange(H, dtype=torch.int64, device=device)[None, :]
    for r0 in range(0, nrow, step):
        r1 = min(nrow, r0 + step)
        r = torch.arange(row_begin + r0, row_begin + r1, dtype=torch.int64, device=device)[:, None]
        x = (r * H + c) * _s64(_GOLD)
        x = (x ^ ((x >> 29) & ((1 << 35) - 1))) * _s64(_MIX1)
        out[r0:r1] = ((x >> 40) & 0xFFFF).to(torch.int16)
    return out


def token_tag_rows_torch(rows, H: int):
    """Same words as token_tag_np for an arbitrary list of global source rows: `rows` is an
    int64 tensor on the target device; returns int16 [len(rows), H].  The caller bounds the
    chunk (8 * len(rows) * H bytes of temporaries)."""
    import torch

    c = torch.arange(H, dtype=torch.int64, device=rows.device)[None, :]
    x = (rows.to(torch.int64)[:, None] * H + c) * _s64(_GOLD)
    x = (x ^ ((x >> 29) & ((1 << 35) - 1))) * _s64(_MIX1)
    return ((x >> 40) & 0xFFFF).to(torch.int16)


def normal_bf16_torch(shape, seed: int, stream: int, device):
    """bf16 tensor ~ N(0,1) of `shape`, counter-based (hash of the flat index),
    generated with torch ops on `device` in bounded chunks."""
    import torch

    total = 1
    for s in shape:
        total *= int(s)
    out = torch.empty(total, dtype=torch.bfloat16, device=device)
    key = int(_mix64(np.array([(seed * 0x100000001B3 + stream * _GOLD) & _M64], dtype=np.uint64))[0])
    step = 1 << 24

    def mix(x):
        x = x + _s64(_GOLD)
        x = (x ^ ((x >> 30) & ((1 << 34) - 1))) * _s64(_MIX1)
        x = (x ^ ((x >> 27) & ((1 << 37) - 1))) * _s64(_MIX2)
        return x ^ ((x >> 31) & ((1 << 33) - 1))

    for o in range(0, total, step):
        e = min(total, o + step)
        i = torch.arange(o, e, dtype=torch.int64, device=device)
        h = mix((i * _s64(_MIX2)) ^ _s64(key))
        u1 = (((h >> 40) & 0xFFFFFF).to(torch.float32) + 0.5) * (1.0 / 16777216.0)
        u2 = (((h >> 8) & 0xFFFFFF).to(torch.float32) + 0.5) * (1.0 / 16777216.0)
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
        out[o:e] = z.to(torch.bfloat16)
    return out.view(*shape)
