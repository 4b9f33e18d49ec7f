"""HIP orch_pack vs the CPU oracle: bit-exact rows."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_23830_amd as orch
import workloads as wl
from gpu_common import bits, run_balance

pytestmark = pytest.mark.gpu

GUARD = 0x7C7C


def pack_with_guards(tokens, Ld, asg, rows, H, dev, inst_begin=0, inst_end=None):
    """Pack into the middle of a guarded buffer; returns (packed, guards_intact)."""
    pad = 64
    buf = torch.full((rows + 2 * pad, H), GUARD, dtype=torch.int16, device=dev)
    out = buf[pad: pad + rows]
    orch.pack(tokens, Ld, asg, inst_begin, inst_end, out=out)
    torch.cuda.synchronize()
    ok = bool((buf[:pad] == GUARD).all()) and bool((buf[pad + rows:] == GUARD).all())
    return out, ok


@pytest.mark.parametrize("cid", [1, 2, 3])
def test_whole_configs(gpu_device, cid):
    w = wl.WORKLOADS[cid]
    L = wl.draw_lengths(w)
    T = int(L.sum())
    Ld, asg = run_balance(L, w.D, w.a, w.b, gpu_device)
    ref = oracle.balance(L, w.D, w.a, w.b)
    tokens = wl.token_tag_torch(0, T, w.H, gpu_device)
    src_before = tokens.clone()
    packed, guards = pack_with_guards(tokens, Ld, asg, T, w.H, gpu_device)
    assert guards
    assert torch.equal(tokens, src_before)  # inputs are never written
    want = oracle.pack(wl.token_tag_np(np.arange(T), w.H), L, ref)
    assert np.array_equal(bits(packed), want)
    assert int(asg.dev_status.item()) == 0


@pytest.mark.parametrize("H", [8, 24, 100, 2, 1, 3, 1280])
def test_row_widths_and_alignment(gpu_device, H):
    # row sizes that force 16-, 8-, 4- and 2-byte accesses; many tiny and empty sequences
    L = wl.random_lengths(40 + H, 700, 0, 9, zero_frac=0.3)
    T = int(L.sum())
    Ld, asg = run_balance(L, 5, 1, 3, gpu_device)
    ref = oracle.balance(L, 5, 1, 3)
    tokens = wl.token_tag_torch(0, T, H, gpu_device)
    packed, guards = pack_with_guards(tokens, Ld, asg, T, H, gpu_device)
    assert guards
    assert np.array_equal(bits(packed), oracle.pack(wl.token_tag_np(np.arange(T), H), L, ref))


@pytest.mark.parametrize("H,n,hi,zero", [(8, 60000, 3, 0.5), (1, 30000, 5, 0.9), (64, 40000, 40, 0.2)])
def test_many_tiny_and_empty_sequences(gpu_device, H, n, hi, zero):
    # thousands of segments under one lookup granule, long runs of empty ones, pieces that straddle
    # dozens of segments: the copy kernel's searches instead of its common path
    L = wl.random_lengths(900 + H, n, 0, hi, zero_frac=zero)
    T = int(L.sum())
    Ld, asg = run_balance(L, 64, 1, 3, gpu_device)
    ref = oracle.balance(L, 64, 1, 3)
    tokens = wl.token_tag_torch(0, T, H, gpu_device)
    packed, guards = pack_with_guards(tokens, Ld, asg, T, H, gpu_device)
    assert guards
    assert np.array_equal(bits(packed), oracle.pack(wl.token_tag_np(np.arange(T), H), L, ref))
    # one instance's share through inst_begin / inst_end
    i0, i1 = 17, 19
    rows = int(ref.tok_off[i1] - ref.tok_off[i0])
    part, guards = pack_with_guards(tokens, Ld, asg, rows, H, gpu_device, i0, i1)
    assert guards
    assert np.array_equal(bits(part), bits(packed)[int(ref.tok_off[i0]): int(ref.tok_off[i1])])


def test_instance_subrange(gpu_device):
    w = wl.WORKLOADS[3]
    L = wl.draw_lengths(w)
    T = int(L.sum())
    Ld, asg = run_balance(L, w.D, w.a, w.b, gpu_device)
    ref = oracle.balance(L, w.D, w.a, w.b)
    tokens = wl.token_tag_torch(0, T, w.H, gpu_device)
    src = wl.token_tag_np(np.arange(T), w.H)
    for lo, hi in [(0, 1), (3, 7), (15, 16), (5, 5)]:
        rows = int(ref.tok_off[hi] - ref.tok_off[lo])
        packed, guards = pack_with_guards(tokens, Ld, asg, rows, w.H, gpu_device, lo, hi)
        assert guards
        assert np.array_equal(bits(packed), oracle.pack(src, L, ref, lo, hi))


def test_edge_cases(gpu_device):
    # n = 0
    L = np.zeros(0, np.int32)
    Ld, asg = run_balance(L, 3, 1, 1, gpu_device)
    tokens = torch.empty((0, 64), dtype=torch.int16, device=gpu_device)
    out = orch.pack(tokens, Ld, asg)
    torch.cuda.synchronize()
    assert out.shape[0] == 0 and int(asg.dev_status.item()) == 0
    # all sequences empty
    L = np.zeros(10, np.int32)
    Ld, asg = run_balance(L, 3, 1, 1, gpu_device)
    orch.pack(tokens, Ld, asg)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == 0
    # one sequence, one instance: identity
    L = np.array([300], np.int32)
    Ld, asg = run_balance(L, 1, 1, 1, gpu_device)
    tokens = wl.token_tag_torch(0, 300, 72, gpu_device)
    assert torch.equal(orch.pack(tokens, Ld, asg), tokens)


def test_too_small_destination_is_refused_on_device(gpu_device):
    L = wl.random_lengths(1, 50, 1, 20)
    T = int(L.sum())
    Ld, asg = run_balance(L, 4, 1, 1, gpu_device)
    tokens = wl.token_tag_torch(0, T, 32, gpu_device)
    buf = torch.full((T, 32), GUARD, dtype=torch.int16, device=gpu_device)
    orch.pack(tokens, Ld, asg, out=buf[: T - 1])
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == -5
    assert bool((buf == GUARD).all())  # nothing was written
    # a wrong T (source shorter than the lengths say) is refused too
    asg.dev_status.zero_()
    orch.pack(tokens[: T - 1], Ld, asg, out=buf)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == -5 and bool((buf == GUARD).all())


def test_c4_streamed_slice(gpu_device):
    """C4's row width (8 KiB) and length law at full n and D; rows are checked
    against the oracle's dst->src row map in chunks, for a range of instances
    whose rows fit comfortably in memory."""
    w = wl.WORKLOADS[4]
    L = wl.draw_lengths(w)
    # compact source: only sequences of the chosen instances carry rows
    ref_full = oracle.balance(L, w.D, w.a, w.b)
    lo, hi = 31, 32
    keep = np.isin(ref_full.inst, np.arange(lo, hi))
    Lc = np.where(keep, L, 0).astype(np.int32)
    # the compacted batch is its own workload: balance it and pack everything
    Ld, asg = run_balance(Lc, w.D, w.a, w.b, gpu_device)
    ref = oracle.balance(Lc, w.D, w.a, w.b)
    T = int(Lc.sum())
    tokens = wl.token_tag_torch(0, T, w.H, gpu_device)
    packed = orch.pack(tokens, Ld, asg)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == 0
    rmap = oracle.row_map(Lc, ref)
    step = 16384
    for r0 in range(0, T, step):
        r1 = min(T, r0 + step)
        assert np.array_equal(bits(packed[r0:r1]), wl.token_tag_np(rmap[r0:r1], w.H)), r0


def assert_rows_match_on_device(packed, rmap, H, dev, chunk_bytes=1 << 29):
    """Every row of `packed` (int16 [rows, H], on the device) against the tag of the source row
    the oracle's map names for it, compared on the device chunk by chunk: no sampling."""
    rows = packed.shape[0]
    assert rmap.shape == (rows,)
    rd = torch.from_numpy(np.ascontiguousarray(rmap, dtype=np.int64)).to(dev)
    step = max(1, chunk_bytes // (2 * H))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        want = wl.token_tag_rows_torch(rd[r0:r1], H)
        assert torch.equal(packed[r0:r1], want), "rows [%d, %d)" % (r0, r1)
        del want


def test_token_tag_generators_agree(gpu_device):
    """The three generators of the source words (numpy, contiguous torch, row-list torch) give
    the same bits, so a device-side comparison is the same check as a host-side one."""
    rows = np.array([0, 1, 5, 2 ** 20 + 3, 11_532_086, 2 ** 31 + 17, 99_999_999], dtype=np.int64)
    for H in (3, 256, 4096, 8192):
        a = wl.token_tag_np(rows, H)
        b = wl.token_tag_rows_torch(torch.from_numpy(rows).to(gpu_device), H)
        assert np.array_equal(bits(b), a)
        c = wl.token_tag_torch(1000, 1100, H, gpu_device)
        assert np.array_equal(bits(c), wl.token_tag_np(np.arange(1000, 1100), H))


def test_c4_whole_batch_every_row(gpu_device):
    """The whole C4 batch (about 94 GB in, 94 GB out) in the launch shape the bench times.
    Every one of the 11.5 M packed rows is compared, on the device, with the tag of the source
    row the oracle's dst -> src map gives for it; the source must be unchanged."""
    w = wl.WORKLOADS[4]
    L = wl.draw_lengths(w)
    T = int(L.sum())
    free, _ = torch.cuda.mem_get_info()
    if free < 2 * T * w.H * 2 + (12 << 30):
        pytest.skip("not enough free HBM for the full C4 pack")
    dev = gpu_device
    Ld, asg = run_balance(L, w.D, w.a, w.b, dev)
    ref = oracle.balance(L, w.D, w.a, w.b)
    tokens = wl.token_tag_torch(0, T, w.H, dev)
    packed = torch.full((T, w.H), GUARD, dtype=torch.int16, device=dev)
    orch.pack(tokens, Ld, asg, out=packed)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == 0
    rmap = oracle.row_map(L, ref)
    assert_rows_match_on_device(packed, rmap, w.H, dev)
    # inputs are never written: the source still holds its own tags
    assert_rows_match_on_device(tokens, np.arange(T, dtype=np.int64), w.H, dev)
    del tokens, packed
    torch.cuda.empty_cache()


def test_c5_straggler_share_every_row(gpu_device):
    """C5 (32768 sequences, 256 instances, 16 KiB rows): the whole batch is 1.6 TB, so the
    most loaded instance's share is packed from a compacted source (only that instance's
    sequences carry rows; the others have length 0 in the `lengths` handed to pack) through
    inst_begin / inst_end, with the assignment balance produced for the full lengths.  Every
    row is compared on the device with the oracle's placement."""
    w = wl.WORKLOADS[5]
    L = wl.draw_lengths(w)
    dev = gpu_device
    _, asg = run_balance(L, w.D, w.a, w.b, dev)
    ref = oracle.balance(L, w.D, w.a, w.b)
    i = int(np.argmax(ref.loads))
    keep = ref.inst == i
    Lc = np.where(keep, L, 0).astype(np.int32)
    Ti = int(Lc.sum())
    assert Ti == int(ref.tok_off[i + 1] - ref.tok_off[i]) and Ti > 300_000
    tokens = wl.token_tag_torch(0, Ti, w.H, dev)
    pad = 16
    buf = torch.full((Ti + 2 * pad, w.H), GUARD, dtype=torch.int16, device=dev)
    out = buf[pad: pad + Ti]
    orch.pack(tokens, torch.from_numpy(Lc).to(dev), asg, i, i + 1, out=out)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == 0
    assert bool((buf[:pad] == GUARD).all()) and bool((buf[pad + Ti:] == GUARD).all())
    # the oracle's placement of the compacted source rows: pack row ids instead of payloads
    ids = np.arange(Ti, dtype=np.int64)[:, None]
    rmap = oracle.pack(ids, Lc, ref, i, i + 1)[:, 0]
    assert np.array_equal(np.sort(rmap), ids[:, 0])
    assert_rows_match_on_device(out, rmap, w.H, dev, chunk_bytes=1 << 30)
    del tokens, buf
    torch.cuda.empty_cache()
