"""HIP orch_pack_composed (rearrangement composition, Sec. 5.3) vs the CPU oracle: bit-exact rows."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_23830_amd as orch
import workloads as wl
from gpu_common import bits, run_balance

pytestmark = pytest.mark.gpu

GUARD = 0x7C7C
SALT = 1 << 36  # tag rows of modality m start at m * SALT


def to_dev(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def host_rows(rows_u16, dev):
    return to_dev(rows_u16.view(np.int16), dev)


def encoder_side(sub, De, phase, m, H, dev):
    """One modality's encoder output in the encoder phase's packed order: the oracle packs tagged
    rows with ITS assignment (host); the device gets the same rows and the device-made assignment."""
    n_rows = int(sub.sum())
    tags = wl.token_tag_np(m * SALT + np.arange(n_rows), H)
    if De is None:
        return tags, None, None
    ref = oracle.balance(sub, De, *phase)
    _, asg = run_balance(sub, De, *phase, dev)
    return oracle.pack(tags, sub, ref), ref, asg


def compose_all(L, split, sub_off, Dm, phase_m, enc, H, dev, lo=0, hi=None, pad=64):
    """Run the three modalities through HIP and oracle; returns (device buffer with guards, rows,
    oracle result, llm assignment)."""
    hi = Dm if hi is None else hi
    mref = oracle.balance(L, Dm, *phase_m)
    _, masg = run_balance(L, Dm, *phase_m, dev)
    rows = int(mref.tok_off[hi] - mref.tok_off[lo])
    buf = torch.full((rows + 2 * pad, H), GUARD, dtype=torch.int16, device=dev)
    out = buf[pad: pad + rows]
    want = np.full((rows, H), GUARD, dtype=np.uint16)
    for m in range(3):
        sub = np.ascontiguousarray(split[:, m])
        De, phase_e = enc[m]
        rows_m, eref, easg = encoder_side(sub, De, phase_e, m, H, dev)
        oracle.pack_composed(rows_m, want, sub, sub_off[:, m], eref, mref, lo, hi)
        src_d = host_rows(rows_m, dev)
        before = src_d.clone()
        orch.pack_composed(src_d, out, to_dev(sub, dev), to_dev(sub_off[:, m], dev), easg, masg, lo, hi)
        torch.cuda.synchronize()
        assert torch.equal(src_d, before)  # inputs are never written
        assert easg is None or int(easg.dev_status.item()) == 0
    assert int(masg.dev_status.item()) == 0
    guards = bool((buf[:pad] == GUARD).all()) and bool((buf[pad + rows:] == GUARD).all())
    return out, guards, want, mref


ENC = {0: (None, None), 1: (4, (1, 6)), 2: (6, (1, 9))}  # text stays in original order


@pytest.mark.parametrize("cid", [1, 2, 3])
def test_three_modalities_whole_configs(gpu_device, cid):
    w = wl.WORKLOADS[cid]
    L = wl.draw_lengths(w)
    split = wl.draw_modality_split(w, L)
    sub_off = wl.draw_interleave_offsets(split, cid)
    out, guards, want, _ = compose_all(L, split, sub_off, w.D, (w.a, w.b), ENC, w.H, gpu_device)
    assert guards
    got = bits(out)
    assert np.array_equal(got, want)
    assert not (want == GUARD).all(axis=1).any()  # the three modalities tile every row


@pytest.mark.parametrize("H", [8, 24, 100, 2, 1, 3, 1280])
def test_row_widths_and_tiny_segments(gpu_device, H):
    # 16-, 8-, 4- and 2-byte accesses; many empty examples and 0- to 3-row sub-sequences
    L = wl.random_lengths(60 + H, 900, 0, 9, zero_frac=0.3)
    split = wl.draw_modality_split(wl.WORKLOADS[1], L)
    sub_off = wl.draw_interleave_offsets(split, H)
    enc = {0: (3, (1, 1)), 1: (None, None), 2: (7, (2, 1))}
    out, guards, want, _ = compose_all(L, split, sub_off, 5, (1, 3), enc, H, gpu_device)
    assert guards and np.array_equal(bits(out), want)


def test_instance_subrange(gpu_device):
    w = wl.WORKLOADS[3]
    L = wl.draw_lengths(w)
    split = wl.draw_modality_split(w, L)
    sub_off = wl.draw_interleave_offsets(split, 9)
    for lo, hi in [(0, 1), (3, 7), (15, 16), (5, 5)]:
        out, guards, want, _ = compose_all(L, split, sub_off, w.D, (w.a, w.b), ENC, 256, gpu_device, lo, hi)
        assert guards and np.array_equal(bits(out), want)


def test_special_cases(gpu_device):
    dev = gpu_device
    w = wl.WORKLOADS[1]
    L = wl.draw_lengths(w)
    T, H = int(L.sum()), 40
    Ld, asg = run_balance(L, w.D, w.a, w.b, dev)
    ref = oracle.balance(L, w.D, w.a, w.b)
    zero = torch.zeros(len(L), dtype=torch.int32, device=dev)
    tokens = wl.token_tag_torch(0, T, H, dev)
    tok_np = wl.token_tag_np(np.arange(T), H)
    # identity source, whole sequences, offset 0: the plain pack (oracle's and the library's own)
    out = torch.zeros_like(tokens)
    orch.pack_composed(tokens, out, Ld, zero, None, asg)
    torch.cuda.synchronize()
    assert np.array_equal(bits(out), oracle.pack(tok_np, L, ref))
    assert torch.equal(out, orch.pack(tokens, Ld, asg))
    # source order = destination order: the identity map
    out2 = torch.zeros_like(tokens)
    orch.pack_composed(out, out2, Ld, zero, asg, asg)
    torch.cuda.synchronize()
    assert torch.equal(out2, out)
    # an empty modality writes nothing
    sent = torch.full_like(tokens, GUARD)
    orch.pack_composed(tokens[:0], sent, zero, zero, None, asg)
    torch.cuda.synchronize()
    assert bool((sent == GUARD).all()) and int(asg.dev_status.item()) == 0
    # n = 0
    L0 = np.zeros(0, np.int32)
    L0d, asg0 = run_balance(L0, 3, 1, 1, dev)
    e = torch.empty((0, H), dtype=torch.int16, device=dev)
    orch.pack_composed(e, e.clone(), L0d, L0d, None, asg0)
    orch.pack_composed(e, e.clone(), L0d, L0d, asg0, asg0)
    torch.cuda.synchronize()
    assert int(asg0.dev_status.item()) == 0


def test_inconsistent_data_is_refused_on_device(gpu_device):
    dev = gpu_device
    L = wl.random_lengths(3, 80, 1, 20)
    T, H = int(L.sum()), 32
    Ld, asg = run_balance(L, 4, 1, 1, dev)
    zero = torch.zeros(len(L), dtype=torch.int32, device=dev)
    tokens = wl.token_tag_torch(0, T, H, dev)
    buf = torch.full((T, H), GUARD, dtype=torch.int16, device=dev)

    def refused(*args, **kw):
        asg.dev_status.zero_()
        orch.pack_composed(*args, **kw)
        torch.cuda.synchronize()
        ok = int(asg.dev_status.item()) == -5 and bool((buf == GUARD).all())
        asg.dev_status.zero_()
        return ok

    # a sub-sequence that overruns its interleaved sequence
    off = zero.clone()
    off[int(np.argmax(L))] = 1
    assert refused(tokens, buf, Ld, off, None, asg)
    # negative offset
    off = zero.clone()
    off[3] = -1
    assert refused(tokens, buf, Ld, off, None, asg)
    # destination too small / source shorter than sub_len says
    assert refused(tokens, buf[: T - 1], Ld, zero, None, asg)
    assert refused(tokens[: T - 1], buf, Ld, zero, None, asg)
    # an encoder segment shorter than the sub-sequence (a longer one is a padded slot and is fine)
    longer = (L + 1).astype(np.int32)
    Lg, dst_longer = run_balance(longer, 4, 1, 1, dev)
    big = torch.full((int(longer.sum()), H), GUARD, dtype=torch.int16, device=dev)
    orch.pack_composed(tokens, big, Lg, zero, asg, dst_longer)
    torch.cuda.synchronize()
    assert int(dst_longer.dev_status.item()) == -5 and bool((big == GUARD).all())
    shorter = np.maximum(L - 1, 0).astype(np.int32)
    orch.pack_composed(tokens, big, to_dev(shorter, dev), zero, asg, asg)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == 0
    want = np.full((int(longer.sum()), H), GUARD, dtype=np.uint16)
    ref = oracle.balance(L, 4, 1, 1)
    oracle.pack_composed(wl.token_tag_np(np.arange(T), H), want, shorter, np.zeros(len(L), np.int32), ref, ref)
    assert np.array_equal(bits(big), want)
    # an encoder assignment whose balance failed
    _, easg = run_balance(L, 3, 1, 1, dev)
    easg.dev_status.fill_(-5)
    assert refused(tokens, buf, Ld, zero, easg, asg)
    # and the same call goes through once the data is consistent
    easg.dev_status.zero_()
    orch.pack_composed(orch.pack(tokens, Ld, easg), buf, Ld, zero, easg, asg)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == 0
    assert np.array_equal(bits(buf), oracle.pack(wl.token_tag_np(np.arange(T), H), L, oracle.balance(L, 4, 1, 1)))


def composed_row_map(sub, sub_off_m, eref, mref, T):
    """dst row -> encoder-buffer row of one modality (-1 where another modality lives), by running
    the oracle on rows that carry their own index."""
    n_rows = int(sub.sum())
    idx = np.arange(n_rows, dtype=np.int64).view(np.uint16).reshape(n_rows, 4)
    out = np.full((T, 4), 0xFFFF, dtype=np.uint16)
    oracle.pack_composed(idx, out, sub, sub_off_m, eref, mref)
    return out.view(np.int64).reshape(T)


def test_c4_full_size_every_row(gpu_device):
    """The whole C4 batch in the launch shape the bench times: three modalities (about 31 GB each)
    in their encoders' packed order, composed into the 92 GB LLM batch; every packed row is
    compared, on the device, with the oracle's composed row map."""
    dev = gpu_device
    w = wl.WORKLOADS[4]
    L = wl.draw_lengths(w)
    T = int(L.sum())
    free, _ = torch.cuda.mem_get_info()
    if free < 2 * T * w.H * 2 + (8 << 30):
        pytest.skip("not enough free HBM for the full C4 composition")
    split = wl.draw_modality_split(w, L)
    sub_off = wl.draw_interleave_offsets(split, 4)
    mref = oracle.balance(L, w.D, w.a, w.b)
    _, masg = run_balance(L, w.D, w.a, w.b, dev)
    packed = torch.full((T, w.H), GUARD, dtype=torch.int16, device=dev)
    enc = {0: (None, None), 1: (32, (1, 6144)), 2: (32, (1, 7680))}
    rmaps = []
    for m in range(3):
        sub = np.ascontiguousarray(split[:, m])
        n_rows = int(sub.sum())
        De, ph = enc[m]
        eref = easg = None
        if De is not None:
            eref = oracle.balance(sub, De, *ph)
            _, easg = run_balance(sub, De, *ph, dev)
        # the encoder buffer's row r carries tag(m * SALT + r): its own position
        rows_d = wl.token_tag_torch(m * SALT, m * SALT + n_rows, w.H, dev)
        orch.pack_composed(rows_d, packed, to_dev(sub, dev), to_dev(sub_off[:, m], dev), easg, masg)
        torch.cuda.synchronize()
        del rows_d
        rmaps.append(composed_row_map(sub, sub_off[:, m], eref, mref, T))
    assert int(masg.dev_status.item()) == 0
    rm = np.stack(rmaps)  # [3, T]
    assert ((rm >= 0).sum(axis=0) == 1).all()  # every row belongs to exactly one modality
    mod = np.argmax(rm >= 0, axis=0)
    src = rm[mod, np.arange(T)] + mod.astype(np.int64) * SALT
    # every packed row, on the device, against the tag of the source row the oracle places there
    srcd = torch.from_numpy(np.ascontiguousarray(src)).to(dev)
    step = (1 << 29) // (2 * w.H)
    for r0 in range(0, T, step):
        r1 = min(T, r0 + step)
        want = wl.token_tag_rows_torch(srcd[r0:r1], w.H)
        assert torch.equal(packed[r0:r1], want), "rows [%d, %d)" % (r0, r1)
        del want
    del packed
    torch.cuda.empty_cache()


# ----------------------------------------------------------------------------
# several sub-sequences per example and modality (Sec. 6, subsequence assembly)
# ----------------------------------------------------------------------------
def compose_pieces_all(L, split, lay, Dm, phase_m, enc, H, dev, lo=0, hi=None, pad=64):
    hi = Dm if hi is None else hi
    mref = oracle.balance(L, Dm, *phase_m)
    _, masg = run_balance(L, Dm, *phase_m, dev)
    rows = int(mref.tok_off[hi] - mref.tok_off[lo])
    buf = torch.full((rows + 2 * pad, H), GUARD, dtype=torch.int16, device=dev)
    out = buf[pad: pad + rows]
    want = np.full((rows, H), GUARD, dtype=np.uint16)
    for m in range(3):
        sub = np.ascontiguousarray(split[:, m])
        pp, po, pl = lay[m]
        De, phase_e = enc[m]
        rows_m, eref, easg = encoder_side(sub, De, phase_e, m, H, dev)
        oracle.pack_composed_pieces(rows_m, want, pp, po, pl, eref, mref, lo, hi)
        src_d = host_rows(rows_m, dev)
        before = src_d.clone()
        orch.pack_composed_pieces(src_d, out, to_dev(pp, dev), to_dev(po, dev), to_dev(pl, dev), easg, masg, lo, hi)
        torch.cuda.synchronize()
        assert torch.equal(src_d, before)
    assert int(masg.dev_status.item()) == 0
    guards = bool((buf[:pad] == GUARD).all()) and bool((buf[pad + rows:] == GUARD).all())
    return out, guards, want, mref, masg


@pytest.mark.parametrize("cid,shrink,keep,H,max_pieces", [(4, 4, 1500, 64, 4), (4, 1, 300, 256, 3), (1, 1, None, 24, 4),
                                                          (3, 1, None, 40, 2)])
def test_pieces_three_modalities(gpu_device, cid, shrink, keep, H, max_pieces):
    w = wl.WORKLOADS[cid]
    L = wl.draw_lengths(w)
    if keep is not None:
        L = L[:keep]
    L = (L // shrink).astype(np.int32)
    split = wl.draw_modality_split(w, L)
    lay = wl.draw_piece_layout(split, 40 + cid, max_pieces)
    enc = {0: (None, None), 1: (max(2, w.D // 2), (1, 6144)), 2: (w.D, (1, 7680))}
    out, guards, want, mref, _ = compose_pieces_all(L, split, lay, w.D, (w.a, w.b), enc, H, gpu_device)
    assert guards
    assert np.array_equal(bits(out), want)
    assert not (want == GUARD).all(axis=1).any()  # the three modalities' pieces cover every row
    # an instance sub-range
    lo, hi = 1, max(2, w.D // 2)
    out2, guards2, want2, _, _ = compose_pieces_all(L, split, lay, w.D, (w.a, w.b), enc, H, gpu_device, lo, hi)
    assert guards2 and np.array_equal(bits(out2), want2)


def test_pieces_one_per_example_equals_pack_composed(gpu_device):
    dev = gpu_device
    w = wl.WORKLOADS[4]
    L = (wl.draw_lengths(w)[:800] // 4).astype(np.int32)
    split = wl.draw_modality_split(w, L)
    sub_off = wl.draw_interleave_offsets(split, 4)
    H = 128
    Ld, masg = run_balance(L, w.D, w.a, w.b, dev)
    T = int(L.sum())
    for m in (1, 2):
        sub = np.ascontiguousarray(split[:, m])
        rows_m, _, easg = encoder_side(sub, 8, (1, 5), m, H, dev)
        src_d = host_rows(rows_m, dev)
        a = torch.full((T, H), GUARD, dtype=torch.int16, device=dev)
        b = a.clone()
        orch.pack_composed(src_d, a, to_dev(sub, dev), to_dev(sub_off[:, m], dev), easg, masg)
        pp = np.arange(len(L) + 1, dtype=np.int32)
        orch.pack_composed_pieces(src_d, b, to_dev(pp, dev), to_dev(sub_off[:, m], dev), to_dev(sub, dev), easg, masg)
        torch.cuda.synchronize()
        assert int(masg.dev_status.item()) == 0 and torch.equal(a, b)


def test_pieces_refused_on_device(gpu_device):
    dev = gpu_device
    L = np.array([10, 6, 8], dtype=np.int32)
    _, asg = run_balance(L, 2, 0, 1, dev)
    rows = host_rows(wl.token_tag_np(np.arange(12), 8), dev)
    pp = to_dev(np.array([0, 2, 3, 4], np.int32), dev)
    good = (np.array([0, 5, 1, 2], np.int32), np.array([3, 5, 2, 2], np.int32))
    out = torch.full((24, 8), GUARD, dtype=torch.int16, device=dev)
    orch.pack_composed_pieces(rows, out, pp, to_dev(good[0], dev), to_dev(good[1], dev), None, asg)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == 0 and int((out != GUARD).all(dim=1).sum().item()) == 12
    bad_cases = [([0, 2, 1, 2], [3, 5, 2, 2], pp),          # overlap inside an example
                 ([5, 0, 1, 2], [5, 3, 2, 2], pp),          # descending pieces
                 ([0, 6, 1, 2], [3, 5, 2, 2], pp),          # past the end of the sequence
                 ([0, 5, 1, -1], [3, 5, 2, 2], pp),         # negative offset
                 ([0, 5, 1, 2], [3, -5, 2, 2], pp),         # negative length
                 ([0, 5, 1, 2], [3, 5, 2, 2], to_dev(np.array([0, 3, 2, 4], np.int32), dev)),   # piece_ptr not monotone
                 ([0, 5, 1, 2], [3, 5, 2, 2], to_dev(np.array([0, 2, 3, 3], np.int32), dev))]   # piece_ptr[n] != n_pieces
    for off, ln, ptr in bad_cases:
        asg.dev_status.zero_()
        out.fill_(GUARD)
        orch.pack_composed_pieces(rows, out, ptr, to_dev(np.array(off, np.int32), dev), to_dev(np.array(ln, np.int32), dev),
                                  None, asg)
        torch.cuda.synchronize()
        assert int(asg.dev_status.item()) == -5, (off, ln)
        assert bool((out == GUARD).all())
    # no pieces at all: nothing is written, no error
    asg.dev_status.zero_()
    empty = torch.zeros(0, dtype=torch.int32, device=dev)
    orch.pack_composed_pieces(rows[:0], out, to_dev(np.zeros(4, np.int32), dev), empty, empty, None, asg)
    torch.cuda.synchronize()
    assert int(asg.dev_status.item()) == 0 and bool((out == GUARD).all())
