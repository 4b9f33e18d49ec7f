"""The library only enqueues work on the caller's stream: no allocation, no host synchronisation,
no fill through the runtime.  Checked by running the whole path on a side stream and by capturing
it into a HIP graph that is replayed on changed inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_23830_amd as orch
import workloads as wl
from gpu_common import assert_assignment_equal, attn_tolerance_check, bits

pytestmark = pytest.mark.gpu


class Path:
    """Static buffers for balance -> pack -> attention forward -> attention backward on one instance."""

    def __init__(self, L, D, a, b, H, Hq, Hkv, d, causal, dev, seed):
        self.L, self.D, self.a, self.b, self.causal = L, D, a, b, causal
        n, T = len(L), int(L.sum())
        self.Ld = torch.from_numpy(L).to(dev)
        self.asg = orch.Assignment.empty(n, D, dev)
        self.tokens = wl.token_tag_torch(0, T, H, dev)
        self.packed = torch.zeros_like(self.tokens)
        self.ws_bal = torch.empty(orch.balance_workspace(n, D), dtype=torch.uint8, device=dev)
        self.ws_pack = torch.empty(orch.pack_workspace(n, D), dtype=torch.uint8, device=dev)
        # attention over the whole batch as one instance's rows (D sequences lists, concatenated layout)
        ref = oracle.balance(L, D, a, b)
        self.i = int(np.argmax(ref.loads))
        self.cu = np.ascontiguousarray(ref.cu_of(self.i))
        Ti, batch = int(self.cu[-1]), len(self.cu) - 1
        lo = int(ref.seq_off[self.i]) + self.i
        self.cu_view = self.asg.cu_seqlens[lo: lo + batch + 1]
        self.q = wl.normal_bf16_torch((Ti, Hq, d), seed, 1, dev)
        self.k = wl.normal_bf16_torch((Ti, Hkv, d), seed, 2, dev)
        self.v = wl.normal_bf16_torch((Ti, Hkv, d), seed, 3, dev)
        self.do = wl.normal_bf16_torch((Ti, Hq, d), seed, 4, dev)
        self.out = torch.zeros_like(self.q)
        self.lse = torch.zeros((Hq, Ti), dtype=torch.float32, device=dev)
        self.dq, self.dk, self.dv = torch.zeros_like(self.q), torch.zeros_like(self.k), torch.zeros_like(self.v)
        self.ws_attn = torch.empty(orch.varlen_attn_workspace(batch, Ti, Hq), dtype=torch.uint8, device=dev)
        self.ws_bwd = torch.empty(orch.varlen_attn_bwd_workspace(batch, Ti, Hq), dtype=torch.uint8, device=dev)
        self.ref = ref

    def run(self):
        orch.balance(self.Ld, self.D, self.a, self.b, out=self.asg, ws=self.ws_bal)
        orch.pack(self.tokens, self.Ld, self.asg, out=self.packed, ws=self.ws_pack)
        orch.varlen_attn_fwd(self.q, self.k, self.v, self.cu_view, self.causal, out=self.out, lse=self.lse,
                             ws=self.ws_attn)
        orch.varlen_attn_bwd(self.q, self.k, self.v, self.out, self.lse, self.do, self.cu_view, self.causal,
                             dq=self.dq, dk=self.dk, dv=self.dv, ws=self.ws_bwd)

    def snapshot(self):
        return [t.clone() for t in (self.packed, self.out, self.lse, self.dq, self.dk, self.dv)]

    def check_against_oracle(self):
        assert_assignment_equal(self.asg, self.ref)
        T, H = self.tokens.shape
        assert np.array_equal(bits(self.packed), oracle.pack(bits(self.tokens), self.L, self.ref))
        want = oracle.attn_fwd(bits(self.q), bits(self.k), bits(self.v), self.cu, self.causal, nthreads=8)
        attn_tolerance_check(self.out.float().cpu().numpy(), want)


def make_path(dev, seed=3):
    w = wl.WORKLOADS[1]
    return Path(wl.draw_lengths(w), w.D, w.a, w.b, 64, 4, 2, 128, True, dev, seed)


def test_side_stream(gpu_device):
    p = make_path(gpu_device)
    p.run()
    torch.cuda.synchronize()
    eager = p.snapshot()
    p.check_against_oracle()
    for t in (p.packed, p.out, p.lse, p.dq, p.dk, p.dv):
        t.zero_()
    side = torch.cuda.Stream(device=gpu_device)  # default priority
    side.wait_stream(torch.cuda.current_stream(gpu_device))
    with torch.cuda.stream(side):
        p.run()
    side.synchronize()
    for a, b in zip(eager, p.snapshot()):
        assert torch.equal(a, b)


def test_graph_capture_and_replay(gpu_device):
    """Capture the four calls once; replay on other token rows, q/k/v and dout (same shapes), with
    eager work and synchronisations between the replays; every replay must equal the eager run."""
    p = make_path(gpu_device)
    p.run()  # warm-up outside capture (module load)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    cap = torch.cuda.Stream(device=gpu_device)
    cap.wait_stream(torch.cuda.current_stream(gpu_device))
    with torch.cuda.stream(cap):
        with torch.cuda.graph(graph, stream=cap):
            p.run()
    torch.cuda.synchronize()
    for rep in range(3):
        seed = 20 + rep
        p.tokens.copy_(wl.token_tag_torch(1000 * rep, 1000 * rep + p.tokens.shape[0], p.tokens.shape[1], gpu_device))
        for t, stream_id in ((p.q, 1), (p.k, 2), (p.v, 3), (p.do, 4)):
            t.copy_(wl.normal_bf16_torch(tuple(t.shape), seed, stream_id, gpu_device))
        for t in (p.packed, p.out, p.lse, p.dq, p.dk, p.dv):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        replayed = p.snapshot()
        p.check_against_oracle()
        for t in (p.packed, p.out, p.lse, p.dq, p.dk, p.dv):
            t.zero_()
        p.run()
        torch.cuda.synchronize()
        for a, b in zip(replayed, p.snapshot()):
            assert torch.equal(a, b)
