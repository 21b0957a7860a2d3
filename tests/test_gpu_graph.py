"""The entry points allocate nothing, never synchronise and enqueue only kernels, so a caller can capture them
into a HIP graph.  Replays (with the program's own eager work and synchronisations between them) must reproduce
the eager results bit for bit."""
import pytest
import torch

import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth

pytestmark = pytest.mark.gpu


def _replay_equals_eager(make_inputs, run, n_replays=3):
    static = [t.cuda() for t in make_inputs(0)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(*static)                       # warm-up outside the capture (loads the library, creates helper streams)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        captured = run(*static)
    for n in range(1, n_replays + 1):
        for dst, src in zip(static, make_inputs(n)):
            dst.copy_(src)                 # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in captured]
        want = run(*static)
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {n}"


def test_forward_and_backward_in_a_graph():
    B, Hq, Hkv, L, D, r, W = 1, 4, 2, 1500, 128, 4, 100
    ws = torch.empty(u.unigist_attn_bwd_workspace(B, Hq, Hkv, L, D, r, W, u.UNIGIST_BF16), dtype=torch.uint8, device="cuda")

    def run(q, k, v, dout):
        out, lse = u.attn_fwd(q, k, v, r, W)
        dq, dk, dv = u.attn_bwd(q, k, v, out, lse, dout, r, W, workspace=ws)
        return out, lse, dq, dk, dv

    _replay_equals_eager(lambda n: synth.attn_inputs(B, Hq, Hkv, L, D, seed=70 + n), run)


def test_decode_in_a_graph():
    B, Hq, Hkv, Lk, D = 8, 8, 2, 3000, 128
    ws = torch.empty(u.unigist_decode_workspace(B, Hq, Hkv, Lk, D, u.UNIGIST_BF16), dtype=torch.uint8, device="cuda")
    ks, vs = synth.e4m3_scales(Hkv, seed=1, device="cuda")

    def run(q, kc, vc):
        out, lse = u.decode(q, kc, vc, workspace=ws)
        k8, v8 = u.quantize_e4m3(kc, ks), u.quantize_e4m3(vc, vs)
        out8, lse8 = u.decode_e4m3(q, k8, v8, ks, vs, workspace=ws)
        return out, lse, out8, lse8

    _replay_equals_eager(lambda n: synth.decode_inputs(B, Hq, Hkv, Lk, D, seed=80 + n), run)


def test_packed_backward_in_a_graph():
    # the packed backward forks onto the library's helper streams and joins them again: inside a capture the
    # helpers become branches of the same graph
    Hq, Hkv, D, r, W = 4, 2, 128, 4, 64
    lens = [700, 90, 1300, 257, 33, 410]
    cu = [0]
    for n in lens:
        cu.append(cu[-1] + n)
    T = cu[-1]
    ws = torch.empty(u.unigist_attn_bwd_varlen_workspace(Hq, Hkv, T, D, r, W, cu, u.UNIGIST_BF16), dtype=torch.uint8, device="cuda")

    def run(q, k, v, dout):
        out, lse = u.attn_fwd_varlen(q, k, v, r, W, cu)
        dq, dk, dv = u.attn_bwd_varlen(q, k, v, out, lse, dout, r, W, cu, workspace=ws)
        return out, lse, dq, dk, dv

    def inputs(n):
        return [t[0] for t in synth.attn_inputs(1, Hq, Hkv, T, D, seed=90 + n)]

    _replay_equals_eager(inputs, run)
