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
        run(*static)                       # warm-up outside the capture (loads the library)
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
    # the bf16 packed backward is one launch of each kernel over a document table that travels as a kernel argument:
    # the table is baked into the captured launches, so the replays must reproduce the eager result bit for bit
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


def test_decoding_steps_in_a_graph():
    # A decoding step (append the token's K/V to the ring cache, advance the positions, decode) changes state, so the
    # captured step is replayed to advance one cache while an identical cache is advanced eagerly: every step's
    # outputs and the caches must stay identical.  One sequence sits out every third step.
    B, Hq, Hkv, D, r, W, n0, steps = 3, 8, 2, 128, 4, 32, 50, 9
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, n0 + steps, D, seed=77)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()

    def fresh_ring():
        rag = u.RaggedKVCache(B, Hkv, n0 + steps + 8, D, r)
        for b in range(B):
            rag.update(b, kd[b, :, :n0].contiguous(), vd[b, :, :n0].contiguous(), max(0, n0 - W))
        rag.gathered()
        return u.RingKVCache(rag, W)

    ring_g, ring_e, ring_w = fresh_ring(), fresh_ring(), fresh_ring()
    kn, vn = torch.empty(B, Hkv, 1, D, dtype=torch.bfloat16, device="cuda"), torch.empty(B, Hkv, 1, D, dtype=torch.bfloat16, device="cuda")
    qt = torch.empty(B, Hq, D, dtype=torch.bfloat16, device="cuda")
    act = torch.ones(B, dtype=torch.int32, device="cuda")
    ws = torch.empty(u.unigist_decode_workspace(B, Hq, Hkv, ring_g.cap, D, u.UNIGIST_BF16), dtype=torch.uint8, device="cuda")

    def step(ring):
        rows = ring.append(kn, vn, act)
        out, lse = u.decode(qt, ring.kc, ring.vc, rows, workspace=ws)
        return out, lse, rows

    def feed(n):
        t = ring_e.t.cpu().tolist()           # the eager cache's positions (the captured one's are the same)
        a = [1, 1, 0 if n % 3 == 2 else 1]
        for b in range(B):
            kn[b] = kd[b, :, t[b] + 1:t[b] + 2]
            vn[b] = vd[b, :, t[b] + 1:t[b] + 2]
            qt[b] = qd[b, :, t[b] + a[b]]
        act.copy_(torch.tensor(a, dtype=torch.int32))

    feed(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(ring_w)                            # warm-up on a cache of its own
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        captured = step(ring_g)
    # the capture itself ran nothing: ring_g is still in its initial state
    for n in range(steps):
        feed(n)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in captured]
        want = step(ring_e)
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"step {n}"
        assert torch.equal(ring_g.t, ring_e.t), f"step {n}"
        for b_, nrows in enumerate(want[2].cpu().tolist()):   # the rows in use (what lies behind them was never written)
            assert torch.equal(ring_g.kc[b_, :, :nrows], ring_e.kc[b_, :, :nrows]), f"step {n}"
            assert torch.equal(ring_g.vc[b_, :, :nrows], ring_e.vc[b_, :, :nrows]), f"step {n}"
    assert ring_e.t.cpu().tolist() == [n0 - 1 + steps, n0 - 1 + steps, n0 - 1 + steps - 3]
