"""Parity on the remaining benchmark shapes at full size: the 128K-token training shape (r=8, W=2048),
the compression-ratio sweep (B=4, L=16384, r in {2,4,8,16,32}) and the compressed-cache decode
(64 sequences x 17 408 keys).  The oracle is evaluated on sampled outputs it can compute one by one
(rows of out/lse/dq, columns of dk/dv with a bounded span of visible rows); whole-tensor identities
cover the rest."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth
from _parity import TOL_GRAD_BF16, TOL_LSE_BF16, TOL_OUT_BF16, check_kv_group, max_abs, out_ok, rel_l2, to_np

pytestmark = pytest.mark.gpu


def sampled_check(q, k, v, dout, res, B, Hq, Hkv, L, r, W, heads, rows, raw_cols, gist_cols, tag):
    """res = (out, lse, dq, dk, dv) on the host; heads = [(b, h)], raw_cols / gist_cols for kv head of heads[0]."""
    out, lse, dq, dk, dv = res
    G = Hq // Hkv
    for b, h in heads:
        g = h // G
        qn, kn, vn, don = to_np(q[b, h]), to_np(k[b, g]), to_np(v[b, g]), to_np(dout[b, h])
        o, l = oracle.attn_fwd_rows(qn, kn, vn, rows, r, W)
        gq = oracle.attn_dq_rows(qn, kn, vn, don, rows, r, W)
        assert out_ok(to_np(out[b, h])[rows], o), (tag, b, h)
        assert max_abs(to_np(lse[b, h])[rows], l) <= TOL_LSE_BF16, (tag, b, h)
        e = rel_l2(to_np(dq[b, h])[rows], gq)
        print(f"{tag} b{b} h{h}: out {max_abs(to_np(out[b, h])[rows], o):.3e} dq {e:.3e}", flush=True)
        assert e <= TOL_GRAD_BF16, (tag, b, h, e)
    b, h0 = heads[0]
    g = h0 // G
    kn, vn = to_np(k[b, g]), to_np(v[b, g])
    for cols, lo, hi in ((raw_cols, min(raw_cols), min(L, max(raw_cols) + W)), (gist_cols, min(gist_cols), L)):
        dks = np.zeros((len(cols), kn.shape[1]))
        dvs = np.zeros_like(dks)
        for h in range(g * G, (g + 1) * G):
            a, c = oracle.attn_dkdv_cols(to_np(q[b, h]), kn, vn, to_np(dout[b, h]), cols, r, W, lo, hi)
            dks += a
            dvs += c
        for n, j in enumerate(cols):
            ek, ev = rel_l2(to_np(dk[b, g])[[j]], dks[[n]]), rel_l2(to_np(dv[b, g])[[j]], dvs[[n]])
            print(f"{tag} key {j}: dk {ek:.3e} dv {ev:.3e}", flush=True)
            assert ek <= TOL_GRAD_BF16 and ev <= TOL_GRAD_BF16, (tag, j, ek, ev)


def identities(dout, dk, dv, Hkv, L):
    G = dout.shape[1] // Hkv
    for b in range(dout.shape[0]):
        s_dv = dv[b].double().sum(dim=1)
        s_do = dout[b].double().reshape(Hkv, G, L, -1).sum(dim=(1, 2))
        assert (s_dv - s_do).abs().max().item() <= 0.05 * np.sqrt(L)
        scale = dk[b].double().abs().mean().item()
        assert dk[b].double().sum(dim=1).abs().max().item() <= 0.4 * np.sqrt(L) * max(scale, 1e-3)


def run(B, Hq, Hkv, L, D, r, W, seed):
    q, k, v, dout = synth.attn_inputs(B, Hq, Hkv, L, D, seed=seed, device="cuda")
    out, lse = u.attn_fwd(q, k, v, r, W)
    dq, dk, dv = u.attn_bwd(q, k, v, out, lse, dout, r, W)
    torch.cuda.synchronize()
    host = [t.cpu() for t in (q, k, v, dout, out, lse, dq, dk, dv)]
    for t in host[4:]:
        assert torch.isfinite(t.float()).all()
    return host


def test_long_context_128k():
    c = synth.WORKLOADS["cfg3_long_128k"]
    B, Hq, Hkv, L, D, r, W = (c[n] for n in ("B", "Hq", "Hkv", "L", "D", "r", "W"))
    print("case", c, flush=True)
    q, k, v, dout, *res = run(B, Hq, Hkv, L, D, r, W, seed=3)
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, W - 1, W, L - 1, L // 2], rng.integers(0, L, 12)]))
    raw = [j for j in (70000 + rng.integers(0, 300, 5)).tolist() if (j + 1) % (r + 1) != 0]
    gists = [L - 1 - ((L - 1 - 8) % 9) - 9 * t for t in (0, 30)]   # positions with (p + 1) % 9 == 0 near the end
    assert all((p + 1) % (r + 1) == 0 for p in gists)
    sampled_check(q, k, v, dout, res, B, Hq, Hkv, L, r, W, [(0, 9), (0, 30)], rows, raw, gists, "cfg3")
    identities(dout, res[3], res[4], Hkv, L)
    # a whole 128-key tile three quarters into the sequence (raw keys and gists; its gists are reached by the last
    # 32 768 rows, i.e. by 8 of the gist phase's 32 segments), kv head 6 with its four query heads
    from concurrent.futures import ThreadPoolExecutor
    g, G = 6, Hq // Hkv
    cols = np.arange(3 * L // 4, 3 * L // 4 + 128)
    kn, vn = to_np(k[0, g]), to_np(v[0, g])

    def one(h):
        return oracle.attn_dkdv_cols(to_np(q[0, h]), kn, vn, to_np(dout[0, h]), cols, r, W, int(cols[0]), L)

    with ThreadPoolExecutor(max_workers=G) as ex:
        parts = list(ex.map(one, range(g * G, (g + 1) * G)))
    gk, gv = sum(p[0] for p in parts), sum(p[1] for p in parts)
    dk, dv = to_np(res[3][0, g])[cols], to_np(res[4][0, g])[cols]
    ek = np.linalg.norm(dk - gk, axis=1) / np.linalg.norm(gk, axis=1)
    ev = np.linalg.norm(dv - gv, axis=1) / np.linalg.norm(gv, axis=1)
    print(f"cfg3 key tile at {int(cols[0])}: dk worst column {ek.max():.3e}, dv worst column {ev.max():.3e}", flush=True)
    assert ek.max() <= TOL_GRAD_BF16 and ev.max() <= TOL_GRAD_BF16


@pytest.mark.parametrize("r", synth.WORKLOADS["cfg4_ratio_sweep"]["r"])
def test_ratio_sweep(r):
    c = synth.WORKLOADS["cfg4_ratio_sweep"]
    B, Hq, Hkv, L, D, W = (c[n] for n in ("B", "Hq", "Hkv", "L", "D", "W"))
    print("case", c, "r =", r, flush=True)
    q, k, v, dout, *res = run(B, Hq, Hkv, L, D, r, W, seed=4 + r)
    rng = np.random.default_rng(r)
    rows = np.unique(np.concatenate([[0, W, L - 1], rng.integers(0, L, 10)]))
    raw = [j for j in (9000 + rng.integers(0, 200, 4)).tolist() if (j + 1) % (r + 1) != 0]
    last_gist = (L // (r + 1)) * (r + 1) - 1
    gists = [last_gist, last_gist - 40 * (r + 1)]
    sampled_check(q, k, v, dout, res, B, Hq, Hkv, L, r, W, [(3, 17), (1, 2)], rows, raw, gists, f"cfg4 r={r}")
    identities(dout, res[3], res[4], Hkv, L)
    # one whole kv group (a different batch entry and kv head for every r), every element
    check_kv_group(f"cfg4 r={r}", q, k, v, dout, res, r % B, (3 * r) % Hkv, r, W)


def test_decode_full_size():
    c = synth.WORKLOADS["cfg5_decode"]
    B, Hq, Hkv, Lk, D = (c[n] for n in ("B", "Hq", "Hkv", "Lk", "D"))
    print("case", c, flush=True)
    q, kc, vc = synth.decode_inputs(B, Hq, Hkv, Lk, D, seed=5, device="cuda")
    out, lse = u.decode(q, kc, vc)
    sl = synth.ragged_seqlens(B, Lk, seed=6).cuda()
    out2, lse2 = u.decode(q, kc, vc, sl)
    torch.cuda.synchronize()
    for b in (0, 1, 31, 63):   # every head of four sequences, full and ragged lengths
        qb, kb, vb = to_np(q[b:b + 1]), to_np(kc[b:b + 1]), to_np(vc[b:b + 1])
        o, l = oracle.decode(qb, kb, vb)
        assert max_abs(to_np(out[b:b + 1]), o) <= TOL_OUT_BF16 and max_abs(to_np(lse[b:b + 1]), l) <= TOL_LSE_BF16
        o, l = oracle.decode(qb, kb, vb, [int(sl[b])])
        assert max_abs(to_np(out2[b:b + 1]), o) <= TOL_OUT_BF16 and max_abs(to_np(lse2[b:b + 1]), l) <= TOL_LSE_BF16
    assert torch.isfinite(out.float()).all() and torch.isfinite(out2.float()).all()


def test_largest_supported_length_forward():
    # L = 2^23 positions per head, the most the entry points accept (one more is UNIGIST_EUNSUPPORTED): the
    # kernels keep byte offsets inside a head in 32 bits, and here they come within one row of 2^30 * 2.  One head of
    # D = 64; rows at both ends and in the middle against the oracle (1.7 million visible keys for the last ones).
    L, D, r, W = 1 << 23, 64, 4, 1024
    g = torch.Generator(device="cuda").manual_seed(6)
    q, k, v = (torch.randn(1, 1, L, D, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16) for _ in range(3))
    out = torch.empty_like(q)
    lse = torch.empty(1, 1, L, device="cuda", dtype=torch.float32)
    st = torch.cuda.current_stream().cuda_stream
    assert u.unigist_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(), 1, 1, 1, L + 1, D, r, W,
                              u.UNIGIST_BF16, st) == 2
    assert u.unigist_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(), 1, 1, 1, L, D, r, W,
                              u.UNIGIST_BF16, st) == 0
    torch.cuda.synchronize()
    rows = np.array([0, 1, W, L // 2 + 3, L - 129, L - 2, L - 1])
    qn, kn, vn = to_np(q[0, 0].cpu()), to_np(k[0, 0].cpu()), to_np(v[0, 0].cpu())
    o, l = oracle.attn_fwd_rows(qn, kn, vn, rows, r, W)
    assert out_ok(to_np(out[0, 0, rows].cpu()), o)
    assert max_abs(to_np(lse[0, 0, rows].cpu()), l) <= TOL_LSE_BF16


def test_one_million_positions_forward_and_backward():
    # 2^20 positions of one head (D = 64): 16384 query chunks, so the gist phase of dK/dV runs with segments of 512
    # chunks (never more than 32 segments per gist tile), 1639 gist tiles, a 3.4 GB workspace
    B, Hq, Hkv, L, D, r, W = 1, 1, 1, 1 << 20, 64, 4, 1024
    q, k, v, dout, *res = run(B, Hq, Hkv, L, D, r, W, seed=8)
    rng = np.random.default_rng(8)
    rows = np.unique(np.concatenate([[0, W, L - 1, L // 2], rng.integers(0, L, 6)]))
    raw = [j for j in (700000 + rng.integers(0, 300, 4)).tolist() if (j + 1) % (r + 1) != 0]
    gists = [L - 1 - ((L - 5) % 5) - 5 * t for t in (0, 40)]       # positions with (p + 1) % 5 == 0 near the end
    assert all((p + 1) % (r + 1) == 0 for p in gists)
    sampled_check(q, k, v, dout, res, B, Hq, Hkv, L, r, W, [(0, 0)], rows, raw, gists, "1M")
    identities(dout, res[3], res[4], Hkv, L)
