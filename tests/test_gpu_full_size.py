"""Parity at the benchmark's full size (32K tokens, GQA 32/8, D=128, r=4, W=1024), in the launch
configuration bench.py times.  One whole kv group (kv head 0 with its four query heads) is compared
with the dense fp64 oracle element by element: every row of out, lse and dq and every column of
dk and dv, gist 4 -- which every segment of the gist phase adds to -- included.  The other groups are
covered on sampled outputs the oracle can compute one by one -- rows of out/lse/dq (row-local) and
columns of dk/dv -- plus identities that hold at any size and involve every element."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth
from _parity import TOL_GRAD_BF16, TOL_LSE_BF16, check_kv_group, max_abs, out_ok, rel_l2, to_np

pytestmark = pytest.mark.gpu

CFG = synth.WORKLOADS["cfg2_llama8b_32k"]


@pytest.fixture(scope="module")
def full():
    B, Hq, Hkv, L, D, r, W = (CFG[n] for n in ("B", "Hq", "Hkv", "L", "D", "r", "W"))
    print("full-size case", CFG, flush=True)
    q, k, v, dout = synth.attn_inputs(B, Hq, Hkv, L, D, seed=0)
    qd, kd, vd, dod = (t.cuda() for t in (q, k, v, dout))
    out, lse = u.attn_fwd(qd, kd, vd, r, W)
    dq, dk, dv = u.attn_bwd(qd, kd, vd, out, lse, dod, r, W)
    torch.cuda.synchronize()
    return dict(q=q, k=k, v=v, dout=dout, out=out.cpu(), lse=lse.cpu(), dq=dq.cpu(), dk=dk.cpu(), dv=dv.cpu())


def test_one_kv_group_element_by_element(full):
    """kv head 0 and query heads 0-3 against the oracle over all 32768 rows: out to the common bound, lse to 1e-4,
    dq per 128-row tile and dk, dv per 128-key tile to 2e-2 relative L2 (per tile, so that an error confined to one
    tile of raw keys cannot hide behind the norm of the gist columns), and every gist column on its own."""
    res = tuple(full[n] for n in ("out", "lse", "dq", "dk", "dv"))
    check_kv_group("cfg2", full["q"], full["k"], full["v"], full["dout"], res, 0, 0, CFG["r"], CFG["W"])


def test_sampled_rows(full):
    L, r, W, G = CFG["L"], CFG["r"], CFG["W"], CFG["Hq"] // CFG["Hkv"]
    rng = np.random.default_rng(0)
    rows = np.unique(np.concatenate([[0, 1, 4, W - 1, W, W + 1, 127, 128, L - 1, L - 2, L // 2],
                                     rng.integers(0, L, 40)]))
    for h in (5, 18, 31):
        g = h // G
        q, k, v, do = (to_np(full[n][0, i]) for n, i in (("q", h), ("k", g), ("v", g), ("dout", h)))
        o, l = oracle.attn_fwd_rows(q, k, v, rows, r, W)
        dq = oracle.attn_dq_rows(q, k, v, do, rows, r, W)
        got_o = to_np(full["out"][0, h])[rows]
        assert out_ok(got_o, o), h
        assert max_abs(to_np(full["lse"][0, h])[rows], l) <= TOL_LSE_BF16
        e = rel_l2(to_np(full["dq"][0, h])[rows], dq)
        print(f"head {h}: out {max_abs(got_o, o):.3e} dq {e:.3e}", flush=True)
        assert e <= TOL_GRAD_BF16


def test_sampled_key_columns(full):
    L, r, W, G = CFG["L"], CFG["r"], CFG["W"], CFG["Hq"] // CFG["Hkv"]
    g = 3
    rng = np.random.default_rng(1)
    # raw keys in three clusters (each cluster shares one span of rows that can see it)
    clusters = []
    for base in (0, 12000, L - 600):
        js = sorted({int(j) for j in base + rng.integers(0, 500, 6) if (j + 1) % (r + 1) != 0} | {base + 1})
        clusters.append([j for j in js if j < L and (j + 1) % (r + 1) != 0])
    clusters[-1].append(L - 1)
    late_gists = [L - 4 - 5 * t for t in (0, 1, 100, 400)]        # positions with (p+1) % 5 == 0
    assert all((p + 1) % (r + 1) == 0 for p in late_gists)
    mid_gist = [24574]                                             # seen by the last 8 194 rows
    assert (mid_gist[0] + 1) % (r + 1) == 0
    k, v = to_np(full["k"][0, g]), to_np(full["v"][0, g])

    def group_sum(cols, row_lo, row_hi):
        def one(h):
            return oracle.attn_dkdv_cols(to_np(full["q"][0, h]), k, v, to_np(full["dout"][0, h]), cols, r, W,
                                         row_lo, row_hi)
        with ThreadPoolExecutor(max_workers=G) as ex:  # one head per thread; numpy releases the GIL
            parts = list(ex.map(one, range(g * G, (g + 1) * G)))
        return sum(p[0] for p in parts), sum(p[1] for p in parts)

    got_dk, got_dv = to_np(full["dk"][0, g]), to_np(full["dv"][0, g])
    # raw keys: only rows j .. j+W-1 can see them
    for js in clusters:
        dk, dv = group_sum(js, min(js), min(L, max(js) + W))
        for n, j in enumerate(js):
            ek, ev = rel_l2(got_dk[[j]], dk[[n]]), rel_l2(got_dv[[j]], dv[[n]])
            assert ek <= TOL_GRAD_BF16 and ev <= TOL_GRAD_BF16, (j, ek, ev)
    # gists: every later row sees them
    cols = late_gists + mid_gist
    dk, dv = group_sum(cols, min(cols), L)
    for n, j in enumerate(cols):
        ek, ev = rel_l2(got_dk[[j]], dk[[n]]), rel_l2(got_dv[[j]], dv[[n]])
        print(f"gist {j}: dk {ek:.3e} dv {ev:.3e}", flush=True)
        assert ek <= TOL_GRAD_BF16 and ev <= TOL_GRAD_BF16, j


def test_identities_over_every_element(full):
    """Rows of P sum to one, hence sum_j dV_j = sum_i dO_i over the heads of the group; and
    sum_j dS_ij = 0 for every row, hence sum_j dK_j = 0.  Both involve every key, early gists included."""
    G = CFG["Hq"] // CFG["Hkv"]
    dv = full["dv"][0].double().sum(dim=1)                                   # [Hkv, D]
    do = full["dout"][0].double().reshape(CFG["Hkv"], G, CFG["L"], -1).sum(dim=(1, 2))
    dk = full["dk"][0].double()
    # dv entries are O(1) with bf16 rounding 2^-9 relative; the sum of L of them is accurate to ~sqrt(L) * 2^-9
    assert (dv - do).abs().max().item() <= 0.05 * np.sqrt(CFG["L"])
    scale = dk.abs().mean().item()
    assert dk.sum(dim=1).abs().max().item() <= 0.05 * np.sqrt(CFG["L"]) * max(scale, 1e-3) * 8
    assert torch.isfinite(full["out"].float()).all() and torch.isfinite(full["dq"].float()).all()
    assert torch.isfinite(full["dk"].float()).all() and torch.isfinite(full["dv"].float()).all()
