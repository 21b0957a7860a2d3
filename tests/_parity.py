"""Helpers for the GPU parity tests: run the oracle on the same seeded tensors and
measure the errors the tolerances are stated in."""
import numpy as np
import torch

import oracle

# Tolerances:
#   bf16 inputs, fp32 accumulation: max-abs error on out <= 1e-2, relative L2 error on
#   dq/dk/dv <= 2e-2; fp32 debug build: <= 1e-5 for all of them.
#   lse is fp32 on both builds: 1e-4 on the bf16 build (measured <= 4e-6; a key dropped or added among several
#   thousand moves it by about 1e-4).
TOL_OUT_BF16 = 1e-2
TOL_LSE_BF16 = 1e-4
TOL_GRAD_BF16 = 2e-2
TOL_F32 = 1e-5


def out_bound(want) -> np.ndarray:
    """The one bound used for bf16 `out` wherever an output can leave the range of an average of many values
    (full-size samples, rows or caches of a few keys): 1e-2 as stated where |out| < 2; from |out| >= 2 on the
    rounding of the *stored* bf16 result alone -- half an ulp, 2^(e-8) for |out| in [2^e, 2^(e+1)), i.e. 7.8e-3 in
    [2, 4) -- is allowed on top, since it is not an error of the arithmetic being checked."""
    w = np.abs(np.asarray(want, dtype=np.float64))
    half_ulp = np.where(w >= 2.0, 2.0 ** (np.floor(np.log2(np.maximum(w, 1e-30))) - 8), 0.0)
    return TOL_OUT_BF16 + half_ulp


def out_ok(got, want) -> bool:
    return bool((np.abs(np.asarray(got, dtype=np.float64) - np.asarray(want, dtype=np.float64)) <= out_bound(want)).all())


def to_np(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a (bf16 or fp32) tensor to float64 on the host."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def max_abs(a, b) -> float:
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)))) if np.size(a) else 0.0


def rel_l2(a, b) -> float:
    """||a - b|| / ||b|| with b the oracle."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = float(np.linalg.norm(b))
    num = float(np.linalg.norm(a - b))
    return num / den if den > 0 else num


def tile_rel_l2(got, want, T=128) -> np.ndarray:
    """Relative L2 error of every block of T consecutive rows (the last one may be shorter)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    n = want.shape[0]
    edges = np.arange(0, n, T)
    num = np.sqrt(np.add.reduceat(((got - want) ** 2).sum(axis=1), edges))
    den = np.sqrt(np.add.reduceat((want ** 2).sum(axis=1), edges))
    return num / np.maximum(den, 1e-300)


def check_kv_group(tag, q, k, v, dout, res, b, g, r, W, gist_period=None):
    """One whole kv group (batch b, kv head g and its query heads) of a bf16 run against the dense oracle, element
    by element: out to the common bound, lse to TOL_LSE_BF16, dq per 128-row tile, dk and dv per 128-key tile and
    every gist column on its own to TOL_GRAD_BF16 (relative L2).  q, k, v, dout and res = (out, lse, dq, dk, dv) are
    host tensors [B, H, L, D]."""
    from concurrent.futures import ThreadPoolExecutor
    out, lse, dq, dk, dv = res
    G = q.shape[1] // k.shape[1]
    L = q.shape[2]
    kn, vn = to_np(k[b, g]), to_np(v[b, g])

    def one(h):
        qn, don = to_np(q[b, h]), to_np(dout[b, h])
        o, l = oracle.attn_fwd_head(qn, kn, vn, r, W)
        gq, gk, gv = oracle.attn_bwd_head(qn, kn, vn, don, r, W)
        return o, l, gq, gk, gv

    with ThreadPoolExecutor(max_workers=G) as ex:  # one head per thread; numpy releases the GIL inside BLAS
        want = list(ex.map(one, range(g * G, (g + 1) * G)))
    worst = {}
    for n, h in enumerate(range(g * G, (g + 1) * G)):
        o, l, gq, _, _ = want[n]
        got_o = to_np(out[b, h])
        eo, el, eq = max_abs(got_o, o), max_abs(to_np(lse[b, h]), l), tile_rel_l2(to_np(dq[b, h]), gq)
        print(f"{tag} b{b} h{h}: out {eo:.3e} lse {el:.3e} dq worst tile {eq.max():.3e} (tile {int(eq.argmax())})", flush=True)
        assert out_ok(got_o, o), (tag, b, h)
        assert el <= TOL_LSE_BF16, (tag, b, h, el)
        assert eq.max() <= TOL_GRAD_BF16, (tag, b, h, int(eq.argmax()), float(eq.max()))
        worst = {"out": max(worst.get("out", 0.0), eo), "lse": max(worst.get("lse", 0.0), el),
                 "dq": max(worst.get("dq", 0.0), float(eq.max()))}
    gk = sum(x[3] for x in want)
    gv = sum(x[4] for x in want)
    ek, ev = tile_rel_l2(to_np(dk[b, g]), gk), tile_rel_l2(to_np(dv[b, g]), gv)
    print(f"{tag} b{b} kv{g}: dk worst tile {ek.max():.3e} (tile {int(ek.argmax())}), dv worst tile {ev.max():.3e} "
          f"(tile {int(ev.argmax())})", flush=True)
    assert ek.max() <= TOL_GRAD_BF16 and ev.max() <= TOL_GRAD_BF16, (tag, float(ek.max()), float(ev.max()))
    worst.update(dk=float(ek.max()), dv=float(ev.max()))
    gists = np.arange(r, L, r + 1)  # every gist column on its own (the early ones collect every segment's partial sums)
    if len(gists):
        ck = tile_rel_l2(to_np(dk[b, g])[gists], gk[gists], T=1)
        cv = tile_rel_l2(to_np(dv[b, g])[gists], gv[gists], T=1)
        print(f"{tag} b{b} kv{g}: gist columns dk worst {ck.max():.3e}, dv worst {cv.max():.3e}", flush=True)
        assert ck.max() <= TOL_GRAD_BF16 and cv.max() <= TOL_GRAD_BF16, (tag, float(ck.max()), float(cv.max()))
    return worst


def oracle_fwd_bwd(q, k, v, dout, r, W, **mask):
    qn, kn, vn, don = (to_np(t) for t in (q, k, v, dout))
    out, lse = oracle.attn_fwd(qn, kn, vn, r, W, **mask)
    dq, dk, dv = oracle.attn_bwd(qn, kn, vn, don, r, W, **mask)
    return out, lse, dq, dk, dv
