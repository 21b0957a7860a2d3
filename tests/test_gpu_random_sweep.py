"""Seeded sweep over small random configurations (lengths, ratios, windows, sinks, window modes, head layouts,
packed documents) through the MFMA kernels against the oracle: corner cases nobody thought of listing."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth
from _parity import TOL_GRAD_BF16, TOL_LSE_BF16, TOL_OUT_BF16, max_abs, out_ok, rel_l2, to_np

pytestmark = pytest.mark.gpu


PADDED_DIMS = (8, 24, 40, 56, 72, 96, 104, 120)  # run on the 64- and 128-wide kernels with the tail zeroed


def _configs(n, seed, dims=(64, 128)):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        D = int(rng.choice(dims))
        Hkv = int(rng.choice([1, 2, 3]))
        G = int(rng.choice([1, 2, 4]))
        L = int(rng.choice([1, 2, 31, 33, 64, 65, 127, 129, 200, 257, 300, 391]))
        r = int(rng.choice([1, 2, 3, 4, 7, 8, 16, 10**6]))
        units = bool(rng.integers(0, 2))
        W = int(rng.choice([1, 2, 3, 5, 8]) if units else rng.choice([1, 2, 5, 17, 32, 33, 64, 100, 128, 10**6]))
        sinks = int(rng.choice([0, 0, 1, 4, 31, 32, 33, 130]))
        out.append((Hkv * G, Hkv, L, D, r, W, sinks, units))
    return out


@pytest.mark.parametrize("chunk", range(6))
def test_random_layouts_match_oracle(chunk):
    cfgs = _configs(12, 100 + chunk) if chunk < 4 else _configs(12, 100 + chunk, PADDED_DIMS)
    for i, (Hq, Hkv, L, D, r, W, sinks, units) in enumerate(cfgs):
        case = f"#{chunk}.{i} Hq{Hq} Hkv{Hkv} L{L} D{D} r{r} W{W} sinks{sinks} units{int(units)}"
        print("case", case, flush=True)
        q, k, v, dout = synth.attn_inputs(1, Hq, Hkv, L, D, seed=1000 + 16 * chunk + i)
        qd, kd, vd, dod = (t.cuda() for t in (q, k, v, dout))
        out, lse = u.attn_fwd(qd, kd, vd, r, W, sinks=sinks, window_mode=int(units))
        dq, dk, dv = u.attn_bwd(qd, kd, vd, out, lse, dod, r, W, sinks=sinks, window_mode=int(units))
        torch.cuda.synchronize()
        qn, kn, vn, don = (to_np(t) for t in (q, k, v, dout))
        o, l = oracle.attn_fwd(qn, kn, vn, r, W, sinks=sinks, units=units)
        g = oracle.attn_bwd(qn, kn, vn, don, r, W, sinks=sinks, units=units)
        assert out_ok(to_np(out), o) and max_abs(to_np(lse), l) <= TOL_LSE_BF16, case
        for got, want in zip((dq, dk, dv), g):
            # a handful of tokens: dS = P (dP - delta) is a difference of nearly equal numbers and delta comes from
            # the bf16 `out`, so the error is bounded absolutely (entries are O(1)) rather than relative to a tiny norm
            if L <= 4:
                assert max_abs(to_np(got), want) <= 2e-2, case
            else:
                assert rel_l2(to_np(got), want) <= TOL_GRAD_BF16, case


@pytest.mark.parametrize("chunk", range(3))
def test_random_packs_match_oracle(chunk):
    rng = np.random.default_rng(200 + chunk)
    for i in range(8):
        D = int(rng.choice([64, 128] if chunk < 2 else PADDED_DIMS))
        Hkv, G = int(rng.choice([1, 2])), int(rng.choice([1, 4]))
        lens = [int(x) for x in rng.choice([0, 1, 5, 32, 33, 64, 100, 129, 200], size=int(rng.integers(1, 6)))]
        if sum(lens) == 0:
            lens.append(7)
        r, W = int(rng.choice([1, 2, 4, 8, 10**6])), int(rng.choice([1, 4, 33, 64, 10**6]))
        cu = [0] + np.cumsum(lens).tolist()
        case = f"#{chunk}.{i} Hq{Hkv * G} Hkv{Hkv} D{D} r{r} W{W} docs{lens}"
        print("case", case, flush=True)
        q, k, v, dout = (t[0] for t in synth.attn_inputs(1, Hkv * G, Hkv, cu[-1], D, seed=2000 + 16 * chunk + i))
        qd, kd, vd, dod = (t.cuda() for t in (q, k, v, dout))
        out, lse = u.attn_fwd_varlen(qd, kd, vd, r, W, cu)
        dq, dk, dv = u.attn_bwd_varlen(qd, kd, vd, out, lse, dod, r, W, cu)
        torch.cuda.synchronize()
        qn, kn, vn, don = (to_np(t)[None] for t in (q, k, v, dout))
        o, l = oracle.attn_fwd(qn, kn, vn, r, W, cu=cu)
        g = oracle.attn_bwd(qn, kn, vn, don, r, W, cu=cu)
        assert out_ok(to_np(out), o[0]) and max_abs(to_np(lse), l[0]) <= TOL_LSE_BF16, case
        for got, want in zip((dq, dk, dv), g):
            assert rel_l2(to_np(got), want[0]) <= TOL_GRAD_BF16, case
