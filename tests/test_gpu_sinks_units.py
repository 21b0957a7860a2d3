"""GPU parity of the *_ex entry points: the layout of Sec. 4.1 with a sink prefix (Eq. 2) and the local
window counted in gist units (the section's wording of Eq. 3), against the fp64 oracle on the same inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth
from _parity import max_abs, oracle_fwd_bwd, rel_l2, to_np
from test_gpu_attention import check
from _parity import out_ok

pytestmark = pytest.mark.gpu


def run_gpu(q, k, v, dout, r, W, sinks, units):
    qd, kd, vd, dod = (t.cuda() for t in (q, k, v, dout))
    out, lse = u.attn_fwd(qd, kd, vd, r, W, sinks=sinks, window_mode=int(units))
    dq, dk, dv = u.attn_bwd(qd, kd, vd, out, lse, dod, r, W, sinks=sinks, window_mode=int(units))
    torch.cuda.synchronize()
    return out, lse, dq, dk, dv


# B, Hq, Hkv, L, D, r, W, sinks, units      (units: W counts previous gist units)
SMALL = [
    (1, 1, 1, 1024, 64, 4, 128, 4, False),   # config 1 plus four sinks
    (1, 1, 1, 1024, 64, 4, 25, 0, True),     # config 1 with the window as 25 units (same span)
    (2, 4, 2, 333, 64, 4, 8, 7, True),       # GQA, ragged tail, sinks not a multiple of anything
    (1, 4, 1, 700, 128, 8, 11, 130, True),   # sinks longer than one 128-row tile
    (1, 2, 2, 257, 128, 2, 1, 1, True),      # a single previous unit
    (1, 2, 1, 384, 64, 4, 10**6, 3, True),   # window >= L: full causal behind the sinks
    (1, 2, 1, 300, 128, 2**31 - 2, 33, 5, True),   # no gists: one endless unit, causal
    (1, 2, 1, 300, 128, 2**31 - 2, 33, 5, False),  # no gists: sinks + sliding window
    (1, 2, 2, 63, 128, 1, 3, 2, True),       # r = 1
    (1, 2, 2, 90, 64, 4, 3, 500, True),      # more sinks than tokens: causal
    (1, 8, 8, 200, 64, 16, 2, 9, True),      # 8 kv heads
    (1, 4, 2, 700, 96, 4, 11, 130, True),    # head dimension 96
    (2, 2, 1, 333, 56, 4, 8, 7, True),       # ... and 56
]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("B,Hq,Hkv,L,D,r,W,sinks,units", SMALL)
def test_small_shapes_match_oracle(B, Hq, Hkv, L, D, r, W, sinks, units, dtype):
    case = f"B{B} Hq{Hq} Hkv{Hkv} L{L} D{D} r{r} W{W} sinks{sinks} units{int(units)} {dtype}"
    print("case", case, flush=True)
    q, k, v, dout = synth.attn_inputs(B, Hq, Hkv, L, D, dtype=dtype, seed=21)
    got = run_gpu(q, k, v, dout, r, W, sinks, units)
    check(case, got, oracle_fwd_bwd(q, k, v, dout, r, W, sinks=sinks, units=units), dtype)


# several 128-row tiles and compact tiles, more than one segment of query chunks (L > 4096)
MID = [
    (1, 2, 1, 9001, 64, 4, 60, 4, True),
    (1, 4, 1, 5000, 128, 2, 43, 0, True),
    (2, 4, 2, 4500, 128, 8, 113, 200, True),
    (1, 2, 1, 6000, 128, 4, 300, 129, False),
]


@pytest.mark.parametrize("B,Hq,Hkv,L,D,r,W,sinks,units", MID)
def test_mid_shapes_match_oracle(B, Hq, Hkv, L, D, r, W, sinks, units):
    case = f"B{B} Hq{Hq} Hkv{Hkv} L{L} D{D} r{r} W{W} sinks{sinks} units{int(units)} bf16"
    print("case", case, flush=True)
    q, k, v, dout = synth.attn_inputs(B, Hq, Hkv, L, D, seed=22)
    got = run_gpu(q, k, v, dout, r, W, sinks, units)
    check(case, got, oracle_fwd_bwd(q, k, v, dout, r, W, sinks=sinks, units=units), torch.bfloat16)


def test_zero_sinks_sliding_is_the_plain_entry_point():
    q, k, v, dout = synth.attn_inputs(1, 4, 2, 700, 128, seed=3)
    a = run_gpu(q, k, v, dout, 4, 64, 0, False)
    qd, kd, vd, dod = (t.cuda() for t in (q, k, v, dout))
    out, lse = u.attn_fwd(qd, kd, vd, 4, 64)
    b = (out, lse) + tuple(u.attn_bwd(qd, kd, vd, out, lse, dod, 4, 64))
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_zero_queries_count_the_visible_keys():
    # q = 0: lse_i = ln |visible keys of i|, counted by the oracle's predicate pair by pair
    B, Hq, Hkv, L, D, r, W, sinks = 1, 2, 1, 900, 128, 4, 6, 3
    _, k, v, _ = synth.attn_inputs(B, Hq, Hkv, L, D, seed=5)
    q = torch.zeros(B, Hq, L, D, dtype=torch.bfloat16)
    out, lse = u.attn_fwd(q.cuda(), k.cuda(), v.cuda(), r, W, sinks=sinks, window_mode=u.UNIGIST_WINDOW_UNITS)
    nvis = oracle.mask_rows(np.arange(L), L, r, W, sinks=sinks, units=True).sum(axis=1)
    assert max_abs(to_np(lse)[0, 0], np.log(nvis)) < 1e-5
    assert u.n_vis(L, r, W, sinks, u.UNIGIST_WINDOW_UNITS) == int(nvis.sum())


def test_full_length_sampled_rows_and_columns():
    # the 32K training shape with 4 sinks and the window as 204 units (about the same span as W = 1024):
    # sampled query rows (out, lse, dq) and sampled key columns (dk, dv) against the oracle
    w = synth.WORKLOADS["cfg2_llama8b_32k"]
    B, Hq, Hkv, L, D, r = w["B"], w["Hq"], w["Hkv"], w["L"], w["D"], w["r"]
    W, sinks = 204, 4
    q, k, v, dout = synth.attn_inputs(B, Hq, Hkv, L, D, seed=23)
    out, lse, dq, dk, dv = run_gpu(q, k, v, dout, r, W, sinks, True)
    rng = np.random.default_rng(0)
    rows = np.unique(np.concatenate([[0, 1, 3, 4, 5, 8, 1023, 1024, 1028, 1029, L - 1],
                                     rng.integers(0, L, 40)]))
    cols = np.unique(np.concatenate([[0, 3, 4, 8, 1028, L - 1, L - 2], rng.integers(0, L, 24)]))
    for h in (0, 13, 31):
        hk = h // (Hq // Hkv)
        qn, kn, vn, don = to_np(q[0, h]), to_np(k[0, hk]), to_np(v[0, hk]), to_np(dout[0, h])
        o, l = oracle.attn_fwd_rows(qn, kn, vn, rows, r, W, sinks=sinks, units=True)
        assert out_ok(to_np(out[0, h])[rows], o), h
        assert max_abs(to_np(lse[0, h])[rows], l) <= 1e-2
        g = oracle.attn_dq_rows(qn, kn, vn, don, rows, r, W, sinks=sinks, units=True)
        assert rel_l2(to_np(dq[0, h])[rows], g) <= 2e-2
    hk = 5
    G = Hq // Hkv
    qs, dos = to_np(q[0, hk * G:(hk + 1) * G]), to_np(dout[0, hk * G:(hk + 1) * G])
    gk = np.zeros((len(cols), D))
    gv = np.zeros((len(cols), D))
    for g in range(G):
        a, b = oracle.attn_dkdv_cols(qs[g], to_np(k[0, hk]), to_np(v[0, hk]), dos[g], cols, r, W, sinks=sinks,
                                     units=True)
        gk += a
        gv += b
    assert rel_l2(to_np(dk[0, hk])[cols], gk) <= 2e-2
    assert rel_l2(to_np(dv[0, hk])[cols], gv) <= 2e-2
