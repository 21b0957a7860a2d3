"""GPU parity: unigist_attn_fwd / unigist_attn_bwd (through the C ABI) against the fp64 oracle,
element by element, on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth
from _parity import (TOL_F32, TOL_GRAD_BF16, TOL_LSE_BF16, TOL_OUT_BF16, max_abs, oracle_fwd_bwd, rel_l2, to_np)

pytestmark = pytest.mark.gpu


def run_gpu(q, k, v, dout, r, W):
    qd, kd, vd, dod = (t.cuda() for t in (q, k, v, dout))
    out, lse = u.attn_fwd(qd, kd, vd, r, W)
    dq, dk, dv = u.attn_bwd(qd, kd, vd, out, lse, dod, r, W)
    torch.cuda.synchronize()
    return out, lse, dq, dk, dv


def check(case, got, want, dtype, tol_f32=TOL_F32, tol_lse=TOL_LSE_BF16):
    out, lse, dq, dk, dv = got
    o_o, o_l, o_dq, o_dk, o_dv = want
    errs = dict(out=max_abs(to_np(out), o_o), lse=max_abs(to_np(lse), o_l), dq=rel_l2(to_np(dq), o_dq),
                dk=rel_l2(to_np(dk), o_dk), dv=rel_l2(to_np(dv), o_dv))
    print(case, {k: f"{v:.3e}" for k, v in errs.items()}, flush=True)
    for t in (out, lse, dq, dk, dv):
        assert torch.isfinite(t.float()).all(), case
    if dtype == torch.float32:
        assert errs["out"] <= tol_f32 and errs["lse"] <= tol_f32, (case, errs)
        assert max(errs["dq"], errs["dk"], errs["dv"]) <= tol_f32, (case, errs)
    else:
        assert errs["out"] <= TOL_OUT_BF16 and errs["lse"] <= tol_lse, (case, errs)
        assert max(errs["dq"], errs["dk"], errs["dv"]) <= TOL_GRAD_BF16, (case, errs)


# B, Hq, Hkv, L, D, r, W
SMALL = [
    (1, 1, 1, 1024, 64, 4, 128),      # config 1
    (2, 4, 2, 333, 64, 4, 40),        # GQA, ragged tail, several tiles
    (1, 4, 1, 700, 128, 8, 100),      # D = 128, group of 4
    (1, 2, 2, 257, 128, 2, 1),        # W = 1: only self + gists
    (1, 2, 1, 384, 64, 4, 10**6),     # window >= L: full causal
    (1, 2, 1, 300, 128, 2**31 - 2, 33),  # no gists: sliding window
    (1, 1, 1, 1, 64, 4, 4),           # a single token
    (1, 2, 2, 63, 128, 1, 3),         # r = 1: every other token is a gist
    (1, 8, 8, 200, 64, 16, 64),       # 8 kv heads: XCD-aware block order
    # head dimensions other than the two the matrix-core kernels are built for (run on the next one, zero-padded)
    (1, 4, 2, 700, 96, 4, 100),
    (2, 2, 1, 333, 80, 2, 40),
    (1, 4, 4, 257, 32, 8, 64),
    (1, 2, 1, 300, 120, 4, 33),
    (1, 2, 2, 200, 8, 4, 16),
]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("B,Hq,Hkv,L,D,r,W", SMALL)
def test_small_shapes_match_oracle(B, Hq, Hkv, L, D, r, W, dtype):
    case = f"B{B} Hq{Hq} Hkv{Hkv} L{L} D{D} r{r} W{W} {dtype}"
    print("case", case, flush=True)
    q, k, v, dout = synth.attn_inputs(B, Hq, Hkv, L, D, dtype=dtype, seed=0)
    got = run_gpu(q, k, v, dout, r, W)
    check(case, got, oracle_fwd_bwd(q, k, v, dout, r, W), dtype)


# mid sizes: several 128-row tiles, many compact gist tiles, more than one segment of query
# chunks in the gist phase of dK/dV (L > 4096), ragged tails in L, in the gist list and in W
MID = [
    (1, 2, 1, 9001, 64, 4, 300),
    (1, 4, 1, 5000, 128, 2, 129),
    (2, 4, 2, 4500, 128, 8, 1024),
    # 8 kv heads (the workgroup order that deals (batch, kv head) pairs to the 8 XCDs) together with a gist phase of
    # several tiles and several segments, and with a group of two query heads
    (1, 8, 8, 5000, 128, 4, 129),
    (1, 16, 8, 9001, 128, 4, 300),
    (2, 8, 4, 6000, 64, 2, 200),
    (1, 8, 8, 5000, 96, 4, 129),
    (1, 4, 2, 4200, 48, 8, 500),
]


@pytest.mark.parametrize("B,Hq,Hkv,L,D,r,W", MID)
def test_mid_shapes_match_oracle(B, Hq, Hkv, L, D, r, W):
    case = f"B{B} Hq{Hq} Hkv{Hkv} L{L} D{D} r{r} W{W} bf16"
    print("case", case, flush=True)
    q, k, v, dout = synth.attn_inputs(B, Hq, Hkv, L, D, seed=11)
    got = run_gpu(q, k, v, dout, r, W)
    check(case, got, oracle_fwd_bwd(q, k, v, dout, r, W), torch.bfloat16)


def test_plain_alu_and_mfma_kernels_agree():
    # the two independent GPU implementations on a shape the oracle would need minutes for
    B, Hq, Hkv, L, D, r, W = 1, 8, 2, 20000, 128, 4, 1024
    q, k, v, dout = synth.attn_inputs(B, Hq, Hkv, L, D, seed=12)
    a = run_gpu(q, k, v, dout, r, W)
    assert u.unigist_debug_force_plain_alu(1) == 0
    try:
        b = run_gpu(q, k, v, dout, r, W)
    finally:
        assert u.unigist_debug_force_plain_alu(0) == 1
    assert max_abs(to_np(a[0]), to_np(b[0])) <= 3.2e-2  # two bf16 roundings of values up to 4
    assert max_abs(to_np(a[1]), to_np(b[1])) <= 1e-4
    for x, y in zip(a[2:], b[2:]):
        assert rel_l2(to_np(x), to_np(y)) <= 1e-2


@pytest.mark.parametrize("B,Hq,Hkv,L,D,r,W", [(1, 4, 2, 700, 128, 4, 64), (1, 16, 8, 9001, 128, 4, 300),
                                              (2, 8, 2, 12000, 64, 2, 500)])
def test_runs_are_bitwise_reproducible(B, Hq, Hkv, L, D, r, W):
    # no kernel uses atomics: the gist phase's segments (several of them from L > 1024 on) are summed in a fixed order
    q, k, v, dout = synth.attn_inputs(B, Hq, Hkv, L, D, seed=3)
    a = run_gpu(q, k, v, dout, r, W)
    b = run_gpu(q, k, v, dout, r, W)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_zero_queries_closed_form():
    # q = 0: lse_i = ln n_vis(i) exactly in the mask, out_i = mean of the visible values
    B, Hq, Hkv, L, D, r, W = 1, 2, 1, 900, 128, 4, 70
    _, k, v, _ = synth.attn_inputs(B, Hq, Hkv, L, D, seed=5)
    q = torch.zeros(B, Hq, L, D, dtype=torch.bfloat16)
    out, lse = u.attn_fwd(q.cuda(), k.cuda(), v.cuda(), r, W)
    i = np.arange(L)
    nvis = np.minimum(i + 1, W) + np.maximum(0, (i - W + 1) // (r + 1))
    assert max_abs(to_np(lse)[0, 0], np.log(nvis)) < 1e-5
    o, _ = oracle.attn_fwd(to_np(q), to_np(k), to_np(v), r, W)
    assert max_abs(to_np(out), o) < 1e-2


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("L,D,r,W,gain", [(1500, 128, 4, 100, 8.0), (900, 64, 8, 300, 16.0), (600, 128, 4, 50, 0.0625)])
def test_peaked_and_flat_softmax(L, D, r, W, gain, dtype):
    # logits of a few hundred (softmax close to one-hot, exponent ranges far beyond one step's reference) and
    # logits close to zero (softmax close to uniform); scaling by a power of two keeps the inputs exact
    q, k, v, dout = synth.attn_inputs(1, 4, 2, L, D, dtype=dtype, seed=61)
    q, k = (q * gain).to(dtype), (k * gain).to(dtype)
    # a few rows whose scores jump by hundreds from one key tile to the next, in both directions
    q[0, :, L // 2] *= 4
    k[0, :, L // 3] *= 4
    case = f"L{L} D{D} r{r} W{W} gain{gain} {dtype}"
    got = run_gpu(q, k, v, dout, r, W)
    want = oracle_fwd_bwd(q, k, v, dout, r, W)
    big = float(np.abs(want[1]).max())      # lse is of the size of the largest logits
    assert big > 50 or gain < 1
    # fp32 build: a logit of size |S| carries a rounding error of a few ulp(|S|) = |S| 2^-23 from its D-term dot
    # product, which goes straight into lse and, relatively, into P; the 1e-5 of ordinary data scales with it
    if dtype == torch.float32:
        check(case, got, want, dtype, tol_f32=max(TOL_F32, 4 * big * 2.0 ** -23))
        return
    # bf16: a near one-hot row returns single values of v, not an average of many.  P is rounded to bf16 before the
    # second MFMA (relative error <= 2^-9 per term, so at most 2^-9 sum_j P_ij |v_j| <= 2^-9 max|v| on out) and the
    # stored result is rounded to bf16 once more (<= 2^-9 |out| <= 2^-9 max|v|): for max|v| around 4 that is beyond
    # the 1e-2 that holds for averaged rows, so the bound here is the one the arithmetic gives
    out, o_o = to_np(got[0]), want[0]
    vmax = float(v.abs().max())
    err = float(np.abs(out - o_o).max())
    print(case, f"out {err:.3e} bound {2e-3 + vmax * 2.0 ** -8:.3e}", flush=True)
    assert err <= 2e-3 + vmax * 2.0 ** -8, case
    # lse and the gradients to the usual bar (lse is of the size of the logits: a few ulp of them, like the fp32 build)
    check(case, (torch.from_numpy(o_o),) + tuple(got[1:]), want, dtype, tol_lse=max(TOL_LSE_BF16, 4 * big * 2.0 ** -23))


@pytest.mark.parametrize("D", [128, 64, 96])
@pytest.mark.parametrize("sinks,units,W", [(0, False, 100), (20, True, 7)], ids=["sliding", "sinks_units"])
def test_projection_layout_gives_the_same_bits(sinks, units, W, D):
    # q, out, dout, dq laid out [B, L, Hq, D] in memory (the strided entry points, no transposing copies): the same
    # kernels on the same numbers, so every result equals the contiguous call's bit for bit; ragged length, two batches
    B, Hq, Hkv, L, r = 2, 8, 2, 1333, 4
    q, k, v, dout = (t.cuda() for t in synth.attn_inputs(B, Hq, Hkv, L, D, seed=61))
    out, lse = u.attn_fwd(q, k, v, r, W, sinks=sinks, window_mode=int(units))
    dq, dk, dv = u.attn_bwd(q, k, v, out, lse, dout, r, W, sinks=sinks, window_mode=int(units))
    blhd = lambda t: t.transpose(1, 2).contiguous().transpose(1, 2)      # same values, [B, L, H, D] in memory
    qs, ds = blhd(q), blhd(dout)
    assert not qs.is_contiguous()
    out_s, lse_s = u.attn_fwd(qs, k, v, r, W, sinks=sinks, window_mode=int(units))
    assert out_s.stride() == qs.stride() and torch.equal(out_s, out) and torch.equal(lse_s, lse)
    dq_s, dk_s, dv_s = u.attn_bwd(qs, k, v, out_s, lse_s, ds, r, W, sinks=sinks, window_mode=int(units))
    assert dq_s.stride() == qs.stride()
    assert torch.equal(dq_s, dq) and torch.equal(dk_s, dk) and torch.equal(dv_s, dv)
    # through autograd, with an upstream gradient in the other layout
    qa, ka, va = qs.detach().requires_grad_(True), k.detach().requires_grad_(True), v.detach().requires_grad_(True)
    o = u.gist_attention(qa, ka, va, r, W, sinks=sinks, window_mode=int(units))
    o.backward(dout)
    assert torch.equal(o, out) and torch.equal(qa.grad, dq) and torch.equal(ka.grad, dk) and torch.equal(va.grad, dv)
