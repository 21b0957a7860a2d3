"""The autograd wrappers: loss.backward() through gist_attention reproduces the oracle's analytic gradients."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth
from _parity import TOL_GRAD_BF16, TOL_OUT_BF16, max_abs, rel_l2, to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mask", [dict(), dict(sinks=5, units=True)], ids=["plain", "sinks_units"])
def test_backward_through_the_wrapper(mask):
    B, Hq, Hkv, L, D, r, W = 1, 4, 2, 600, 128, 4, (64 if not mask else 9)
    q, k, v, dout = synth.attn_inputs(B, Hq, Hkv, L, D, seed=41)
    qd, kd, vd = (t.cuda().requires_grad_(True) for t in (q, k, v))
    kw = dict(sinks=mask.get("sinks", 0), window_mode=int(mask.get("units", False)))
    out = u.gist_attention(qd, kd, vd, r, W, **kw)
    (out.float() * dout.cuda().float()).sum().backward()
    qn, kn, vn, don = (to_np(t) for t in (q, k, v, dout))
    o, _ = oracle.attn_fwd(qn, kn, vn, r, W, **mask)
    g = oracle.attn_bwd(qn, kn, vn, don, r, W, **mask)
    assert max_abs(to_np(out), o) <= TOL_OUT_BF16
    for got, want in zip((qd.grad, kd.grad, vd.grad), g):
        assert rel_l2(to_np(got), want) <= TOL_GRAD_BF16


@pytest.mark.parametrize("W,sinks,units", [(40, 0, False), (3, 20, True)], ids=["sliding", "sinks_units"])
def test_backward_through_the_varlen_wrapper(W, sinks, units):
    Hq, Hkv, D, r, cu = 4, 1, 64, 4, [0, 130, 131, 500]
    q, k, v, dout = synth.attn_inputs(1, Hq, Hkv, cu[-1], D, seed=42)
    qd, kd, vd = (t[0].cuda().requires_grad_(True) for t in (q, k, v))
    out = u.gist_attention_varlen(qd, kd, vd, r, W, cu, sinks=sinks, window_mode=int(units))
    (out.float() * dout[0].cuda().float()).sum().backward()
    qn, kn, vn, don = (to_np(t) for t in (q, k, v, dout))
    g = oracle.attn_bwd(qn, kn, vn, don, r, W, cu=cu, sinks=sinks, units=units)
    for got, want in zip((qd.grad, kd.grad, vd.grad), g):
        assert rel_l2(to_np(got), want[0]) <= TOL_GRAD_BF16
