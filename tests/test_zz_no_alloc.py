"""The allocation-free decode entry point against unigist_decode, through the C ABI: two calls in a row on the
built-in scratch array, the second with a smaller input, each bit-identical to the workspace version and within
the decode tolerances of the oracle; sizes beyond the array are refused."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth
from _parity import TOL_LSE_BF16, TOL_OUT_BF16, max_abs, to_np

pytestmark = pytest.mark.gpu


def _run_both(B, Hq, Hkv, Lk, D, dtype, seed, ragged):
    q, kc, vc = synth.decode_inputs(B, Hq, Hkv, Lk, D, dtype=dtype, seed=seed)
    seqlens = None
    if ragged:
        g = torch.Generator().manual_seed(seed)
        seqlens = torch.randint(1, Lk + 1, (B,), generator=g, dtype=torch.int32)
        seqlens[0] = Lk
    qd, kd, vd = q.cuda(), kc.cuda(), vc.cuda()
    sd = seqlens.cuda() if seqlens is not None else None
    dt = u.binding._dt(qd)
    out_a = torch.full_like(qd, float("nan"))
    lse_a = torch.full((B, Hq), float("nan"), device="cuda")
    out_b, lse_b = out_a.clone(), lse_a.clone()
    need = u.unigist_decode_workspace(B, Hq, Hkv, Lk, D, dt)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    sp = sd.data_ptr() if sd is not None else None
    torch.cuda.synchronize()
    # from here on no torch call that could allocate until both results are in
    rc_a = u.unigist_decode(qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), out_a.data_ptr(), lse_a.data_ptr(), B, Hq, Hkv, Lk,
                            sp, D, dt, ws.data_ptr(), need, st)
    rc_b = u.unigist_decode_noalloc(qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), out_b.data_ptr(), lse_b.data_ptr(), B, Hq,
                                    Hkv, Lk, sp, D, dt, st)
    torch.cuda.synchronize()
    assert rc_a == 0 and rc_b == 0, (rc_a, rc_b)
    assert torch.equal(out_a, out_b) and torch.equal(lse_a, lse_b)
    o, l = oracle.decode(to_np(q), to_np(kc), to_np(vc), seqlens=None if seqlens is None else seqlens.numpy())
    tol_o, tol_l = (1e-5, 1e-5) if dtype == torch.float32 else (TOL_OUT_BF16, TOL_LSE_BF16)
    assert max_abs(to_np(out_b), o) <= tol_o
    assert max_abs(to_np(lse_b), l) <= tol_l


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_two_calls_second_smaller(dtype):
    # the first call fills several slices per sequence; the second, smaller one must not see what it left behind
    _run_both(4, 32, 8, 5000, 128, dtype, seed=11, ragged=True)
    _run_both(2, 8, 2, 700, 128, dtype, seed=12, ragged=False)
    _run_both(1, 4, 4, 300, 64, dtype, seed=13, ragged=True)


def test_refuses_what_does_not_fit():
    B, Hq, Hkv, Lk, D = 2048, 32, 8, 4096, 128
    need = u.unigist_decode_workspace(B, Hq, Hkv, Lk, D, u.UNIGIST_BF16)
    assert need > u.unigist_decode_noalloc_scratch_bytes()
    x = torch.zeros(16, device="cuda")  # never touched: the call is refused before any launch
    rc = u.unigist_decode_noalloc(x.data_ptr(), x.data_ptr(), x.data_ptr(), x.data_ptr(), None, B, Hq, Hkv, Lk, None, D,
                                  u.UNIGIST_BF16, None)
    assert rc == 4 and "scratch" in u.unigist_status_str(rc)
    assert u.unigist_decode_noalloc(None, None, None, None, None, 1, 4, 1, 100, None, 128, u.UNIGIST_BF16, None) == 1
    assert u.unigist_decode_noalloc(x.data_ptr(), x.data_ptr(), x.data_ptr(), x.data_ptr(), None, 1, 4, 1, 100, None, 100,
                                    u.UNIGIST_BF16, None) == 2


def test_under_graph_capture():
    # what the entry point is for: a captured decode step that allocates nothing; replays with new cache contents
    # equal the eager unigist_decode bit for bit
    B, Hq, Hkv, Lk, D = 3, 8, 2, 1500, 128
    q, kc, vc = (t.cuda() for t in synth.decode_inputs(B, Hq, Hkv, Lk, D, seed=21))
    out = torch.zeros_like(q)
    lse = torch.zeros(B, Hq, device="cuda")
    dt = u.binding._dt(q)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):   # first call outside the capture: looks up the scratch array's address on this device
        assert u.unigist_decode_noalloc(q.data_ptr(), kc.data_ptr(), vc.data_ptr(), out.data_ptr(), lse.data_ptr(), B, Hq, Hkv,
                                        Lk, None, D, dt, side.cuda_stream) == 0
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        rc = u.unigist_decode_noalloc(q.data_ptr(), kc.data_ptr(), vc.data_ptr(), out.data_ptr(), lse.data_ptr(), B, Hq, Hkv,
                                      Lk, None, D, dt, torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    for n in range(3):
        q2, k2, v2 = (t.cuda() for t in synth.decode_inputs(B, Hq, Hkv, Lk, D, seed=30 + n))
        q.copy_(q2), kc.copy_(k2), vc.copy_(v2)
        out.zero_(), lse.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        want_o, want_l = u.decode(q, kc, vc)
        torch.cuda.synchronize()
        assert torch.equal(out, want_o) and torch.equal(lse, want_l), n
