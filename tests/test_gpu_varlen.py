"""GPU parity of the *_varlen entry points: documents packed into one sequence, attention confined to each
document (Sec. 5.1), against the fp64 oracle evaluated with the packed predicate on the same inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth
from _parity import max_abs, rel_l2, to_np
from test_gpu_attention import check
from _parity import out_ok

pytestmark = pytest.mark.gpu


def packed_inputs(Hq, Hkv, T, D, dtype, seed):
    q, k, v, dout = synth.attn_inputs(1, Hq, Hkv, T, D, dtype=dtype, seed=seed)
    return q[0], k[0], v[0], dout[0]


def run_gpu(q, k, v, dout, r, W, cu, sinks=0, units=False):
    qd, kd, vd, dod = (t.cuda() for t in (q, k, v, dout))
    out, lse = u.attn_fwd_varlen(qd, kd, vd, r, W, cu, sinks=sinks, window_mode=int(units))
    dq, dk, dv = u.attn_bwd_varlen(qd, kd, vd, out, lse, dod, r, W, cu, sinks=sinks, window_mode=int(units))
    torch.cuda.synchronize()
    return out, lse, dq, dk, dv


def oracle_packed(q, k, v, dout, r, W, cu, **mask):
    qn, kn, vn, don = (to_np(t)[None] for t in (q, k, v, dout))
    out, lse = oracle.attn_fwd(qn, kn, vn, r, W, cu=cu, **mask)
    dq, dk, dv = oracle.attn_bwd(qn, kn, vn, don, r, W, cu=cu, **mask)
    return out[0], lse[0], dq[0], dk[0], dv[0]


# Hq, Hkv, D, r, W, document lengths
SMALL = [
    (1, 1, 64, 4, 128, [300, 500, 224]),              # multiples of nothing in particular
    (4, 2, 64, 4, 40, [1, 2, 130, 0, 64, 136]),        # one-token documents, an empty one, tile-sized ones
    (4, 1, 128, 8, 100, [257, 443]),                   # D = 128, group of 4
    (2, 2, 128, 2, 1, [90, 90, 77]),                   # W = 1
    (2, 1, 64, 4, 10**6, [200, 184]),                  # window >= L: causal inside each document
    (2, 1, 128, 2**31 - 2, 33, [150, 150]),            # no gists
    (8, 8, 64, 16, 64, [100, 100]),                    # 8 kv heads
    (2, 2, 128, 4, 16, [700]),                         # one document == the plain entry point's case
    (4, 2, 96, 4, 40, [257, 1, 300, 130]),             # head dimension 96
    (2, 1, 40, 2, 50, [200, 333]),                     # ... and 40
]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("Hq,Hkv,D,r,W,lens", SMALL)
def test_small_packs_match_oracle(Hq, Hkv, D, r, W, lens, dtype):
    cu = [0] + np.cumsum(lens).tolist()
    case = f"Hq{Hq} Hkv{Hkv} D{D} r{r} W{W} docs{lens} {dtype}"
    print("case", case, flush=True)
    q, k, v, dout = packed_inputs(Hq, Hkv, cu[-1], D, dtype, seed=31)
    got = run_gpu(q, k, v, dout, r, W, cu)
    check(case, got, oracle_packed(q, k, v, dout, r, W, cu), dtype)


# Hq, Hkv, D, r, W, sinks, unit windows, document lengths: the layout with sinks and unit-aligned windows
# restarting in every document (the training setting of Sec. 5.1)
SMALL_EX = [
    (4, 2, 64, 4, 3, 10, True, [300, 7, 500, 10, 11, 224]),      # documents shorter than, equal to, one past the sinks
    (4, 1, 128, 2, 6, 33, True, [257, 443, 1]),
    (2, 2, 128, 4, 40, 5, False, [90, 190, 77]),                 # sinks with the sliding window
    (2, 1, 64, 8, 1, 128, True, [129, 600, 128]),                # 128 sinks, window of one unit
]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("Hq,Hkv,D,r,W,sinks,units,lens", SMALL_EX)
def test_small_packs_with_sinks_and_unit_windows_match_oracle(Hq, Hkv, D, r, W, sinks, units, lens, dtype):
    cu = [0] + np.cumsum(lens).tolist()
    case = f"Hq{Hq} Hkv{Hkv} D{D} r{r} W{W} sinks{sinks} units{int(units)} docs{lens} {dtype}"
    print("case", case, flush=True)
    q, k, v, dout = packed_inputs(Hq, Hkv, cu[-1], D, dtype, seed=34)
    got = run_gpu(q, k, v, dout, r, W, cu, sinks=sinks, units=units)
    check(case, got, oracle_packed(q, k, v, dout, r, W, cu, sinks=sinks, units=units), dtype)


def test_mid_pack_with_sinks_and_unit_windows_matches_oracle():
    # the paper's proportions in small (r = 4, a window of 25 units, 128 sinks): documents long enough for gists
    # left of the window (the gist phase and its per-document partial sums) next to short ones
    lens = [4500, 37, 3000, 130, 1463]
    cu = [0] + np.cumsum(lens).tolist()
    q, k, v, dout = packed_inputs(4, 1, cu[-1], 128, torch.bfloat16, seed=35)
    got = run_gpu(q, k, v, dout, 4, 25, cu, sinks=128, units=True)
    check(f"docs{lens}", got, oracle_packed(q, k, v, dout, 4, 25, cu, sinks=128, units=True), torch.bfloat16)


def test_mid_pack_matches_oracle():
    # documents longer than 4096 (several dK/dV segments) next to short ones, ragged everywhere
    lens = [4500, 37, 3000, 1463]
    cu = [0] + np.cumsum(lens).tolist()
    q, k, v, dout = packed_inputs(4, 1, cu[-1], 128, torch.bfloat16, seed=32)
    got = run_gpu(q, k, v, dout, 4, 300, cu)
    check(f"docs{lens}", got, oracle_packed(q, k, v, dout, 4, 300, cu), torch.bfloat16)


def test_more_documents_than_one_launch_holds():
    # The bf16 kernels cover 64 documents per launch: 150 documents (empty ones among them) need three launches
    # of every kernel.  Two documents are long enough to have gists left of their window (gist-phase partial
    # sums, which each document keeps in slots of its own), and the longest ones do not come first.
    rng = np.random.default_rng(5)
    lens = rng.integers(0, 40, size=150).tolist()
    lens[3], lens[77], lens[140] = 700, 0, 900
    cu = [0] + np.cumsum(lens).tolist()
    q, k, v, dout = packed_inputs(4, 2, cu[-1], 64, torch.bfloat16, seed=33)
    got = run_gpu(q, k, v, dout, 2, 24, cu)
    check(f"{len(lens)} docs", got, oracle_packed(q, k, v, dout, 2, 24, cu), torch.bfloat16)


def test_single_document_is_the_plain_entry_point():
    q, k, v, dout = packed_inputs(4, 2, 700, 128, torch.bfloat16, seed=3)
    a = run_gpu(q, k, v, dout, 4, 64, [0, 700])
    qd, kd, vd, dod = (t[None].cuda() for t in (q, k, v, dout))
    out, lse = u.attn_fwd(qd, kd, vd, 4, 64)
    b = (out, lse) + tuple(u.attn_bwd(qd, kd, vd, out, lse, dod, 4, 64))
    for x, y in zip(a, b):
        assert torch.equal(x, y[0])


def test_documents_do_not_see_each_other():
    # changing one document's keys, values and upstream gradients leaves every other document's results bit-identical
    lens = [200, 333, 150]
    cu = [0] + np.cumsum(lens).tolist()
    q, k, v, dout = packed_inputs(2, 1, cu[-1], 64, torch.bfloat16, seed=33)
    a = run_gpu(q, k, v, dout, 4, 50, cu)
    k2, v2, d2 = k.clone(), v.clone(), dout.clone()
    k2[:, cu[1]:cu[2]] += 1.0
    v2[:, cu[1]:cu[2]] -= 2.0
    d2[:, cu[1]:cu[2]] *= 3.0
    b = run_gpu(q, k2, v2, d2, 4, 50, cu)
    for x, y in zip(a, b):
        for lo, hi in ((cu[0], cu[1]), (cu[2], cu[3])):
            assert torch.equal(x[:, lo:hi], y[:, lo:hi])
        assert not torch.equal(x[:, cu[1]:cu[2]], y[:, cu[1]:cu[2]])


@pytest.mark.parametrize("Wm,sinks,units", [(None, 0, False), (25, 128, True)], ids=["sliding", "sinks_units"])
def test_full_length_pack_sampled_rows_and_columns(Wm, sinks, units):
    # the 32K training shape as a pack of five documents (each padded to a multiple of r as in App. B), with the
    # sliding window of the benchmark and in the paper's layout (128 sinks, a window of 25 units):
    # sampled rows and key columns of two documents against the oracle on those documents alone
    w = synth.WORKLOADS["cfg2_llama8b_32k"]
    Hq, Hkv, T, D, r, W = w["Hq"], w["Hkv"], w["L"], w["D"], w["r"], w["W"]
    W = W if Wm is None else Wm
    mask = dict(sinks=sinks, units=units) if sinks or units else {}
    lens = [8192, 4100, 12288, 1020, 7168]
    assert sum(lens) == T
    cu = [0] + np.cumsum(lens).tolist()
    q, k, v, dout = packed_inputs(Hq, Hkv, T, D, torch.bfloat16, seed=34)
    out, lse, dq, dk, dv = run_gpu(q, k, v, dout, r, W, cu, sinks=sinks, units=units)
    rng = np.random.default_rng(1)
    G = Hq // Hkv
    for d in (1, 2):
        a, b = cu[d], cu[d + 1]
        n = b - a
        rows = np.unique(np.concatenate([[0, 1, 4, W - 1, W, W + 1, sinks, sinks + 1, n - 1], rng.integers(0, n, 24)]))
        cols = np.unique(np.concatenate([[0, 4, 9, n - 1, n - 2], rng.integers(0, n, 12)]))
        for h in (3, 30):
            hk = h // G
            qn, kn, vn, don = (to_np(t[h_, a:b]) for t, h_ in ((q, h), (k, hk), (v, hk), (dout, h)))
            o, l = oracle.attn_fwd_rows(qn, kn, vn, rows, r, W, **mask)
            assert out_ok(to_np(out[h, a:b])[rows], o), (d, h)
            assert max_abs(to_np(lse[h, a:b])[rows], l) <= 1e-2
            assert rel_l2(to_np(dq[h, a:b])[rows], oracle.attn_dq_rows(qn, kn, vn, don, rows, r, W, **mask)) <= 2e-2
        hk = 6
        gk = np.zeros((len(cols), D))
        gv = np.zeros((len(cols), D))
        for g in range(G):
            x, y = oracle.attn_dkdv_cols(to_np(q[hk * G + g, a:b]), to_np(k[hk, a:b]), to_np(v[hk, a:b]),
                                         to_np(dout[hk * G + g, a:b]), cols, r, W, **mask)
            gk += x
            gv += y
        assert rel_l2(to_np(dk[hk, a:b])[cols], gk) <= 2e-2
        assert rel_l2(to_np(dv[hk, a:b])[cols], gv) <= 2e-2


def test_back_to_back_backward_calls_share_a_workspace():
    # two backward calls enqueued without a synchronisation between them, on one workspace buffer, with
    # different packs (more documents than streams in the first, fewer in the second): the second call's
    # kernels may not start before the first call's have finished with the workspace
    Hq, Hkv, D, r, W = 4, 2, 128, 4, 48
    packs = [[600, 90, 1300, 257, 33, 410, 5], [2000, 300]]
    ins, fwd = [], []
    for n, lens in enumerate(packs):
        q, k, v, dout = packed_inputs(Hq, Hkv, sum(lens), D, torch.bfloat16, seed=40 + n)
        ins.append((q, k, v, dout))
        qd, kd, vd, dod = (t.cuda() for t in (q, k, v, dout))
        cu = [0] + np.cumsum(lens).tolist()
        fwd.append((qd, kd, vd, dod, cu) + tuple(u.attn_fwd_varlen(qd, kd, vd, r, W, cu)))
    need = max(u.unigist_attn_bwd_varlen_workspace(Hq, Hkv, f[4][-1], D, r, W, f[4], 0) for f in fwd)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    grads = [u.attn_bwd_varlen(qd, kd, vd, out, lse, dod, r, W, cu, workspace=ws) for qd, kd, vd, dod, cu, out, lse in fwd]
    torch.cuda.synchronize()
    for (q, k, v, dout), f, g in zip(ins, fwd, grads):
        want = oracle_packed(q, k, v, dout, r, W, f[4])
        check(f"docs{np.diff(f[4]).tolist()}", (f[5], f[6]) + tuple(g), want, torch.bfloat16)


def test_every_gradient_row_is_written():
    # the backward fully overwrites dq, dk, dv (no zero-initialisation by the caller): buffers pre-filled with NaN
    # come back without one, for a pack with empty, one-token and ragged documents
    Hq, Hkv, D, r, W = 4, 2, 128, 4, 40
    lens = [0, 1, 300, 0, 129, 64, 1, 777, 0]
    cu = [0] + np.cumsum(lens).tolist()
    T = cu[-1]
    q, k, v, dout = (t.cuda() for t in packed_inputs(Hq, Hkv, T, D, torch.bfloat16, seed=36))
    out, lse = u.attn_fwd_varlen(q, k, v, r, W, cu)
    nan = float("nan")
    dq, dk, dv = torch.full_like(q, nan), torch.full_like(k, nan), torch.full_like(v, nan)
    ws = torch.empty(u.unigist_attn_bwd_varlen_workspace(Hq, Hkv, T, D, r, W, cu, u.UNIGIST_BF16), dtype=torch.uint8, device="cuda")
    st = u.unigist_attn_bwd_varlen(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(), dout.data_ptr(),
                                   dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), Hq, Hkv, T, D, r, W, cu, u.UNIGIST_BF16,
                                   ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert st == 0
    assert not bool(torch.isnan(dq).any()) and not bool(torch.isnan(dk).any()) and not bool(torch.isnan(dv).any())
    assert not bool(torch.isnan(out).any()) and not bool(torch.isnan(lse).any())


@pytest.mark.parametrize("D", [128, 64, 96])
@pytest.mark.parametrize("sinks,units,W", [(0, False, 100), (20, True, 7)], ids=["sliding", "sinks_units"])
def test_packed_projection_layout_gives_the_same_bits(sinks, units, W, D):
    # q, out, dout, dq laid out [T, Hq, D] in memory, as a packed projection output: same bits as the [Hq, T, D] call
    Hq, Hkv, r = 8, 2, 4
    lens = [700, 0, 33, 1500, 129]
    cu = [0] + np.cumsum(lens).tolist()
    q, k, v, dout = (t.cuda() for t in packed_inputs(Hq, Hkv, cu[-1], D, torch.bfloat16, seed=37))
    kw = dict(sinks=sinks, window_mode=int(units))
    out, lse = u.attn_fwd_varlen(q, k, v, r, W, cu, **kw)
    dq, dk, dv = u.attn_bwd_varlen(q, k, v, out, lse, dout, r, W, cu, **kw)
    thd = lambda t: t.transpose(0, 1).contiguous().transpose(0, 1)        # same values, [T, H, D] in memory
    qs = thd(q)
    out_s, lse_s = u.attn_fwd_varlen(qs, k, v, r, W, cu, **kw)
    assert out_s.stride() == qs.stride() and torch.equal(out_s, out) and torch.equal(lse_s, lse)
    dq_s, dk_s, dv_s = u.attn_bwd_varlen(qs, k, v, out_s, lse_s, thd(dout), r, W, cu, **kw)
    assert dq_s.stride() == qs.stride() and torch.equal(dq_s, dq) and torch.equal(dk_s, dk) and torch.equal(dv_s, dv)
    qa, ka, va = qs.detach().requires_grad_(True), k.detach().requires_grad_(True), v.detach().requires_grad_(True)
    o = u.gist_attention_varlen(qa, ka, va, r, W, cu, **kw)
    o.backward(dout)
    assert torch.equal(o, out) and torch.equal(qa.grad, dq) and torch.equal(ka.grad, dk) and torch.equal(va.grad, dv)
