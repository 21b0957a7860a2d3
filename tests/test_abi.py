"""The C-ABI library loads and exports what include/unigist.h declares; argument
validation is exercised through calls that return before anything is launched."""
import ctypes as C
import os
import re

import numpy as np

import pytest

import paper_2509_15763_amd as u
from paper_2509_15763_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "unigist.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(unigist_[a-z_0-9]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    lib = u.load()
    names = _declared()
    assert "unigist_attn_fwd" in names and "unigist_decode" in names and len(names) >= 9
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_binding_has_the_same_names():
    for n in _declared():
        if n == "unigist_blockmap_free":
            continue  # the binding frees the map itself
        assert callable(getattr(u, n)), n


def test_status_strings():
    assert u.unigist_status_str(0) == "ok"
    assert "invalid" in u.unigist_status_str(1)
    assert "unsupported" in u.unigist_status_str(2)
    assert "launch" in u.unigist_status_str(3).lower()


FAKE = 0x1000  # non-null pointer that is never dereferenced: every call below fails validation first


@pytest.mark.parametrize("kw,want", [
    (dict(), None),
    (dict(B=0), 1), (dict(L=0), 1), (dict(W=0), 1), (dict(r=0), 1), (dict(Hq=6, Hkv=4), 1),
    (dict(D=100), 2), (dict(D=256), 2), (dict(D=4), 2), (dict(dt=7), 2), (dict(L=(1 << 23) + 1), 2),
])
def test_attn_argument_validation(kw, want):
    a = dict(B=1, Hq=4, Hkv=2, L=64, D=64, r=4, W=8, dt=0)
    a.update(kw)
    shape = (a["B"], a["Hq"], a["Hkv"], a["L"], a["D"], a["r"], a["W"], a["dt"])
    if want is None:
        # valid shape but null tensors -> EINVAL, still nothing launched
        assert u.unigist_attn_fwd(None, None, None, None, None, *shape) == 1
        assert u.unigist_attn_bwd_workspace(*shape) > 0
        assert u.unigist_attn_bwd(*([FAKE] * 9), *shape, None, 0) == 1
        assert u.unigist_attn_bwd(*([FAKE] * 9), *shape, FAKE + 0x100 - 0x1000 % 256, 16) == 1  # too small
        return
    assert u.unigist_attn_fwd(FAKE, FAKE, FAKE, FAKE, FAKE, *shape) == want
    assert u.unigist_attn_bwd(*([FAKE] * 9), *shape, FAKE, 1 << 40) == want
    assert u.unigist_attn_bwd_workspace(*shape) == 0


def test_ex_argument_validation():
    # B, Hq, Hkv, L, D, r, W, sinks, window_mode, dt
    ok = (1, 4, 2, 64, 64, 4, 8, 3, 1, 0)
    assert u.unigist_attn_bwd_workspace_ex(*ok) > 0
    assert u.unigist_attn_fwd_ex(None, None, None, None, None, *ok) == 1  # null tensors
    for bad in [(1, 4, 2, 64, 64, 4, 8, -1, 1, 0), (1, 4, 2, 64, 64, 4, 8, 3, 2, 0), (1, 4, 2, 64, 64, 4, 8, 3, -1, 0)]:
        assert u.unigist_attn_bwd_workspace_ex(*bad) == 0
        assert u.unigist_attn_fwd_ex(FAKE, FAKE, FAKE, FAKE, FAKE, *bad) == 1
        assert u.unigist_attn_bwd_ex(*([FAKE] * 9), *bad, FAKE, 1 << 40, 31) == 1
    # the workspace depends on the layout only through the number of compact (sink + gist) tiles
    assert u.unigist_attn_bwd_workspace_ex(1, 4, 2, 4096, 64, 4, 8, 0, 0, 0) == u.unigist_attn_bwd_workspace(
        1, 4, 2, 4096, 64, 4, 8, 0)


def test_varlen_argument_validation():
    ok = dict(Hq=4, Hkv=2, T=100, D=64, r=4, W=8)
    cu = [0, 30, 30, 100]
    args = tuple(ok.values())
    assert u.unigist_attn_bwd_varlen_workspace(*args, cu, 0) > 0
    assert u.unigist_attn_fwd_varlen(None, None, None, None, None, *args, cu, 0) == 1          # null tensors
    assert u.unigist_attn_fwd_varlen(FAKE, FAKE, FAKE, FAKE, FAKE, *args, None, 0) == 1        # no boundaries
    for bad in ([1, 30, 100], [0, 30, 99], [0, 60, 40, 100], [0, 30, 101]):
        assert u.unigist_attn_fwd_varlen(FAKE, FAKE, FAKE, FAKE, FAKE, *args, bad, 0) == 1
        assert u.unigist_attn_bwd_varlen_workspace(*args, bad, 0) == 0
        assert u.unigist_attn_bwd_varlen(*([FAKE] * 9), *args, bad, 0, FAKE, 1 << 40) == 1
    assert u.unigist_attn_bwd_varlen(*([FAKE] * 9), *args, cu, 0, FAKE, 16) == 1                # workspace too small
    # the layout with sinks and unit windows: the same checks plus the two extra arguments
    ex = (4, 2, 100, 64, 4, 8)
    assert u.unigist_attn_bwd_varlen_workspace_ex(*ex, 5, 1, cu, 0) > 0
    assert u.unigist_attn_bwd_varlen_workspace_ex(*ex, -1, 1, cu, 0) == 0
    assert u.unigist_attn_bwd_varlen_workspace_ex(*ex, 5, 2, cu, 0) == 0
    assert u.unigist_attn_fwd_varlen_ex(FAKE, FAKE, FAKE, FAKE, FAKE, *ex, -1, 0, cu, 0) == 1
    assert u.unigist_attn_fwd_varlen_ex(FAKE, FAKE, FAKE, FAKE, FAKE, *ex, 5, 2, cu, 0) == 1
    assert u.unigist_attn_fwd_varlen_ex(None, FAKE, FAKE, FAKE, FAKE, *ex, 5, 1, cu, 0) == 1
    assert u.unigist_attn_bwd_varlen_ex(*([FAKE] * 9), *ex, 5, 1, cu, 0, FAKE, 16) == 1         # workspace too small
    assert u.unigist_attn_bwd_varlen_ex(*([FAKE] * 9), *ex, 5, 3, cu, 0, FAKE, 1 << 40) == 1
    assert u.unigist_attn_bwd_varlen_workspace(*ex, cu, 0) == u.unigist_attn_bwd_varlen_workspace_ex(*ex, 0, 0, cu, 0)
    # fp32 runs document by document: one slice per stream the documents are spread over, each sized for the
    # longest document
    one = u.unigist_attn_bwd_workspace(1, 4, 2, 5000, 64, 4, 8, 1)
    assert u.unigist_attn_bwd_varlen_workspace(4, 2, 6000, 64, 4, 8, [0, 5000, 6000], 1) == 4 * ((one + 255) // 256 * 256)
    # bf16 runs the whole pack in one launch per kernel: two fp32 values per (head, row) plus the gist partial sums
    # of every document (5000 rows with r = 4: 1000 gists, 8 tiles of 128 per kv head, one segment each, reduced
    # once more); never less than the document-by-document need, which the debug switch falls back to
    pack = u.unigist_attn_bwd_varlen_workspace(4, 2, 6000, 64, 4, 8, [0, 5000, 6000], 0)
    one = u.unigist_attn_bwd_workspace(1, 4, 2, 5000, 64, 4, 8, 0)
    assert pack >= 4 * ((one + 255) // 256 * 256)
    assert pack >= 2 * 4 * 6000 * 4 + 2 * (2 * 7) * (2 * 64 * 128 * 4)


def test_cache_ex_argument_validation():
    assert u.unigist_cache_rows_ex(8, 12, 2, 2) == 9        # sinks 0 1, gists 4 7, positions 8 .. 12
    assert u.unigist_cache_rows_ex(1, 5, 2, 4) == 6         # window start inside the sinks: everything is kept
    assert u.unigist_cache_rows_ex(8, 12, 2, -1) == -1
    assert u.unigist_cache_rows_ex(3, 5, 4, 0) == u.unigist_cache_rows(3, 5, 4)
    ok = dict(kc_in=FAKE, vc_in=FAKE, s_old=0, t_old=9, cap_in=64, k_new=FAKE, v_new=FAKE, n_new=4, new_rows=4,
              kc_out=FAKE, vc_out=FAKE, s_new=6, cap_out=64, B=1, Hkv=2, D=64, r=4, sinks=3, dt=0)
    bad = dict(ok, sinks=-1)
    assert u.unigist_cache_update_ex(*bad.values()) == 1
    bad = dict(ok, cap_out=5)                                # 3 sinks + gist 7? no: always < 6 = 0 1 2; rows 3 + 8 > 5
    assert u.unigist_cache_update_ex(*bad.values()) == 1
    # prefill: unknown window mode, negative sinks, cache start right of the first query's window
    pre = lambda **kw: u.unigist_prefill_chunk_ex(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 4, 2, 64, 64, 4, 2,
                                                  kw.get("sinks", 3), kw.get("mode", 1), 500, kw.get("s", 0), 4096, 0)
    assert pre(mode=2) == 1 and pre(sinks=-1) == 1
    # query 500 with 3 sinks, r = 4: unit (500 - 3) // 5 = 99, window starts at unit 97 = position 488
    assert pre(s=489) == 1


def test_decode_argument_validation():
    ok = dict(B=2, Hq=4, Hkv=2, Lk=100, D=128, dt=0)
    ws = u.unigist_decode_workspace(*ok.values())
    assert ws > 0 and ws % 256 == 0

    def call(ws_ptr=0x10000, ws_bytes=1 << 40, q=FAKE, **kw):
        a = dict(ok)
        a.update(kw)
        return u.unigist_decode(q, FAKE, FAKE, FAKE, None, a["B"], a["Hq"], a["Hkv"], a["Lk"], None, a["D"], a["dt"],
                                ws_ptr, ws_bytes)
    assert call(q=None) == 1
    assert call(B=0) == 1 and call(Lk=0) == 1 and call(Hq=3) == 1
    assert call(D=20) == 2 and call(D=256) == 2 and call(dt=5) == 2
    assert call(ws_bytes=ws - 1) == 1
    assert call(ws_ptr=0x10010) == 1  # misaligned workspace
    assert u.unigist_decode_workspace(2, 3, 2, 100, 128, 0) == 0


def test_cpu_tensors_are_refused():
    import torch
    q = torch.zeros(1, 1, 8, 64)
    with pytest.raises(u.UnigistError):
        u.attn_fwd(q, q, q, 4, 4)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "_HERE", str(tmp_path))
    with pytest.raises(u.UnigistError, match="no fallback"):
        binding.load()


def test_cache_argument_validation():
    assert u.unigist_cache_rows(0, -1, 4) == 0 and u.unigist_cache_rows(5, 9, 4) == 6
    assert u.unigist_cache_rows(10, 3, 4) == -1 and u.unigist_cache_rows(-1, 3, 4) == -1

    def call(**kw):
        a = dict(kc_in=FAKE, vc_in=FAKE, s_old=0, t_old=9, cap_in=64, k_new=FAKE, v_new=FAKE, n_new=4, new_rows=4,
                 kc_out=FAKE, vc_out=FAKE, s_new=5, cap_out=64, B=1, Hkv=2, D=128, r=4, dt=0)
        a.update(kw)
        return u.unigist_cache_update(*a.values())
    assert call(s_new=15) == 1          # beyond t_new + 1
    assert call(s_old=3, s_new=2) == 1  # the window start never moves left
    assert call(cap_out=8) == 1         # 1 gist + 9 rows do not fit
    assert call(n_new=5) == 1           # more rows than the new buffer holds
    assert call(kc_out=None) == 1 and call(k_new=None) == 1 and call(kc_in=None) == 1
    assert call(D=100) == 2 and call(D=192) == 2 and call(dt=3) == 2
    # prefill: f32 is not built, sizes are checked before anything is launched
    p = dict(q=FAKE, kc=FAKE, vc=FAKE, out=FAKE, lse=FAKE, B=1, Hq=2, Hkv=1, C=64, D=128, r=4, W=100, p0=500, s=401,
             cap=1024, dt=1)
    assert u.unigist_prefill_chunk(*p.values()) == 2
    p.update(dt=0, s=402)
    assert u.unigist_prefill_chunk(*p.values()) == 1
    p.update(s=401, cap=100)
    assert u.unigist_prefill_chunk(*p.values()) == 1
    p.update(cap=1024, q=None)
    assert u.unigist_prefill_chunk(*p.values()) == 1
    # prefill on a row slice: heads q_rows >= C rows apart
    pv = dict(q=FAKE, kc=FAKE, vc=FAKE, out=FAKE, lse=FAKE, B=1, Hq=2, Hkv=1, C=64, q_rows=63, D=128, r=4, W=100, sinks=0,
              window_mode=0, p0=500, s=401, cap=1024, dt=0)
    assert u.unigist_prefill_chunk_view(*pv.values()) == 1
    pv.update(q_rows=1 << 24)
    assert u.unigist_prefill_chunk_view(*pv.values()) == 2
    pv.update(q_rows=4096, s=402)
    assert u.unigist_prefill_chunk_view(*pv.values()) == 1
    # forward / backward with explicit strides of the query-side tensors
    fs = dict(q=FAKE, k=FAKE, v=FAKE, out=FAKE, lse=FAKE, B=1, Hq=4, Hkv=2, L=100, D=64, r=4, W=8, sinks=0, window_mode=0,
              q_bs=100 * 256, q_hs=64, q_rs=256, dt=0)
    badf = lambda **kw: u.unigist_attn_fwd_strided(*dict(fs, **kw).values())
    assert badf(q_rs=32) == 1 and badf(q_rs=260) == 1 and badf(q_hs=4) == 1 and badf(out=FAKE + 8) == 1 and badf(dt=1) == 2
    assert badf(L=1 << 23, q_rs=1 << 12) == 2 and badf(q=None) == 1 and badf(window_mode=3) == 1
    bs = dict(q=FAKE, k=FAKE, v=FAKE, out=FAKE, lse=FAKE, dout=FAKE, dq=FAKE, dk=FAKE, dv=FAKE, B=1, Hq=4, Hkv=2, L=100, D=64,
              r=4, W=8, sinks=0, window_mode=0, q_bs=100 * 256, q_hs=64, q_rs=256, dt=0, ws=FAKE, ws_bytes=1 << 40)
    badb = lambda **kw: u.unigist_attn_bwd_strided(*dict(bs, **kw).values())
    assert badb(q_rs=260) == 1 and badb(dq=FAKE + 8) == 1 and badb(ws_bytes=16) == 1 and badb(ws=FAKE + 16) == 1 and badb(dt=1) == 2
    # the packed calls with explicit strides
    vs = dict(q=FAKE, k=FAKE, v=FAKE, out=FAKE, lse=FAKE, Hq=4, Hkv=2, T=100, D=64, r=4, W=8, sinks=0, window_mode=0,
              cu=[0, 30, 100], q_hs=64, q_rs=256, dt=0)
    badv = lambda **kw: u.unigist_attn_fwd_varlen_strided(*dict(vs, **kw).values())
    assert badv(q_rs=260) == 1 and badv(q_rs=32) == 1 and badv(cu=[0, 30, 99]) == 1 and badv(dt=1) == 2 and badv(out=None) == 1
    wb = dict(q=FAKE, k=FAKE, v=FAKE, out=FAKE, lse=FAKE, dout=FAKE, dq=FAKE, dk=FAKE, dv=FAKE, Hq=4, Hkv=2, T=100, D=64, r=4,
              W=8, sinks=0, window_mode=0, cu=[0, 30, 100], q_hs=64, q_rs=256, dt=0, ws=FAKE, ws_bytes=1 << 40)
    badw = lambda **kw: u.unigist_attn_bwd_varlen_strided(*dict(wb, **kw).values())
    assert badw(q_hs=12) == 1 and badw(ws_bytes=16) == 1 and badw(dout=FAKE + 8) == 1 and badw(dt=1) == 2
    # prefill with explicit strides: multiples of 8 elements, rows that do not overlap, aligned bases
    ps = dict(q=FAKE, kc=FAKE, vc=FAKE, out=FAKE, lse=FAKE, B=1, Hq=2, Hkv=1, C=64, D=128, r=4, W=100, sinks=0,
              window_mode=0, p0=500, s=401, cap=1024, q_bs=64 * 256, q_hs=128, q_rs=256, dt=0)
    bads = lambda **kw: u.unigist_prefill_chunk_strided(*dict(ps, **kw).values())
    assert bads(q_rs=64) == 1 and bads(q_rs=260) == 1 and bads(q_hs=0) == 1 and bads(q_bs=-8) == 1 and bads(q=FAKE + 8) == 1
    assert bads(s=402) == 1 and bads(dt=1) == 2 and bads(q=None) == 1
    # prefill over a cache of codes: the same checks plus scales, alignment and workspace
    e = dict(q=FAKE, kc=FAKE, vc=FAKE, k_scale=FAKE, v_scale=FAKE, out=FAKE, lse=FAKE, B=1, Hq=2, Hkv=1, C=64, D=128,
             r=4, W=100, sinks=0, window_mode=0, p0=500, s=401, cap=1024, ws=FAKE, ws_bytes=1 << 30)
    bad = lambda **kw: u.unigist_prefill_chunk_e4m3(*dict(e, **kw).values())
    need = u.unigist_prefill_chunk_e4m3_workspace(1, 1, 128, 401, 563, 4, 0)
    assert need == 2 * (80 + 163) * 128 * 2                  # 80 gists left of 401, positions 401 .. 563, K and V
    assert u.unigist_prefill_chunk_e4m3_workspace(1, 1, 128, 401, 399, 4, 0) == 0
    assert bad(s=402) == 1 and bad(cap=100) == 1 and bad(ws_bytes=need - 1) == 1 and bad(D=100) == 2
    assert bad(kc=FAKE + 8) == 1 and bad(ws=FAKE + 16) == 1
    for name in ("q", "kc", "vc", "k_scale", "v_scale", "out", "lse", "ws"):
        assert bad(**{name: None}) == 1, name
    # ragged prefill: the host checks what it can see (the per-sequence states live in device memory)
    g = dict(q=FAKE, kc=FAKE, vc=FAKE, out=FAKE, lse=FAKE, B=2, Hq=2, Hkv=1, C=64, D=128, r=4, W=100, sinks=0,
             window_mode=0, p0=FAKE, n=FAKE, s=FAKE, cap=1024, rows_out=FAKE, dt=0)
    bad = lambda **kw: u.unigist_prefill_chunk_ragged(*dict(g, **kw).values())
    assert bad(dt=1) == 2 and bad(D=100) == 2
    assert bad(C=0) == 1 and bad(cap=0) == 1 and bad(window_mode=2) == 1 and bad(sinks=-1) == 1 and bad(Hq=3, Hkv=2) == 1
    for name in ("q", "kc", "vc", "out", "lse", "p0", "n", "s", "rows_out"):
        assert bad(**{name: None}) == 1, name


def test_ring_cache_rows_and_argument_validation():
    import oracle
    # rows in use of the ring layout = the number of positions the query at t sees (Sec. 4.1 with the sliding window)
    for r, W, sinks in [(4, 16, 0), (2, 5, 3), (8, 1, 0), (3, 100, 40)]:
        for units in (False, True):
            for t in list(range(0, 60)) + [199, 1000]:
                want = len(oracle.compressed_cache_positions(t, r, W, sinks=sinks, units=units))
                assert u.unigist_cache_ring_rows(t, r, W, sinks, int(units)) == want, (r, W, sinks, units, t)
            assert u.unigist_cache_ring_rows(-1, r, W, sinks, int(units)) == 0
    assert u.unigist_cache_ring_rows(-2, 4, 16, 0, 0) == -1 and u.unigist_cache_ring_rows(5, 0, 16, 0, 0) == -1
    assert u.unigist_cache_ring_rows(5, 4, 16, 0, 2) == -1
    ok = dict(kc=FAKE, vc=FAKE, k_new=FAKE, v_new=FAKE, new_rows=1, t_old=FAKE, n_new=FAKE, cap=64, rows_out=FAKE, B=2,
              Hkv=2, D=64, r=4, W=16, sinks=0, window_mode=1, dt=0)
    bad = lambda **kw: u.unigist_cache_ring_append(*dict(ok, **kw).values())
    assert bad(W=0) == 1 and bad(cap=0) == 1 and bad(new_rows=0) == 1 and bad(sinks=-1) == 1 and bad(D=100) == 2 and bad(dt=3) == 2
    assert bad(window_mode=2) == 1
    for name in ("kc", "vc", "k_new", "v_new", "t_old", "n_new", "rows_out"):
        assert bad(**{name: None}) == 1, name
    cv = dict(kc_in=FAKE, vc_in=FAKE, s=FAKE, t=FAKE, cap_in=64, kc_out=FAKE, vc_out=FAKE, cap_out=64, rows_out=FAKE, B=2,
              Hkv=2, D=64, r=4, W=16, sinks=0, window_mode=0, dt=2)
    for fn in (u.unigist_cache_to_ring, u.unigist_cache_from_ring):
        assert fn(*dict(cv, W=0).values()) == 1 and fn(*dict(cv, cap_out=0).values()) == 1 and fn(*dict(cv, r=0).values()) == 1
        for name in ("kc_in", "vc_in", "s", "t", "kc_out", "vc_out", "rows_out"):
            assert fn(*dict(cv, **{name: None}).values()) == 1, name


def test_probe_argument_validation():
    assert u.unigist_probe_mfma_rate(None, FAKE, FAKE, 1, 1) == 1
    assert u.unigist_probe_mfma_rate(FAKE, None, FAKE, 1, 1) == 1
    assert u.unigist_probe_mfma_rate(FAKE, FAKE, None, 1, 1) == 1
    assert u.unigist_probe_mfma_rate(FAKE, FAKE, FAKE, 0, 1) == 1
    assert u.unigist_probe_mfma_rate(FAKE, FAKE, FAKE, 65537, 1) == 1
    assert u.unigist_probe_mfma_rate(FAKE, FAKE, FAKE, 1, 0) == 1


def test_e4m3_argument_validation():
    q = u.unigist_quantize_e4m3
    assert q(FAKE, FAKE, None, 1, 2, 3, 128, 0) == 1
    assert q(None, FAKE, FAKE, 1, 2, 3, 128, 0) == 1
    assert q(FAKE, FAKE, FAKE, 0, 2, 3, 128, 0) == 1
    assert q(FAKE, FAKE, FAKE, 1, 2, 3, 100, 0) == 2
    assert q(FAKE, FAKE, FAKE, 1, 2, 3, 104, 0) == 2            # one-byte codes: head dimensions in multiples of 16
    assert q(FAKE, FAKE, FAKE, 1, 2, 3, 128, 2) == 2            # E4M3 is not an input type
    assert q(FAKE + 8, FAKE, FAKE, 1, 2, 3, 128, 0) == 1        # 16-byte alignment
    d = u.unigist_decode_e4m3
    ws = u.unigist_decode_workspace(2, 8, 2, 100, 128, 0)
    good = dict(q=FAKE, kc=FAKE, vc=FAKE, k_scale=FAKE, v_scale=FAKE, out=FAKE, lse=None, B=2, Hq=8, Hkv=2, Lk=100,
                seqlens=None, D=128, ws=FAKE, ws_bytes=ws)
    for name, val, want in [("k_scale", None, 1), ("v_scale", None, 1), ("kc", None, 1), ("Hkv", 3, 1), ("D", 100, 2),
                            ("ws_bytes", ws - 1, 1), ("ws", FAKE + 64, 1), ("kc", FAKE + 8, 1), ("q", FAKE + 8, 1), ("B", 0, 1)]:
        assert d(**{**good, name: val}) == want, name
    # the attention calls do not take the storage type
    assert u.unigist_attn_fwd(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 4, 2, 64, 128, 4, 8, 2) == 2
    assert u.unigist_decode(FAKE, FAKE, FAKE, FAKE, None, 2, 8, 2, 100, None, 128, 2, FAKE, ws) == 2


def test_ragged_cache_update_argument_validation():
    f = u.unigist_cache_update_ragged
    good = dict(kc_in=FAKE, vc_in=FAKE, s_old=FAKE, t_old=FAKE, cap_in=64, k_new=FAKE, v_new=FAKE, n_new=FAKE, new_rows=8,
                kc_out=FAKE, vc_out=FAKE, s_new=FAKE, cap_out=64, rows_out=FAKE, B=2, Hkv=2, D=128, r=4, sinks=0, dt=0)
    for name, val, want in [("s_old", None, 1), ("t_old", None, 1), ("n_new", None, 1), ("s_new", None, 1), ("rows_out", None, 1),
                            ("kc_out", None, 1), ("kc_in", None, 1), ("k_new", None, 1), ("cap_out", 0, 1), ("r", 0, 1),
                            ("D", 100, 2), ("dt", 7, 2), ("B", 0, 1), ("new_rows", -1, 1)]:
        assert f(**{**good, name: val}) == want, name


def test_window_start_gives_the_state_whose_cache_is_the_visible_set():
    # a cache in state (unigist_window_start(t), t) holds exactly what query t may see (Sec. 4.3 with Eq. 3)
    import oracle
    for r, W, sinks, mode in [(4, 7, 0, 0), (2, 1, 0, 0), (3, 50, 0, 0), (4, 2, 5, 1), (2, 1, 0, 1), (3, 3, 9, 0), (5, 1, 2, 1)]:
        for t in list(range(0, 40)) + [97, 128, 1000]:
            s = u.unigist_window_start(t, r, W, sinks, mode)
            assert 0 <= s <= t
            want = oracle.compressed_cache_positions(t, r, W, sinks=sinks, units=bool(mode))
            assert np.array_equal(oracle.cache_positions(s, t, r, sinks), want), (r, W, sinks, mode, t)
    assert u.unigist_window_start(-1, 4, 8) == 0 and u.unigist_window_start(-2, 4, 8) == -1
    assert u.unigist_window_start(5, 0, 8) == -1 and u.unigist_window_start(5, 4, 0) == -1


def test_debug_switch_returns_the_previous_setting():
    assert u.unigist_debug_force_plain_alu(1) == 0
    assert u.unigist_debug_force_plain_alu(0) == 1
    assert u.unigist_debug_force_plain_alu(0) == 0
