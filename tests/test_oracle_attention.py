"""Pins for the oracle's forward, backward and decode arithmetic.

Each test compares the oracle with something other than itself: explicit loops,
closed forms, library attention (torch SDPA in fp64 on the CPU) on the special
cases that reduce to it, library autograd, and central finite differences.
"""
import math

import numpy as np
import pytest
import torch

import oracle


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _loops_forward(q, k, v, r, W):
    """Triple loops, plain exp (no max subtraction), the predicate written out."""
    L, D = q.shape
    out = np.zeros((L, D))
    lse = np.zeros(L)
    for i in range(L):
        z = 0.0
        acc = [0.0] * D
        for j in range(L):
            gist = (j + 1) % (r + 1) == 0
            if j <= i and (gist or i - j < W):
                s = 0.0
                for d in range(D):
                    s += q[i, d] * k[j, d]
                e = math.exp(s / math.sqrt(D))
                z += e
                for d in range(D):
                    acc[d] += e * v[j, d]
        out[i] = [a / z for a in acc]
        lse[i] = math.log(z)
    return out, lse


@pytest.mark.parametrize("L,D,r,W", [(23, 4, 4, 6), (32, 8, 2, 5), (17, 3, 1, 1), (20, 4, 7, 3)])
def test_forward_matches_explicit_loops(L, D, r, W):
    q, k, v = _rand((L, D), 1), _rand((L, D), 2), _rand((L, D), 3)
    want_o, want_l = _loops_forward(q, k, v, r, W)
    for block in (512, 5):  # row blocking must not change anything
        o, l = oracle.attn_fwd_head(q, k, v, r, W, block=block)
        np.testing.assert_allclose(o, want_o, rtol=0, atol=1e-13)
        np.testing.assert_allclose(l, want_l, rtol=0, atol=1e-13)


def _sdpa(q, k, v, mask=None, causal=False):
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a))[None, None]
    m = None if mask is None else torch.from_numpy(mask)[None, None]
    o = torch.nn.functional.scaled_dot_product_attention(t(q), t(k), t(v), attn_mask=m, is_causal=causal)
    return o[0, 0].numpy()


def test_full_window_equals_library_causal_attention():
    L, D = 130, 16
    q, k, v = _rand((L, D), 4), _rand((L, D), 5), _rand((L, D), 6)
    o, _ = oracle.attn_fwd_head(q, k, v, r=4, W=L)
    np.testing.assert_allclose(o, _sdpa(q, k, v, causal=True), rtol=0, atol=1e-13)


def test_no_gists_equals_library_sliding_window_attention():
    L, D, W = 130, 16, 9
    q, k, v = _rand((L, D), 7), _rand((L, D), 8), _rand((L, D), 9)
    band = np.tril(np.ones((L, L), dtype=bool)) & ~np.tril(np.ones((L, L), dtype=bool), -W)
    o, _ = oracle.attn_fwd_head(q, k, v, r=10**6, W=W)
    np.testing.assert_allclose(o, _sdpa(q, k, v, mask=band), rtol=0, atol=1e-13)


def test_zero_queries_closed_form():
    # q = 0 => uniform softmax over the visible set: lse = ln n_vis(i), out = mean of visible v
    L, D, r, W = 300, 8, 4, 37
    k, v = _rand((L, D), 10), _rand((L, D), 11)
    o, l = oracle.attn_fwd_head(np.zeros((L, D)), k, v, r, W)
    for i in range(L):
        n = min(i + 1, W) + max(0, (i - W + 1) // (r + 1))
        assert abs(l[i] - math.log(n)) < 1e-13
        vis = [j for j in range(i + 1) if (j + 1) % (r + 1) == 0 or i - j < W]
        assert len(vis) == n
        np.testing.assert_allclose(o[i], v[vis].mean(axis=0), rtol=0, atol=1e-13)


def test_constant_values_and_row_sums():
    L, D, r, W = 120, 8, 4, 11
    q, k = _rand((L, D), 12), _rand((L, D), 13)
    c = _rand((D,), 14)
    o, _ = oracle.attn_fwd_head(q, k, np.tile(c, (L, 1)), r, W)
    np.testing.assert_allclose(o, np.tile(c, (L, 1)), rtol=0, atol=1e-13)
    # softmax rows sum to one: V = identity columns recovers P itself
    o, _ = oracle.attn_fwd_head(q, k, np.eye(L), r, W)
    np.testing.assert_allclose(o.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    assert np.array_equal(o > 0, oracle.mask_rows(np.arange(L), L, r, W))


def test_invisible_keys_cannot_influence_a_row():
    L, D, r, W = 200, 8, 4, 16
    q, k, v = _rand((L, D), 15), _rand((L, D), 16), _rand((L, D), 17)
    i = 150
    o0, l0 = oracle.attn_fwd_rows(q, k, v, [i], r, W)
    k2, v2 = k.copy(), v.copy()
    for j in range(L):
        if not (j <= i and ((j + 1) % (r + 1) == 0 or i - j < W)):
            k2[j] = 1e4
            v2[j] = -1e4
    o1, l1 = oracle.attn_fwd_rows(q, k2, v2, [i], r, W)
    assert np.array_equal(o0, o1) and np.array_equal(l0, l1)


def _loss(q, k, v, dout, r, W):
    o, _ = oracle.attn_fwd_head(q, k, v, r, W)
    return float((o * dout).sum())


@pytest.mark.parametrize("L,D,r,W", [(14, 3, 4, 4), (12, 2, 2, 3)])
def test_backward_matches_finite_differences(L, D, r, W):
    q, k, v, do = (_rand((L, D), s) for s in (20, 21, 22, 23))
    dq, dk, dv = oracle.attn_bwd_head(q, k, v, do, r, W, block=5)
    h = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for idx in np.ndindex(L, D):
            old = x[idx]
            x[idx] = old + h
            fp = _loss(q, k, v, do, r, W)
            x[idx] = old - h
            fm = _loss(q, k, v, do, r, W)
            x[idx] = old
            fd = (fp - fm) / (2 * h)
            assert abs(fd - g[idx]) <= 1e-7 * max(1.0, abs(g[idx])), (name, idx, fd, g[idx])


def test_backward_matches_library_autograd():
    L, D, r, W = 90, 8, 4, 13
    q, k, v, do = (_rand((L, D), s) for s in (24, 25, 26, 27))
    tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (q, k, v))
    M = torch.from_numpy(oracle.mask_rows(np.arange(L), L, r, W))
    o = torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None], tv[None], attn_mask=M[None])
    (o[0] * torch.from_numpy(do)).sum().backward()
    dq, dk, dv = oracle.attn_bwd_head(q, k, v, do, r, W, block=32)
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.attn_dq_rows(q, k, v, do, [3, 50, 89], r, W), dq[[3, 50, 89]], rtol=0, atol=1e-13)


def test_column_sampled_backward_equals_full_backward():
    L, D, r, W = 150, 8, 4, 17
    q, k, v, do = (_rand((L, D), s) for s in (50, 51, 52, 53))
    _, dk, dv = oracle.attn_bwd_head(q, k, v, do, r, W)
    cols = [0, 4, 9, 77, 78, 79, 149]
    a = oracle.attn_dkdv_cols(q, k, v, do, cols, r, W, 0, 60, block=16)
    b = oracle.attn_dkdv_cols(q, k, v, do, cols, r, W, 60, None, block=64)
    np.testing.assert_allclose(a[0] + b[0], dk[cols], rtol=0, atol=1e-13)
    np.testing.assert_allclose(a[1] + b[1], dv[cols], rtol=0, atol=1e-13)
    # rows before a raw key or outside its window add nothing
    z = oracle.attn_dkdv_cols(q, k, v, do, [78], r, W, 78 + W, None)
    assert not z[0].any() and not z[1].any()


def test_backward_structural_zeros():
    # dout non-zero only on rows i >= j0 + W: raw keys j <= j0 get no gradient, gists do
    L, D, r, W, j0 = 80, 4, 4, 6, 30
    q, k, v, do = (_rand((L, D), s) for s in (28, 29, 30, 31))
    do[: j0 + W] = 0.0
    _, dk, dv = oracle.attn_bwd_head(q, k, v, do, r, W)
    for j in range(j0 + 1):
        if (j + 1) % (r + 1) == 0:
            assert np.abs(dk[j]).max() > 0 and np.abs(dv[j]).max() > 0
        else:
            assert not dk[j].any() and not dv[j].any()


def test_gqa_is_sum_over_the_group():
    B, Hq, Hkv, L, D, r, W = 2, 4, 2, 40, 4, 3, 7
    q, do = _rand((B, Hq, L, D), 32), _rand((B, Hq, L, D), 33)
    k, v = _rand((B, Hkv, L, D), 34), _rand((B, Hkv, L, D), 35)
    o, l = oracle.attn_fwd(q, k, v, r, W)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, r, W)
    krep, vrep = np.repeat(k, Hq // Hkv, axis=1), np.repeat(v, Hq // Hkv, axis=1)
    o2, l2 = oracle.attn_fwd(q, krep, vrep, r, W)
    dq2, dk2, dv2 = oracle.attn_bwd(q, krep, vrep, do, r, W)
    assert np.array_equal(o, o2) and np.array_equal(l, l2) and np.array_equal(dq, dq2)
    np.testing.assert_allclose(dk, dk2.reshape(B, Hkv, Hq // Hkv, L, D).sum(2), rtol=0, atol=1e-13)
    np.testing.assert_allclose(dv, dv2.reshape(B, Hkv, Hq // Hkv, L, D).sum(2), rtol=0, atol=1e-13)
    # query head h must use kv head h // (Hq/Hkv): check one head against the single-head routine
    o_h, _ = oracle.attn_fwd_head(q[1, 3], k[1, 1], v[1, 1], r, W)
    assert np.array_equal(o[1, 3], o_h)


def test_decode_equals_last_row_of_forward():
    # cache = all gists + raw tokens inside the window of the last position, in any order
    L, D, r, W = 257, 8, 4, 21
    q, k, v = _rand((L, D), 36), _rand((L, D), 37), _rand((L, D), 38)
    t = L - 1
    o_row, l_row = oracle.attn_fwd_rows(q, k, v, [t], r, W)
    pos = oracle.compressed_cache_positions(t, r, W)
    perm = np.random.default_rng(0).permutation(len(pos))
    kc, vc = k[pos][perm], v[pos][perm]
    o, l = oracle.decode(q[t][None, None], kc[None, None], vc[None, None])
    np.testing.assert_allclose(o[0, 0], o_row[0], rtol=0, atol=1e-13)
    np.testing.assert_allclose(l[0, 0], l_row[0], rtol=0, atol=1e-13)


def test_decode_ragged_and_gqa_against_loops():
    B, Hq, Hkv, Lk, D = 3, 4, 2, 19, 4
    q, kc, vc = _rand((B, Hq, D), 39), _rand((B, Hkv, Lk, D), 40), _rand((B, Hkv, Lk, D), 41)
    seqlens = [19, 1, 7]
    o, l = oracle.decode(q, kc, vc, seqlens)
    for b in range(B):
        for h in range(Hq):
            g = h // 2
            e = [math.exp(sum(q[b, h, d] * kc[b, g, j, d] for d in range(D)) / math.sqrt(D)) for j in range(seqlens[b])]
            z = sum(e)
            want = [sum(e[j] * vc[b, g, j, d] for j in range(seqlens[b])) / z for d in range(D)]
            np.testing.assert_allclose(o[b, h], want, rtol=0, atol=1e-13)
            assert abs(l[b, h] - math.log(z)) < 1e-13


def test_sinks_and_unit_window_thread_through_forward_and_backward():
    # library attention + autograd with the explicitly built mask, and the rows/columns variants
    L, D, r, k, S = 70, 8, 4, 1, 3
    kw = dict(sinks=S, units=True)
    q, kk, v, do = (_rand((L, D), s) for s in (60, 61, 62, 63))
    M = oracle.mask_rows(np.arange(L), L, r, k, **kw)
    assert M[40].sum() != oracle.mask_rows([40], L, r, k)[0].sum()          # the keyword arguments matter
    tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (q, kk, v))
    o = torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None], tv[None], attn_mask=torch.from_numpy(M)[None])
    (o[0] * torch.from_numpy(do)).sum().backward()
    out, _ = oracle.attn_fwd_head(q, kk, v, r, k, **kw)
    dq, dk, dv = oracle.attn_bwd_head(q, kk, v, do, r, k, block=16, **kw)
    np.testing.assert_allclose(out, o[0].detach().numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=0, atol=1e-12)
    rows = [0, 2, 3, 40, 69]
    np.testing.assert_allclose(oracle.attn_fwd_rows(q, kk, v, rows, r, k, **kw)[0], out[rows], rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.attn_dq_rows(q, kk, v, do, rows, r, k, **kw), dq[rows], rtol=0, atol=1e-13)
    a = oracle.attn_dkdv_cols(q, kk, v, do, [1, 7, 30], r, k, **kw)
    np.testing.assert_allclose(a[0], dk[[1, 7, 30]], rtol=0, atol=1e-13)
    np.testing.assert_allclose(a[1], dv[[1, 7, 30]], rtol=0, atol=1e-13)


# ---------------------------------------------------------------- packed documents (cu=)
def test_packed_attention_is_the_documents_side_by_side():
    # dense evaluation with the packed predicate == each document through the (pinned) single-document path
    rng = np.random.default_rng(7)
    cu, r, W, D = [0, 37, 37, 90, 91, 150], 4, 9, 16
    T = cu[-1]
    q, k, v, do = (rng.standard_normal((1, 2, T, D)) for _ in range(4))
    k, v = k[:, :1], v[:, :1]
    out, lse = oracle.attn_fwd(q, k, v, r, W, cu=cu)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, r, W, cu=cu)
    for a, b in zip(cu[:-1], cu[1:]):
        if a == b:
            continue
        o1, l1 = oracle.attn_fwd(q[:, :, a:b], k[:, :, a:b], v[:, :, a:b], r, W)
        g = oracle.attn_bwd(q[:, :, a:b], k[:, :, a:b], v[:, :, a:b], do[:, :, a:b], r, W)
        assert np.allclose(out[:, :, a:b], o1, atol=1e-12) and np.allclose(lse[:, :, a:b], l1, atol=1e-12)
        for x, y in zip((dq, dk, dv), g):
            assert np.allclose(x[:, :, a:b], y, atol=1e-12)


def test_packed_attention_against_library_sdpa_with_explicit_mask():
    import torch
    rng = np.random.default_rng(8)
    cu, r, W, D = [0, 20, 53, 64], 3, 6, 8
    T = cu[-1]
    q, k, v = (rng.standard_normal((1, 1, T, D)) for _ in range(3))
    out, _ = oracle.attn_fwd(q, k, v, r, W, cu=cu)
    # mask written out pair by pair from the definition, not through the oracle's predicate
    m = torch.zeros(T, T, dtype=torch.bool)
    for i in range(T):
        for j in range(i + 1):
            d = max(c for c in cu[:-1] if c <= i)
            if j >= d and (((j - d + 1) % (r + 1) == 0) or i - j < W):
                m[i, j] = True
    ref = torch.nn.functional.scaled_dot_product_attention(*(torch.from_numpy(x) for x in (q, k, v)), attn_mask=m)
    assert np.allclose(out, ref.numpy(), atol=1e-12)
