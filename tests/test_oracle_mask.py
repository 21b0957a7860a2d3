"""Pins for the oracle's layout and mask predicate (Sec. 4.1, Eq. 2 and Eq. 3)."""
import os

import numpy as np
import pytest

import oracle
from conftest import GOLDEN


def _read_rows(path):
    with open(path) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


def test_hand_derived_visible_sets():
    rows = _read_rows(os.path.join(GOLDEN, "visible_sets_L10_r4_W3.txt"))
    M = oracle.mask_rows(np.arange(10), 10, 4, 3)
    assert len(rows) == 10
    for ln in rows:
        i, keys = ln.split(":")
        want = sorted(int(t) for t in keys.split())
        got = np.nonzero(M[int(i)])[0].tolist()
        assert got == want, (i, got, want)


def test_gist_positions_follow_eq2():
    # r raw tokens then one gist, repeated; trailing partial unit has no gist
    r, L = 4, 23
    layout = []
    while len(layout) < L:
        layout += ["x"] * r + ["g"]
    layout = layout[:L]
    got = oracle.is_gist(np.arange(L), r)
    assert got.tolist() == [c == "g" for c in layout]
    assert int(got.sum()) == L // (r + 1)


@pytest.mark.parametrize("line", _read_rows(os.path.join(GOLDEN, "n_vis_closed_form.txt")))
def test_pair_counts_match_closed_form(line):
    L, r, W, want = (int(t) for t in line.split())
    if L > 40000:
        # 1.7e10 pairs is too slow pair by pair: count per row on a strided row sample
        # and compare each row with the closed form instead.
        rows = np.unique(np.concatenate([np.arange(0, L, 997), [W - 1, W, W + r, L - 1]]))
        M = oracle.mask_rows(rows, L, r, W)
        got = M.sum(axis=1)
        wantrow = np.minimum(rows + 1, W) + np.maximum(0, (rows - W + 1) // (r + 1))
        assert np.array_equal(got, wantrow)
        return
    assert oracle.count_visible(L, r, W) == want


def test_window_covering_everything_is_causal():
    L = 97
    for W in (L, L + 5, 10**9):
        M = oracle.mask_rows(np.arange(L), L, 4, W)
        assert np.array_equal(M, np.tril(np.ones((L, L), dtype=bool)))


def test_no_gists_is_a_band():
    L, W = 101, 7
    for r in (L, L + 3, 2**31 - 1):
        M = oracle.mask_rows(np.arange(L), L, r, W)
        band = np.tril(np.ones((L, L), dtype=bool)) & ~np.tril(np.ones((L, L), dtype=bool), -W)
        assert np.array_equal(M, band)


def test_every_row_sees_itself_and_is_causal():
    L = 64
    for r, W in [(1, 1), (4, 1), (4, 5), (8, 17), (3, 64)]:
        M = oracle.mask_rows(np.arange(L), L, r, W)
        assert M.diagonal().all()
        assert not np.triu(M, 1).any()
        # every earlier gist is visible, every raw key outside the window is not
        g = oracle.is_gist(np.arange(L), r)
        for i in range(L):
            for j in range(i + 1):
                assert M[i, j] == (g[j] or i - j < W)


def test_compressed_cache_positions():
    # t = 9 in the micro-example sees {4, 7, 8, 9}
    assert oracle.compressed_cache_positions(9, 4, 3).tolist() == [4, 7, 8, 9]
    # cache size = window + gists left of it
    t, r, W = 147455, 8, 1024
    pos = oracle.compressed_cache_positions(t, r, W)
    assert len(pos) == W + (t - W + 1) // (r + 1)


def test_cache_state_holds_the_visible_set():
    # state (s, t) with s at the window start of query t holds exactly what query t may see (Eq. 3),
    # and a later window start only ever drops raw tokens
    for r, W in [(4, 3), (4, 16), (8, 5), (2, 1)]:
        for t in (0, 1, 7, 40, 123):
            s = max(0, t - W + 1)
            assert np.array_equal(oracle.cache_positions(s, t, r), oracle.compressed_cache_positions(t, r, W))
            wide = oracle.cache_positions(max(0, s - 5), t, r)
            dropped = np.setdiff1d(wide, oracle.cache_positions(s, t, r))
            assert not oracle.is_gist(dropped, r).any()
    assert oracle.cache_positions(5, 9, 4).tolist() == [4, 5, 6, 7, 8, 9]
    assert oracle.cache_positions(0, -1, 4).tolist() == []


def test_hand_derived_visible_sets_with_sinks_and_unit_window():
    rows = _read_rows(os.path.join(GOLDEN, "visible_sets_L14_r2_sinks2_units1.txt"))
    M = oracle.mask_rows(np.arange(14), 14, 2, 1, sinks=2, units=True)
    assert len(rows) == 14
    for ln in rows:
        i, keys = ln.split(":")
        assert np.nonzero(M[int(i)])[0].tolist() == sorted(int(t) for t in keys.split()), i


def test_unit_window_is_sandwiched_between_sliding_windows():
    # current unit + k previous units covers at least k(r+1)+1 and at most (k+1)(r+1) positions
    L = 150
    for r, k in [(4, 1), (4, 3), (2, 0), (8, 2)]:
        U = oracle.mask_rows(np.arange(L), L, r, k, units=True)
        small = oracle.mask_rows(np.arange(L), L, r, k * (r + 1) + 1)
        big = oracle.mask_rows(np.arange(L), L, r, (k + 1) * (r + 1))
        assert not (small & ~U).any() and not (U & ~big).any()
        # rows at the end of a unit (gist queries) see exactly (k+1)(r+1) window positions
        g = np.nonzero(oracle.is_gist(np.arange(L), r))[0]
        assert np.array_equal(U[g], big[g])


def test_sinks_are_always_visible_and_shift_the_layout():
    L, r, S = 60, 4, 3
    g = oracle.is_gist(np.arange(L), r, sinks=S)
    assert np.nonzero(g)[0].tolist() == list(range(S + r, L, r + 1))
    for units, W in [(False, 6), (True, 1)]:
        M = oracle.mask_rows(np.arange(L), L, r, W, sinks=S, units=units)
        assert M[:, :S].sum() == sum(min(i + 1, S) for i in range(L))      # every later row sees every sink
        assert M.diagonal().all() and not np.triu(M, 1).any()
        # with the sinks cut off the pattern is the sink-free one
        assert np.array_equal(M[S:, S:], oracle.mask_rows(np.arange(L - S), L - S, r, W, units=units))
    # a huge unit window is plain causal attention
    assert np.array_equal(oracle.mask_rows(np.arange(L), L, r, 10**6, sinks=S, units=True), np.tril(np.ones((L, L), bool)))


# ---------------------------------------------------------------- packed documents (cu=)
def test_packed_hand_derived_visible_sets():
    rows = _read_rows(os.path.join(GOLDEN, "visible_sets_packed_T11_r2_W2.txt"))
    M = oracle.mask_rows(np.arange(11), 11, 2, 2, cu=[0, 4, 11])
    assert len(rows) == 11
    for ln in rows:
        i, keys = ln.split(":")
        assert np.nonzero(M[int(i)])[0].tolist() == sorted(int(t) for t in keys.split()), i


@pytest.mark.parametrize("cu,r,W", [([0, 5, 5, 17, 18, 40], 3, 4), ([0, 64], 4, 9), ([0, 1, 2, 3], 1, 1),
                                     ([0, 30, 61, 100], 4, 10**6), ([0, 33, 77], 10**6, 5)])
def test_packed_mask_is_block_diagonal_of_the_single_document_masks(cu, r, W):
    T = cu[-1]
    M = oracle.mask_rows(np.arange(T), T, r, W, cu=cu)
    want = np.zeros((T, T), dtype=bool)
    for a, b in zip(cu[:-1], cu[1:]):
        if b > a:
            want[a:b, a:b] = oracle.mask_rows(np.arange(b - a), b - a, r, W)
    assert np.array_equal(M, want)
    # one document is the plain mask; every query sees itself
    assert np.array_equal(oracle.mask_rows(np.arange(T), T, r, W, cu=[0, T]), oracle.mask_rows(np.arange(T), T, r, W))
    assert M.diagonal().all()


@pytest.mark.parametrize("cu,r,W,sinks", [([0, 5, 5, 17, 18, 40], 3, 1, 2), ([0, 30, 61, 100], 4, 2, 7),
                                           ([0, 3, 40], 2, 3, 5)])
def test_packed_mask_with_sinks_and_unit_windows_restarts_in_every_document(cu, r, W, sinks):
    # Sec. 4.1's layout inside every document of a pack (Sec. 5.1): each document has its own sinks (a document
    # shorter than the sink prefix is all sinks, i.e. plain causal) and its own gist units
    T = cu[-1]
    M = oracle.mask_rows(np.arange(T), T, r, W, cu=cu, sinks=sinks, units=True)
    want = np.zeros((T, T), dtype=bool)
    for a, b in zip(cu[:-1], cu[1:]):
        if b > a:
            want[a:b, a:b] = oracle.mask_rows(np.arange(b - a), b - a, r, W, sinks=sinks, units=True)
            if b - a <= sinks:
                assert np.array_equal(want[a:b, a:b], np.tri(b - a, dtype=bool))
    assert np.array_equal(M, want)
    # the first `sinks` positions of a document are seen by all of its later queries and by no other document's
    for a, b in zip(cu[:-1], cu[1:]):
        n = min(sinks, b - a)
        assert M[b - 1:b, a:a + n].all() if b > a else True
        assert not M[b:, a:a + n].any()


def test_cache_state_with_sinks_and_unit_windows():
    # the worked example with 2 sinks and unit windows (tests/golden/visible_sets_L14_r2_sinks2_units1.txt):
    # query 12 sees 0 1 4 7 8 9 10 11 12; its window starts at position 8, so state (8, 12) holds exactly that
    assert oracle.cache_positions(8, 12, 2, sinks=2).tolist() == [0, 1, 4, 7, 8, 9, 10, 11, 12]
    assert oracle.compressed_cache_positions(12, 2, 1, sinks=2, units=True).tolist() == [0, 1, 4, 7, 8, 9, 10, 11, 12]
    for r, k, sinks in [(2, 1, 2), (4, 3, 5), (3, 2, 0), (4, 1, 40)]:
        for t in (0, 1, sinks, sinks + 1, 30, 77):
            vis = oracle.compressed_cache_positions(t, r, k, sinks=sinks, units=True)
            s = t if t < sinks else sinks + max(0, (t - sinks) // (r + 1) - k) * (r + 1)   # first position of t's window
            assert np.array_equal(oracle.cache_positions(s, t, r, sinks=sinks), vis)
            # starting the window region earlier only adds raw tokens
            wide = oracle.cache_positions(max(0, s - 4), t, r, sinks=sinks)
            extra = np.setdiff1d(wide, vis)
            assert not (oracle.is_gist(extra, r, sinks) | (extra < sinks)).any()
