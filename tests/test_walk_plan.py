"""The tile walks the kernels execute (Sec. 4.2), checked pair by pair against the oracle's mask on the CPU.

unigist_plan_row_tile, unigist_bwd_plan_build and unigist_plan_key_tile evaluate on the host the functions the
forward, dQ and dK/dV kernels call for every decision about which tiles to visit, skip or mask.  For every query
row of the benchmark shapes (a spread of row tiles for the 128K shape) the test paints the regions those plans
visit over the oracle's dense mask row and requires:
  * every visible pair lies in exactly one visited region of the forward walk, of the dQ walk and of the dK/dV
    walk (and no pair, visible or not, in more than one);
  * a region visited without the in-tile mask holds visible pairs only;
  * a skipped region holds no visible pair;
  * the partial-sum slots of the dK/dV gist phase are what the reduction assumes.
"""
from collections import defaultdict

import numpy as np
import pytest

import oracle
import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth

SKIP, FULL, MASKED = 0, 1, 2


def compact_positions(n, r, sinks):
    """Positions of the first n entries of the compact list: the sinks, then the gists (as the header states)."""
    c = np.arange(n, dtype=np.int64)
    return np.where(c < sinks, c, sinks + (c - sinks) * (r + 1) + r)


class KeySide:
    """All dK/dV workgroups of a shape, indexed by the query chunk they stream."""

    def __init__(self, B, Hq, Hkv, L, D, r, W, sinks, mode):
        self.bp = bp = u.unigist_bwd_plan_build(B, Hq, Hkv, L, D, r, W, sinks, mode)
        assert bp["key_tile"] == 128 and bp["chunk_rows"] == 64
        assert bp["n_chunks"] == -(-L // 64) and bp["n_key_tiles"] == -(-L // 128)
        self.gist = defaultdict(list)    # chunk -> [(tile, nfar of the chunk, kind [4, 2])]
        self.window = defaultdict(list)  # chunk -> [(tile, kind [4, 2])]
        segc, nseg, slot0 = bp["seg_chunks"], bp["n_segs"], bp["slot0"]
        assert slot0[0] == 0 and len(slot0) == nseg + 1 and nseg <= 32
        segs_of_tile = defaultdict(list)
        chunks_of = {}
        for sg in range(nseg):
            assert slot0[sg + 1] >= slot0[sg]
            for t in range(slot0[sg + 1] - slot0[sg]):
                p = u.unigist_plan_key_tile(B, Hq, Hkv, L, D, r, W, sinks, mode, 1, t, sg)
                chunks_of[(sg, t)] = (p["c_lo"], p["c_hi"])
                # a workgroup of the plan has work, inside its segment
                assert sg * segc <= p["c_lo"] <= p["c_hi"] < min((sg + 1) * segc, bp["n_chunks"]), (sg, t, p["c_lo"], p["c_hi"])
                segs_of_tile[t].append(sg)
                for n, c in enumerate(range(p["c_lo"], p["c_hi"] + 1)):
                    self.gist[c].append((t, int(p["nfar"][n]), p["kind"][:, n]))
        # launch order of the gist phase: every slot exactly once; either plain segment-major from the last segment
        # down, or the units that walk a whole segment first (in that order) and the shorter ones last, longest first
        order = [u.unigist_plan_gist_unit(B, Hq, Hkv, L, D, r, W, sinks, mode, n) for n in range(slot0[nseg])]
        assert sorted(order) == sorted(chunks_of)
        plain = [(sg, t) for sg in range(nseg - 1, -1, -1) for t in range(slot0[sg + 1] - slot0[sg])]
        if order != plain:
            whole = [chunks_of[x][0] == x[0] * segc for x in order]
            k = whole.index(False) if False in whole else len(order)
            assert not any(whole[k:]) and order[:k] == [x for x in plain if chunks_of[x][0] == x[0] * segc]
            lens = [chunks_of[x][1] - chunks_of[x][0] + 1 for x in order[k:]]
            assert lens == sorted(lens, reverse=True) and (not lens or lens[0] <= segc)
        self.reordered = order != plain
        # the reduction adds, for every compact tile, the slots of all segments from its first one to the last
        assert sorted(segs_of_tile) == list(range(bp["n_gist_tiles"]))
        for t, sgs in segs_of_tile.items():
            assert sgs == list(range(sgs[0], nseg)), (t, sgs)
        for t in range(bp["n_key_tiles"]):
            p = u.unigist_plan_key_tile(B, Hq, Hkv, L, D, r, W, sinks, mode, 0, t)
            assert p["c_lo"] == 2 * t and p["c_lo"] <= p["c_hi"] < bp["n_chunks"]
            for n, c in enumerate(range(p["c_lo"], p["c_hi"] + 1)):
                self.window[c].append((t, p["kind"][:, n]))
        per_block = 2 * D * 128 * 4
        assert bp["partial_bytes"] == B * Hkv * slot0[nseg] * per_block
        assert bp["reduced_bytes"] == B * Hkv * bp["n_gist_tiles"] * per_block
        a = lambda x: (x + 255) & ~255
        assert bp["workspace_bytes"] == 2 * a(B * Hq * L * 4) + a(bp["partial_bytes"]) + a(bp["reduced_bytes"])


def check_row_tile(M, i0, L, r, W, sinks, mode, kernel):
    """M: oracle mask of the rows i0 .. i0+127 (those below L) against all L keys."""
    p = u.unigist_plan_row_tile(L, r, W, sinks, mode, kernel, i0 // 128)
    Bm, Bn, rpw = p["Bm"], p["Bn"], p["rows_per_wave"]
    assert (Bm, rpw) == (128, 32) and Bn == (32 if kernel == u.UNIGIST_WALK_FWD else 64)
    nrows = M.shape[0]
    cover = np.zeros(M.shape, dtype=np.int8)
    ngt, nfar, kind = p["n_gist_steps"], p["nfar"], p["kind"]
    assert ngt == -(-nfar // Bn) and kind.shape == (4, ngt + p["n_window_steps"])
    pos = compact_positions(nfar, r, sinks)
    if nfar:
        assert pos.max() < p["wstart"] and M[:, pos].all()          # left of the window phase, visible to every row
        cover[:, pos] += 1
    for it in range(ngt):                                            # no mask <=> the step is full of far entries
        want = FULL if (it + 1) * Bn <= nfar else MASKED
        assert (kind[:, it] == want).all()
    for w in range(4):
        r0, r1 = w * 32, min(nrows, w * 32 + 32)
        if r0 >= nrows:
            continue
        for n in range(p["n_window_steps"]):
            j0 = p["wstart"] + n * Bn
            j1 = min(L, j0 + Bn)
            kd = kind[w, ngt + n]
            sub = M[r0:r1, j0:j1]
            if kd == SKIP:
                assert not sub.any()
                continue
            if kd == FULL:
                assert sub.all() and j1 - j0 == Bn
            cover[r0:r1, j0:j1] += 1
    # nothing right of the last window step may be visible (it is not: those keys are not causal)
    assert cover.max() <= 1
    assert (cover[M] == 1).all()


def check_chunk(M, c, L, r, sinks, ks):
    """M: oracle mask of the rows 64 c .. 64 c + 63 (those below L); ks: KeySide."""
    nrows = M.shape[0]
    cover = np.zeros(M.shape, dtype=np.int8)
    for tile, nfar, kind in ks.gist[c]:
        n_in = min(128, nfar - 128 * tile)
        assert n_in > 0                                              # the workgroup would not stream the chunk otherwise
        pos = compact_positions(128 * tile + n_in, r, sinks)[128 * tile:]
        assert M[:, pos].all()
        cover[:, pos] += 1
        for w in range(4):
            for qb in range(2):
                full = 128 * tile + 32 * w + 32 <= nfar and 64 * c + 32 * qb + 32 <= L
                assert kind[w, qb] == (FULL if full else MASKED)     # never skipped
    for tile, kind in ks.window[c]:
        for w in range(4):
            j0 = 128 * tile + 32 * w
            j1 = min(L, j0 + 32)
            if j0 >= L:
                continue
            for qb in range(2):
                r0, r1 = 32 * qb, min(nrows, 32 * qb + 32)
                if r0 >= nrows:
                    continue
                sub = M[r0:r1, j0:j1]
                if kind[w, qb] == SKIP:
                    assert not sub.any()
                    continue
                if kind[w, qb] == FULL:
                    assert sub.all() and j1 - j0 == 32 and r1 - r0 == 32
                cover[r0:r1, j0:j1] += 1
    assert cover.max() <= 1
    assert (cover[M] == 1).all()


def run_shape(B, Hq, Hkv, L, D, r, W, sinks, units, tiles):
    mode = int(units)
    ks = KeySide(B, Hq, Hkv, L, D, r, W, sinks, mode)
    for t in tiles:
        rows = np.arange(128 * t, min(L, 128 * t + 128))
        M = oracle.mask_rows(rows, L, r, W, sinks=sinks, units=units)
        check_row_tile(M, 128 * t, L, r, W, sinks, mode, u.UNIGIST_WALK_FWD)
        check_row_tile(M, 128 * t, L, r, W, sinks, mode, u.UNIGIST_WALK_DQ)
        for c in (2 * t, 2 * t + 1):
            if 64 * c < L:
                check_chunk(M[64 * c - 128 * t: 64 * c - 128 * t + 64], c, L, r, sinks, ks)
    return ks


def test_benchmark_shape_32k_every_row():
    c = synth.WORKLOADS["cfg2_llama8b_32k"]
    ks = run_shape(c["B"], c["Hq"], c["Hkv"], c["L"], c["D"], c["r"], c["W"], 0, False, range(c["L"] // 128))
    # the scratch of the backward: about half of the full (tile, segment) rectangle, and what the ABI reports
    bp = ks.bp
    assert bp["slot0"][-1] <= 0.55 * bp["n_gist_tiles"] * bp["n_segs"]
    assert bp["workspace_bytes"] == u.unigist_attn_bwd_workspace(c["B"], c["Hq"], c["Hkv"], c["L"], c["D"], c["r"], c["W"], 0)
    assert bp["workspace_bytes"] <= 510e6
    assert ks.reordered  # the short units of this shape fit the launch-order table


def test_long_context_128k_spread_of_tiles():
    c = synth.WORKLOADS["cfg3_long_128k"]
    n = c["L"] // 128
    tiles = sorted(set(list(range(0, 20)) + list(range(n - 3, n)) + list(range(20, n, 11))))
    ks = run_shape(c["B"], c["Hq"], c["Hkv"], c["L"], c["D"], c["r"], c["W"], 0, False, tiles)
    assert ks.bp["workspace_bytes"] == u.unigist_attn_bwd_workspace(c["B"], c["Hq"], c["Hkv"], c["L"], c["D"], c["r"], c["W"], 0)
    assert ks.bp["workspace_bytes"] <= 2.1e9


@pytest.mark.parametrize("r", synth.WORKLOADS["cfg4_ratio_sweep"]["r"])
def test_ratio_sweep(r):
    c = synth.WORKLOADS["cfg4_ratio_sweep"]
    n = c["L"] // 128
    tiles = range(n)
    run_shape(c["B"], c["Hq"], c["Hkv"], c["L"], c["D"], r, c["W"], 0, False, tiles)


# ragged lengths, windows shorter and longer than the tiles, sinks shorter and longer than a tile, unit windows,
# no gists, window over everything, many segments (L > 64 * 32 * 16 doubles the segment length)
SHAPES = [
    # B, Hq, Hkv, L, D, r, W, sinks, units
    (1, 4, 1, 5000, 128, 4, 129, 0, False),
    (2, 8, 8, 9001, 128, 2, 300, 0, False),
    (1, 2, 1, 4097, 64, 8, 1, 0, False),
    (1, 2, 1, 3000, 64, 4, 10 ** 6, 0, False),
    (1, 2, 2, 2500, 128, 10 ** 6, 333, 0, False),
    (1, 4, 1, 6000, 128, 4, 25, 128, True),
    (1, 4, 2, 7000, 128, 3, 1, 5, True),
    (1, 8, 2, 4500, 64, 4, 204, 300, True),
    (1, 4, 4, 3333, 128, 7, 64, 77, False),
    (1, 2, 1, 40000, 128, 16, 700, 0, False),
    (1, 2, 1, 63, 64, 1, 3, 0, False),
    (1, 1, 1, 1, 64, 4, 4, 0, False),
]


@pytest.mark.parametrize("B,Hq,Hkv,L,D,r,W,sinks,units", SHAPES)
def test_other_shapes(B, Hq, Hkv, L, D, r, W, sinks, units):
    n = -(-L // 128)
    tiles = range(n) if n <= 80 else sorted(set(list(range(12)) + list(range(n - 3, n)) + list(range(12, n, 7))))
    run_shape(B, Hq, Hkv, L, D, r, W, sinks, units, tiles)


def test_launch_order_falls_back_to_segment_major_when_the_short_units_do_not_fit_the_table():
    # ratio 1 at 196 608 tokens: 128-chunk segments, each first reaching 17 compact tiles inside it -- more short
    # units than the 512 the plan carries, so the gist phase is launched in plain segment-major order
    B, Hq, Hkv, L, D, r, W = 1, 2, 1, 196608, 64, 1, 64
    bp = u.unigist_bwd_plan_build(B, Hq, Hkv, L, D, r, W)
    nseg, slot0 = bp["n_segs"], bp["slot0"]
    plain = [(sg, t) for sg in range(nseg - 1, -1, -1) for t in range(slot0[sg + 1] - slot0[sg])]
    assert len(plain) == slot0[nseg] > 9000
    for n in list(range(0, len(plain), 37)) + [len(plain) - 1]:
        assert u.unigist_plan_gist_unit(B, Hq, Hkv, L, D, r, W, 0, 0, n) == plain[n]
    # half the length fits: a permutation that is not the plain order
    L = 98304
    bp = u.unigist_bwd_plan_build(B, Hq, Hkv, L, D, r, W)
    nseg, slot0 = bp["n_segs"], bp["slot0"]
    plain = [(sg, t) for sg in range(nseg - 1, -1, -1) for t in range(slot0[sg + 1] - slot0[sg])]
    order = [u.unigist_plan_gist_unit(B, Hq, Hkv, L, D, r, W, 0, 0, n) for n in range(slot0[nseg])]
    assert sorted(order) == sorted(plain) and order != plain


def test_closed_forms_of_the_sliding_mode_agree_with_the_search():
    # In the sliding mode the first and last chunk of a dK/dV workgroup come from closed forms, in the unit mode from
    # a binary search over the monotone far(c).  A unit window of W units and r = 1 ... is not a sliding window, so
    # the two branches are compared through what they must both satisfy: the chunk ranges of the window phase
    # partition, for every chunk, the key tiles from far(c) to the diagonal.
    for (L, r, W) in [(32768, 4, 1024), (16384, 32, 1024), (9001, 2, 300), (5000, 4, 129), (4097, 8, 1)]:
        bp = u.unigist_bwd_plan_build(1, 4, 1, L, 128, r, W)
        first = {}
        last = {}
        for t in range(bp["n_key_tiles"]):
            p = u.unigist_plan_key_tile(1, 4, 1, L, 128, r, W, 0, 0, 0, t)
            for c in range(p["c_lo"], p["c_hi"] + 1):
                first.setdefault(c, t)
                last[c] = t
        for c in range(bp["n_chunks"]):
            far = (max(0, 64 * c - W + 1) // 128) * 128          # first key of the chunk's window phase
            assert first[c] == far // 128 and last[c] == (64 * c) // 128, (L, r, W, c)
