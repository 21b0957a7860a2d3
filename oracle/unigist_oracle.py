"""Plain fp64 definition of UniGist's gist-masked causal attention (CPU, numpy).

THIS IS TEST INFRASTRUCTURE.  It is the yardstick the HIP kernels are compared
against; it is slow on purpose, shares no code with the kernels and must never
be imported by the product package.

What it follows
---------------
* Sequence layout: the gist-augmented sequence of Sec. 4.1, Eq. 2: an optional
  prefix of sink tokens, then r raw tokens, one gist, r raw tokens, one gist, ...
  With 0-based positions and no sinks a position p holds a gist iff
  (p + 1) % (r + 1) == 0.  A trailing group of fewer than r raw tokens has no
  closing gist.
* Visible set: Sec. 4.1, Eq. 3 -- (gists U local window) intersected with the
  causal set {j <= t}, the same rule for raw and gist queries.  The local window
  is read as a per-token sliding window counted in interleaved positions:
  key j is inside the window of query i iff 0 <= i - j < W.  (The paper words the
  window in whole gist units; the sliding reading is the one the workload
  definitions of this build fix.  The unit-aligned wording and the sink prefix are
  available through the keyword arguments sinks= and units=True.)
* Everything else is ordinary softmax attention: S = Q K^T / sqrt(D), masked
  entries are -inf, P = softmax over keys, out = P V, lse = ln sum_j exp(S_ij).
  The gradients are the exact derivative of l = sum(out * dout).
* Packed documents (Sec. 5.1, cross-document masking): with the keyword cu=boundaries the predicate
  additionally requires query and key to lie in the same document and counts positions from the
  document's first token.
* Decode (Sec. 4.3, "Inference"): one query over a cache from which the
  invisible raw tokens have already been removed, so every cached key counts.

There is no tiling, no skipping and no reordering here.  Long sequences are
handled a block of query rows at a time purely so that the L x L score matrix
is never resident; every row is still scored against every key it is allowed
to be scored against and masked by evaluating the predicate pair by pair.

Pins (tests/test_oracle_*.py): hand-derived visible sets, closed-form pair
counts, brute-force loops on tiny inputs, W >= L == causal library attention,
r >= L == banded library attention, q == 0 closed form, finite differences,
library autograd.
"""
from __future__ import annotations

import math
import numpy as np

__all__ = [
    "is_gist", "visible", "mask_rows", "count_visible",
    "attn_fwd_head", "attn_bwd_head", "attn_fwd", "attn_bwd",
    "attn_fwd_rows", "attn_dq_rows", "attn_dkdv_cols", "decode", "compressed_cache_positions",
    "cache_positions",
]


# --------------------------------------------------------------------------
# layout and mask (Eq. 2, Eq. 3)
# --------------------------------------------------------------------------
def is_gist(p, r, sinks=0):
    """True where 0-based position p holds a gist token (Eq. 2): after `sinks` sink tokens the
    sequence repeats r raw tokens followed by one gist.

    r is the compression ratio (raw tokens per gist).  Python ints are used for
    r + 1 so that a huge r ("no gists at all") cannot overflow.
    """
    p = np.asarray(p, dtype=np.int64)
    period = int(r) + 1
    return (p >= sinks) & ((p - sinks + 1) % period == 0)


def visible(i, j, r, W, sinks=0, units=False):
    """Eq. 3: may query i attend to key j?  Key j must be causal and be a sink, a gist, or inside the
    local window of i.

    units=False: the window is the W most recent positions (sliding per token) -- the reading the
    workloads of this build use.  units=True: the window is worded as in Sec. 4.1: the gist unit that
    contains i plus the W previous gist units (a unit = r raw tokens and the gist that follows them).
    Sink queries (i < sinks) belong to no unit; they see the sinks up to themselves.
    """
    i = np.asarray(i, dtype=np.int64)
    j = np.asarray(j, dtype=np.int64)
    causal = j <= i
    if units:
        period = int(r) + 1
        unit_i = (i - sinks) // period
        unit_j = (j - sinks) // period
        in_window = (i >= sinks) & (j >= sinks) & (unit_j >= unit_i - int(W))
    else:
        in_window = (i - j) < int(W)
    return causal & ((j < sinks) | is_gist(j, r, sinks) | in_window)


def mask_rows(rows, L, r, W, cu=None, **mask):
    """Boolean [len(rows), L] matrix of visible(i, j) for the given query rows.

    cu (optional): document boundaries of a packed sequence, cu[0] = 0 <= cu[1] <= ... <= cu[-1] = L.
    Then attention never crosses a boundary (cross-document masking, Sec. 5.1) and inside a document
    the rule is the one above with positions counted from the document's first token, so the gist
    period and the window restart there.
    """
    rows = np.asarray(rows, dtype=np.int64)
    cols = np.arange(L, dtype=np.int64)
    if cu is None:
        return visible(rows[:, None], cols[None, :], r, W, **mask)
    cu = np.asarray(cu, dtype=np.int64)
    doc_r = np.searchsorted(cu, rows, side="right") - 1   # the document holding each position
    doc_c = np.searchsorted(cu, cols, side="right") - 1
    same = doc_r[:, None] == doc_c[None, :]
    return same & visible((rows - cu[doc_r])[:, None], (cols - cu[doc_c])[None, :], r, W, **mask)


def count_visible(L, r, W, block=1024, **mask):
    """Number of visible (i, j) pairs, by evaluating the predicate on every pair."""
    total = 0
    for i0 in range(0, L, block):
        rows = np.arange(i0, min(L, i0 + block))
        total += int(np.count_nonzero(mask_rows(rows, L, r, W, **mask)))
    return total


# --------------------------------------------------------------------------
# one head, a set of query rows against all keys
# --------------------------------------------------------------------------
def _softmax_rows(q_rows, k, rows, r, W, **mask):
    """Scores, mask and softmax of the given query rows against every key.

    Returns P [n, L] and lse [n]; masked entries of P are exactly 0.
    """
    L, D = k.shape
    S = (q_rows @ k.T) / math.sqrt(D)
    M = mask_rows(rows, L, r, W, **mask)
    S = np.where(M, S, -np.inf)
    m = S.max(axis=1)
    E = np.exp(S - m[:, None])
    Z = E.sum(axis=1)
    P = E / Z[:, None]
    lse = m + np.log(Z)
    return P, lse


def attn_fwd_head(q, k, v, r, W, block=512, **mask):
    """Forward for one head.  q, k, v: float64 [L, D].  Returns out [L, D], lse [L]."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    L = q.shape[0]
    out = np.empty((L, v.shape[1]))
    lse = np.empty(L)
    for i0 in range(0, L, block):
        rows = np.arange(i0, min(L, i0 + block))
        P, lse[rows] = _softmax_rows(q[rows], k, rows, r, W, **mask)
        out[rows] = P @ v
    return out, lse


def attn_bwd_head(q, k, v, dout, r, W, block=512, row_lo=0, row_hi=None, **mask):
    """Gradients of l = sum(out * dout) for one head.

    dV_j = sum_i P_ij dO_i;  dP_ij = dO_i . v_j;  delta_i = sum_j P_ij dP_ij;
    dS_ij = P_ij (dP_ij - delta_i);  dQ_i = sum_j dS_ij k_j / sqrt(D);
    dK_j = sum_i dS_ij q_i / sqrt(D).
    Returns dq, dk, dv (all [L, D]).  With row_lo/row_hi only those query rows are
    processed: dq is filled for them (zero elsewhere) and dk, dv hold their share of the sums.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    L, D = q.shape
    row_hi = L if row_hi is None else row_hi
    inv = 1.0 / math.sqrt(D)
    dq = np.zeros((L, D))
    dk = np.zeros((L, D))
    dv = np.zeros((L, D))
    for i0 in range(row_lo, row_hi, block):
        rows = np.arange(i0, min(row_hi, i0 + block))
        P, _ = _softmax_rows(q[rows], k, rows, r, W, **mask)
        dO = dout[rows]
        dv += P.T @ dO
        dP = dO @ v.T
        delta = (P * dP).sum(axis=1)
        dS = P * (dP - delta[:, None])
        dq[rows] = (dS @ k) * inv
        dk += (dS.T @ q[rows]) * inv
    return dq, dk, dv


# --------------------------------------------------------------------------
# [B, H, L, D] tensors with grouped-query heads
# --------------------------------------------------------------------------
def _kv_head(h, Hq, Hkv):
    assert Hq % Hkv == 0
    return h // (Hq // Hkv)


def attn_fwd(q, k, v, r, W, block=512, **mask):
    """q [B,Hq,L,D], k/v [B,Hkv,L,D]  ->  out [B,Hq,L,D], lse [B,Hq,L] (float64)."""
    q = np.asarray(q, dtype=np.float64)
    B, Hq, L, D = q.shape
    Hkv = k.shape[1]
    out = np.empty((B, Hq, L, D))
    lse = np.empty((B, Hq, L))
    for b in range(B):
        for h in range(Hq):
            g = _kv_head(h, Hq, Hkv)
            out[b, h], lse[b, h] = attn_fwd_head(q[b, h], k[b, g], v[b, g], r, W, block, **mask)
    return out, lse


def attn_bwd(q, k, v, dout, r, W, block=512, **mask):
    """Returns dq [B,Hq,L,D], dk, dv [B,Hkv,L,D]; dk/dv summed over the q heads of a group."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    B, Hq, L, D = q.shape
    Hkv = k.shape[1]
    dq = np.empty((B, Hq, L, D))
    dk = np.zeros((B, Hkv, L, D))
    dv = np.zeros((B, Hkv, L, D))
    for b in range(B):
        for h in range(Hq):
            g = _kv_head(h, Hq, Hkv)
            dq[b, h], dk_h, dv_h = attn_bwd_head(q[b, h], k[b, g], v[b, g], dout[b, h], r, W, block, **mask)
            dk[b, g] += dk_h
            dv[b, g] += dv_h
    return dq, dk, dv


# --------------------------------------------------------------------------
# sampled rows (out, lse and dq of a row depend on that row of q/dout only)
# --------------------------------------------------------------------------
def attn_fwd_rows(q, k, v, rows, r, W, **mask):
    """One head: out and lse for a chosen set of query rows.  q, k, v [L, D]."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    P, lse = _softmax_rows(q[rows], k, rows, r, W, **mask)
    return P @ v, lse


def attn_dq_rows(q, k, v, dout, rows, r, W, **mask):
    """One head: dq for a chosen set of query rows."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    D = q.shape[1]
    P, _ = _softmax_rows(q[rows], k, rows, r, W, **mask)
    dP = dout[rows] @ v.T
    delta = (P * dP).sum(axis=1)
    dS = P * (dP - delta[:, None])
    return (dS @ k) / math.sqrt(D)


def attn_dkdv_cols(q, k, v, dout, cols, r, W, row_lo=0, row_hi=None, block=512, **mask):
    """One query head: what the query rows row_lo .. row_hi-1 add to dK and dV of the chosen key
    columns.  Same formulas as attn_bwd_head, with the sums over i restricted to those rows and
    only the requested columns of dS and P kept.  Summing the results over disjoint row ranges
    that cover 0 .. L-1 (and over the query heads of a group) gives dK[cols], dV[cols]."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    cols = np.asarray(cols, dtype=np.int64)
    L, D = q.shape
    row_hi = L if row_hi is None else row_hi
    dk = np.zeros((len(cols), D))
    dv = np.zeros((len(cols), D))
    for i0 in range(row_lo, row_hi, block):
        rows = np.arange(i0, min(row_hi, i0 + block))
        P, _ = _softmax_rows(q[rows], k, rows, r, W, **mask)
        dO = dout[rows]
        dP = dO @ v.T
        delta = (P * dP).sum(axis=1)
        Pc = P[:, cols]
        dSc = Pc * (dP[:, cols] - delta[:, None])
        dv += Pc.T @ dO
        dk += (dSc.T @ q[rows]) / math.sqrt(D)
    return dk, dv


# --------------------------------------------------------------------------
# decode over the compressed cache (Sec. 4.3)
# --------------------------------------------------------------------------
def compressed_cache_positions(t, r, W, **mask):
    """Positions a cache holds when position t is the query (Fig. 4): every sink and gist
    up to t plus the raw tokens still inside t's window.  Ascending order."""
    j = np.arange(t + 1, dtype=np.int64)
    return j[visible(np.int64(t), j, r, W, **mask)]


def cache_positions(s, t, r, sinks=0):
    """Positions a compressed cache in state (s, t) holds, in row order (Sec. 4.3, Fig. 4): the sinks and
    gists that lie left of position s, then every position s .. t.  With s the first position of query
    t's window this is the visible set of query t."""
    j = np.arange(t + 1, dtype=np.int64)
    keep = (j >= s) | (j < sinks) | is_gist(j, r, sinks)
    return j[keep]


def decode(q, kcache, vcache, seqlens=None):
    """q [B,Hq,D]; kcache, vcache [B,Hkv,Lk,D]; seqlens [B] or None (= all Lk).

    Every cached key of a sequence is visible.  Returns out [B,Hq,D], lse [B,Hq].
    """
    q = np.asarray(q, dtype=np.float64)
    kcache = np.asarray(kcache, dtype=np.float64)
    vcache = np.asarray(vcache, dtype=np.float64)
    B, Hq, D = q.shape
    Hkv, Lk = kcache.shape[1], kcache.shape[2]
    out = np.empty((B, Hq, D))
    lse = np.empty((B, Hq))
    for b in range(B):
        n = Lk if seqlens is None else int(seqlens[b])
        for h in range(Hq):
            g = _kv_head(h, Hq, Hkv)
            s = (kcache[b, g, :n] @ q[b, h]) / math.sqrt(D)
            m = s.max()
            e = np.exp(s - m)
            z = e.sum()
            out[b, h] = (e / z) @ vcache[b, g, :n]
            lse[b, h] = m + math.log(z)
    return out, lse
