"""GPU parity of the compressed-cache maintenance and the chunk-wise prefill (Sec. 4.3, Fig. 4) against
the oracle: the cache after any sequence of appends/evictions equals a direct gather of the positions the
oracle says the state holds (bit-exact); every prefill chunk equals the same rows of the one-pass
attention over the whole sequence; decode on the cache left by the prefill equals the last row."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth
from _parity import TOL_LSE_BF16, TOL_OUT_BF16, max_abs, out_ok, to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32], ids=["bf16", "f32"])
@pytest.mark.parametrize("B,Hkv,D,r,L", [(2, 2, 128, 4, 700), (1, 3, 64, 8, 513), (1, 1, 128, 1, 64), (2, 1, 64, 10**6, 300),
                                          (2, 2, 96, 4, 700), (1, 1, 8, 2, 300)])
def test_cache_updates_are_exact_gathers(B, Hkv, D, r, L, dtype):
    print("case", B, Hkv, D, r, L, dtype, flush=True)
    _, k, v, _ = synth.attn_inputs(B, Hkv, Hkv, L, D, dtype=dtype, seed=21)
    kd, vd = k.cuda(), v.cuda()
    cache = u.KVCache(B, Hkv, L, D, r, dtype=dtype)
    rng = np.random.default_rng(5)
    steps = 0
    while cache.t < L - 1:
        n = int(min(L - 1 - cache.t, rng.choice([0, 1, 3, 64, 200])))
        s_new = int(rng.integers(cache.s, cache.t + n + 2))     # anywhere up to "keep gists only"
        lo, hi = cache.t + 1, cache.t + 1 + n
        cache.update(kd[:, :, lo:hi].contiguous() if n else None, vd[:, :, lo:hi].contiguous() if n else None, s_new)
        pos = torch.from_numpy(oracle.cache_positions(cache.s, cache.t, r))
        assert cache.rows == len(pos)
        assert torch.equal(cache.kc[:, :, :cache.rows].cpu(), k[:, :, pos])
        assert torch.equal(cache.vc[:, :, :cache.rows].cpu(), v[:, :, pos])
        steps += 1
    assert steps >= 1


@pytest.mark.parametrize("B,Hq,Hkv,L,D,r,W,C", [
    (1, 4, 1, 3000, 128, 4, 256, 512),      # several chunks, window shorter than a chunk
    (2, 4, 2, 2500, 128, 8, 1024, 1000),    # ragged last chunk, window longer than a chunk
    (1, 2, 2, 1100, 64, 4, 100, 300),       # D = 64
    (1, 2, 1, 900, 128, 2**31 - 2, 50, 256),  # no gists
    (2, 4, 2, 2000, 96, 4, 256, 512),       # head dimension 96
    (1, 2, 1, 1100, 24, 4, 100, 300),       # ... and 24
])
def test_chunkwise_prefill_equals_one_pass(B, Hq, Hkv, L, D, r, W, C):
    case = f"B{B} Hq{Hq} Hkv{Hkv} L{L} D{D} r{r} W{W} C{C}"
    print("case", case, flush=True)
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, L, D, seed=22)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    full_out, full_lse = u.attn_fwd(qd, kd, vd, r, W)
    cap = u.unigist_cache_rows(0, L - 1, r)                # generous: nothing would need to be dropped
    cache = u.KVCache(B, Hkv, cap, D, r)
    outs, lses, max_rows = [], [], 0
    for p0 in range(0, L, C):
        n = min(C, L - p0)
        # append the chunk's keys, drop what no query of this chunk (or later) can see any more
        cache.update(kd[:, :, p0:p0 + n].contiguous(), vd[:, :, p0:p0 + n].contiguous(), max(0, p0 - W + 1))
        max_rows = max(max_rows, cache.rows)
        o, l = u.prefill_chunk(qd[:, :, p0:p0 + n].contiguous(), cache, r, W, p0)
        outs.append(o)
        lses.append(l)
    out, lse = torch.cat(outs, dim=2), torch.cat(lses, dim=2)
    torch.cuda.synchronize()
    # same kernel, same visible sets: only the order of the key tiles may differ
    assert max_abs(to_np(out), to_np(full_out)) <= 1.6e-2 and max_abs(to_np(lse), to_np(full_lse)) <= 1e-4
    # against the oracle on sampled rows of the whole sequence
    rows = np.unique(np.concatenate([[0, C - 1, C, min(L - 1, C + 1), L - 1], np.random.default_rng(1).integers(0, L, 24)]))
    for b, h in [(0, 0), (B - 1, Hq - 1)]:
        g = h // (Hq // Hkv)
        o, l = oracle.attn_fwd_rows(to_np(q[b, h]), to_np(k[b, g]), to_np(v[b, g]), rows, r, W)
        assert max_abs(to_np(out[b, h])[rows], o) <= TOL_OUT_BF16, case
        assert max_abs(to_np(lse[b, h])[rows], l) <= TOL_LSE_BF16, case
    # the cache never held more than window + chunk + gists rows
    assert max_rows <= W + C + L // (min(r, L) + 1) + 1
    # decode the last position on the cache the prefill left behind, evicted down to its window
    t = L - 1
    cache.update(None, None, max(0, t - W + 1))
    sl = torch.full((B,), cache.rows, dtype=torch.int32, device="cuda")
    o2, l2 = u.decode(qd[:, :, t].contiguous(), cache.kc, cache.vc, sl)
    od, ld = oracle.decode(to_np(q[:, :, t]), to_np(cache.kc[:, :, :cache.rows]), to_np(cache.vc[:, :, :cache.rows]))
    assert max_abs(to_np(o2), od) <= TOL_OUT_BF16 and max_abs(to_np(l2), ld) <= TOL_LSE_BF16
    assert max_abs(to_np(o2), to_np(full_out[:, :, t])) <= 1.6e-2


def _window_start(i, r, W, sinks, units):
    if not units:
        return max(0, i - W + 1)
    if i < sinks:
        return i
    return sinks + max(0, (i - sinks) // (r + 1) - W) * (r + 1)


@pytest.mark.parametrize("B,Hkv,D,r,L,sinks", [(2, 2, 128, 4, 700, 5), (1, 3, 64, 8, 513, 128), (1, 1, 128, 1, 64, 70)])
def test_cache_updates_with_sinks_are_exact_gathers(B, Hkv, D, r, L, sinks):
    _, k, v, _ = synth.attn_inputs(B, Hkv, Hkv, L, D, seed=23)
    kd, vd = k.cuda(), v.cuda()
    cache = u.KVCache(B, Hkv, L, D, r, sinks=sinks)
    rng = np.random.default_rng(6)
    while cache.t < L - 1:
        n = int(min(L - 1 - cache.t, rng.choice([0, 1, 3, 64, 200])))
        s_new = int(rng.integers(cache.s, cache.t + n + 2))
        lo, hi = cache.t + 1, cache.t + 1 + n
        cache.update(kd[:, :, lo:hi].contiguous() if n else None, vd[:, :, lo:hi].contiguous() if n else None, s_new)
        pos = torch.from_numpy(oracle.cache_positions(cache.s, cache.t, r, sinks=sinks))
        assert cache.rows == len(pos)
        assert torch.equal(cache.kc[:, :, :cache.rows].cpu(), k[:, :, pos])
        assert torch.equal(cache.vc[:, :, :cache.rows].cpu(), v[:, :, pos])


@pytest.mark.parametrize("B,Hq,Hkv,L,D,r,W,C,sinks,units", [
    (1, 4, 1, 3000, 128, 4, 25, 512, 128, True),     # the paper's setting in small: 128 sinks, window of 25 units
    (2, 4, 2, 2500, 128, 8, 110, 1000, 7, True),     # window longer than a chunk
    (1, 2, 2, 1100, 64, 4, 100, 300, 33, False),     # sinks with the sliding window, D = 64
    (1, 2, 1, 900, 128, 4, 3, 256, 300, True),       # the first chunk lies inside the sinks
    (1, 4, 2, 1500, 96, 4, 25, 400, 128, True),      # head dimension 96
])
def test_chunkwise_prefill_with_sinks_equals_one_pass(B, Hq, Hkv, L, D, r, W, C, sinks, units):
    case = f"B{B} Hq{Hq} Hkv{Hkv} L{L} D{D} r{r} W{W} C{C} sinks{sinks} units{int(units)}"
    print("case", case, flush=True)
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, L, D, seed=24)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    cache = u.KVCache(B, Hkv, L, D, r, sinks=sinks)
    outs, lses = [], []
    for p0 in range(0, L, C):
        n = min(C, L - p0)
        cache.update(kd[:, :, p0:p0 + n].contiguous(), vd[:, :, p0:p0 + n].contiguous(), _window_start(p0, r, W, sinks, units))
        o, l = u.prefill_chunk(qd[:, :, p0:p0 + n].contiguous(), cache, r, W, p0, window_mode=int(units))
        outs.append(o)
        lses.append(l)
    out, lse = torch.cat(outs, dim=2), torch.cat(lses, dim=2)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, sinks - 1, sinks, C - 1, C, min(L - 1, C + 1), L - 1],
                                     np.random.default_rng(2).integers(0, L, 24)]))
    for b, h in [(0, 0), (B - 1, Hq - 1)]:
        g = h // (Hq // Hkv)
        o, l = oracle.attn_fwd_rows(to_np(q[b, h]), to_np(k[b, g]), to_np(v[b, g]), rows, r, W, sinks=sinks, units=units)
        assert max_abs(to_np(out[b, h])[rows], o) <= TOL_OUT_BF16, case
        assert max_abs(to_np(lse[b, h])[rows], l) <= TOL_LSE_BF16, case
    # decode the last position on the cache evicted down to its visible set
    t = L - 1
    cache.update(None, None, _window_start(t, r, W, sinks, units))
    assert cache.rows == len(oracle.compressed_cache_positions(t, r, W, sinks=sinks, units=units))
    sl = torch.full((B,), cache.rows, dtype=torch.int32, device="cuda")
    o2, l2 = u.decode(qd[:, :, t].contiguous(), cache.kc, cache.vc, sl)
    for b, h in [(0, 0), (B - 1, Hq - 1)]:
        g = h // (Hq // Hkv)
        o, l = oracle.attn_fwd_rows(to_np(q[b, h]), to_np(k[b, g]), to_np(v[b, g]), [t], r, W, sinks=sinks, units=units)
        assert max_abs(to_np(o2[b, h]), o[0]) <= TOL_OUT_BF16 and abs(float(l2[b, h]) - l[0]) <= TOL_LSE_BF16


def test_prefill_rejects_a_cache_that_dropped_too_much():
    B, Hq, Hkv, D, r, W, C, p0 = 1, 2, 1, 128, 4, 100, 64, 500
    cap = 1024
    z = torch.zeros(B, Hkv, cap, D, dtype=torch.bfloat16, device="cuda")
    q = torch.zeros(B, Hq, C, D, dtype=torch.bfloat16, device="cuda")
    out, lse = torch.empty_like(q), torch.empty(B, Hq, C, device="cuda")
    args = lambda s: (q.data_ptr(), z.data_ptr(), z.data_ptr(), out.data_ptr(), lse.data_ptr(), B, Hq, Hkv, C, D, r, W, p0, s, cap, 0)
    assert u.unigist_prefill_chunk(*args(p0 - W + 1)) == 0
    assert u.unigist_prefill_chunk(*args(p0 - W + 2)) == 1      # first query would miss a raw token
    torch.cuda.synchronize()


def test_ragged_batch_of_caches_then_decode():
    # sequences of one batch at different lengths and window starts: each slab is an exact gather of its own
    # positions, and one decode call over the batch equals the oracle sequence by sequence
    B, Hq, Hkv, D, r, W = 4, 8, 2, 128, 4, 48
    lens = [700, 33, 412, 1]
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, max(lens), D, seed=25)
    kd, vd = k.cuda(), v.cuda()
    cache = u.RaggedKVCache(B, Hkv, max(lens), D, r)
    rng = np.random.default_rng(9)
    for b, n_b in enumerate(lens):
        while cache.t[b] < n_b - 1:
            n = int(min(n_b - 1 - cache.t[b], rng.choice([1, 2, 50, 300])))
            lo, hi = cache.t[b] + 1, cache.t[b] + 1 + n
            cache.update(b, kd[b, :, lo:hi].contiguous(), vd[b, :, lo:hi].contiguous(), max(0, hi - 1 - W + 1))
    kc, vc, sl = cache.gathered()
    qt = torch.stack([q[b, :, n_b - 1] for b, n_b in enumerate(lens)]).contiguous()      # each sequence's last position
    out, lse = u.decode(qt.cuda(), kc, vc, sl)
    torch.cuda.synchronize()
    for b, n_b in enumerate(lens):
        pos = oracle.compressed_cache_positions(n_b - 1, r, W)
        assert int(sl[b]) == len(pos)
        assert torch.equal(kc[b, :, :len(pos)].cpu(), k[b][:, pos]) and torch.equal(vc[b, :, :len(pos)].cpu(), v[b][:, pos])
        o, l = oracle.decode(to_np(qt[b:b + 1]), to_np(k[b:b + 1][:, :, pos]), to_np(v[b:b + 1][:, :, pos]))
        assert max_abs(to_np(out[b]), o[0]) <= TOL_OUT_BF16 and max_abs(to_np(lse[b]), l[0]) <= TOL_LSE_BF16


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.uint8], ids=["bf16", "e4m3"])
def test_batched_ragged_updates_then_decode(dtype):
    # one launch per step for the whole batch, states read from device memory: every sequence appends and evicts
    # at its own pace; a sequence given an impossible state is reported as -1 and left alone
    B, Hq, Hkv, D, r, W = 5, 8, 2, 128, 4, 40
    lens = [300, 33, 212, 1, 150]
    Lmax = max(lens)
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, Lmax, D, seed=26)
    ks, vs = synth.e4m3_scales(Hkv, seed=9)
    if dtype == torch.uint8:
        kq = torch.from_numpy(oracle.quantize_e4m3(k.to(torch.float32).numpy(), ks.numpy()))
        vq = torch.from_numpy(oracle.quantize_e4m3(v.to(torch.float32).numpy(), vs.numpy()))
    else:
        kq, vq = k, v
    kd, vd = kq.cuda(), vq.cuda()
    cache = u.RaggedKVCache(B, Hkv, Lmax, D, r, dtype=dtype)
    rng = np.random.default_rng(10)
    step = 0
    while any(cache.t[b] < lens[b] - 1 for b in range(B)):
        n_new = [int(min(lens[b] - 1 - cache.t[b], rng.choice([0, 1, 7, 64]))) for b in range(B)]
        nmax = max(max(n_new), 1)
        kn = torch.zeros(B, Hkv, nmax, D, dtype=kd.dtype, device="cuda")
        vn = torch.zeros_like(kn)
        for b in range(B):
            lo = cache.t[b] + 1
            kn[b, :, :n_new[b]] = kd[b, :, lo:lo + n_new[b]]
            vn[b, :, :n_new[b]] = vd[b, :, lo:lo + n_new[b]]
        s_new = [max(cache.s[b], cache.t[b] + n_new[b] - W + 1, 0) for b in range(B)]
        rows = cache.update_batch(kn, vn, n_new, s_new).cpu().tolist()
        kc, vc = cache.current()
        for b in range(B):
            pos = oracle.cache_positions(cache.s[b], cache.t[b], r)
            assert rows[b] == len(pos), (step, b)
            assert torch.equal(kc[b, :, :len(pos)].cpu(), kq[b][:, pos]) and torch.equal(vc[b, :, :len(pos)].cpu(), vq[b][:, pos])
        step += 1
    assert step > 3
    kc, vc = cache.current()
    sl = torch.tensor([cache.rows(b) for b in range(B)], dtype=torch.int32, device="cuda")
    qt = torch.stack([q[b, :, n_b - 1] for b, n_b in enumerate(lens)]).contiguous()
    if dtype == torch.uint8:
        out, lse = u.decode_e4m3(qt.cuda(), kc, vc, ks.cuda(), vs.cuda(), sl)
    else:
        out, lse = u.decode(qt.cuda(), kc, vc, sl)
    for b, n_b in enumerate(lens):
        pos = oracle.compressed_cache_positions(n_b - 1, r, W)
        assert int(sl[b]) == len(pos)
        if dtype == torch.uint8:
            o, l = oracle.decode_e4m3(to_np(qt[b:b + 1]), kq[b:b + 1][:, :, pos].numpy(), vq[b:b + 1][:, :, pos].numpy(), ks.numpy(), vs.numpy())
        else:
            o, l = oracle.decode(to_np(qt[b:b + 1]), to_np(k[b:b + 1][:, :, pos]), to_np(v[b:b + 1][:, :, pos]))
        assert max_abs(to_np(out[b]), o[0]) <= TOL_OUT_BF16 and max_abs(to_np(lse[b]), l[0]) <= TOL_LSE_BF16
    # an impossible request (window start behind the old one for sequence 1, too many rows for sequence 2)
    before_k = cache.current()[0].clone()
    s_bad = list(cache.s)
    s_bad[1] = cache.s[1] - 1 if cache.s[1] > 0 else cache.t[1] + 5
    n_bad = [0] * B
    n_bad[2] = 3                      # more than the new_rows of the call below
    kn = torch.zeros(B, Hkv, 1, D, dtype=kd.dtype, device="cuda")
    saved = (list(cache.s), list(cache.t), list(cache.cur))
    rows = cache.update_batch(kn, kn, n_bad, s_bad).cpu().tolist()
    assert rows[1] == -1 and rows[2] == -1 and all(rows[b] >= 0 for b in (0, 3, 4))
    kc2 = cache.current()[0]
    for b in (0, 3, 4):
        n = rows[b]
        assert torch.equal(kc2[b, :, :n], before_k[b, :, :n])


@pytest.mark.parametrize("sinks,units,W", [(0, False, 40), (9, True, 6)], ids=["sliding", "sinks_units"])
def test_batched_ragged_prefill_equals_one_pass(sinks, units, W):
    # One launch per step for the whole batch: every sequence is prefilled in chunks of its own sizes (none at
    # all in some steps), the states are read from device memory.  Every row each sequence ever gets must equal
    # that row of the one-pass attention over the sequence; rows past a sequence's chunk are left alone.
    B, Hq, Hkv, D, r, C = 5, 8, 2, 128, 4, 200
    lens = [700, 33, 412, 1, 150]
    Lmax = max(lens)
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, Lmax, D, seed=27)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    cache = u.RaggedKVCache(B, Hkv, Lmax, D, r, sinks=sinks)
    rng = np.random.default_rng(11)
    got_o = [torch.zeros(Hq, n, D, dtype=torch.bfloat16) for n in lens]
    got_l = [torch.zeros(Hq, n) for n in lens]
    step = 0
    while any(cache.t[b] < lens[b] - 1 for b in range(B)):
        n_new = [int(min(lens[b] - 1 - cache.t[b], rng.choice([0, 1, 37, 130, C]))) for b in range(B)]
        kn = torch.zeros(B, Hkv, C, D, dtype=kd.dtype, device="cuda")
        vn = torch.zeros_like(kn)
        qn = torch.zeros(B, Hq, C, D, dtype=qd.dtype, device="cuda")
        for b in range(B):
            lo = cache.t[b] + 1
            kn[b, :, :n_new[b]] = kd[b, :, lo:lo + n_new[b]]
            vn[b, :, :n_new[b]] = vd[b, :, lo:lo + n_new[b]]
            qn[b, :, :n_new[b]] = qd[b, :, lo:lo + n_new[b]]
        # window start: what the chunk's first query needs (an empty chunk keeps the old one)
        s_new = [max(cache.s[b], _window_start(cache.t[b] + 1, r, W, sinks, units)) if n_new[b] else cache.s[b]
                 for b in range(B)]
        p0 = [cache.t[b] + 1 for b in range(B)]
        rows_u = cache.update_batch(kn, vn, n_new, s_new).cpu().tolist()
        out = torch.full((B, Hq, C, D), 7.0, dtype=torch.bfloat16, device="cuda")
        lse = torch.full((B, Hq, C), 7.0, device="cuda")
        _, _, rows = cache.prefill_batch(qn, n_new, W, window_mode=int(units), out=out, lse=lse)
        torch.cuda.synchronize()
        assert rows.cpu().tolist() == rows_u, step
        out, lse = out.cpu(), lse.cpu()
        for b in range(B):
            got_o[b][:, p0[b]:p0[b] + n_new[b]] = out[b, :, :n_new[b]]
            got_l[b][:, p0[b]:p0[b] + n_new[b]] = lse[b, :, :n_new[b]]
            assert bool((out[b, :, n_new[b]:] == 7.0).all()) and bool((lse[b, :, n_new[b]:] == 7.0).all()), (step, b)
        step += 1
    assert step > 3
    for b, n_b in enumerate(lens):
        rows = np.unique(np.concatenate([[0, n_b - 1, min(n_b - 1, sinks)], np.random.default_rng(b).integers(0, n_b, 12)]))
        for h in (0, Hq - 1):
            g = h // (Hq // Hkv)
            o, l = oracle.attn_fwd_rows(to_np(q[b, h, :n_b]), to_np(k[b, g, :n_b]), to_np(v[b, g, :n_b]), rows, r, W,
                                        sinks=sinks, units=units)
            assert max_abs(to_np(got_o[b][h])[rows], o) <= TOL_OUT_BF16, (b, h)
            assert max_abs(to_np(got_l[b][h])[rows], l) <= TOL_LSE_BF16, (b, h)


def test_ragged_prefill_with_equal_states_is_the_plain_call_and_bad_states_are_reported():
    B, Hq, Hkv, D, r, W, C, L = 3, 4, 2, 64, 4, 50, 300, 900
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, L, D, seed=28)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    plain = u.KVCache(B, Hkv, L, D, r)
    ragged = u.RaggedKVCache(B, Hkv, L, D, r)
    for p0 in range(0, L, C):
        kn, vn, qn = (t[:, :, p0:p0 + C].contiguous() for t in (kd, vd, qd))
        s = max(0, p0 - W + 1)
        plain.update(kn, vn, s)
        a_o, a_l = u.prefill_chunk(qn, plain, r, W, p0)
        ragged.update_batch(kn, vn, [C] * B, [s] * B)
        b_o, b_l, rows = ragged.prefill_batch(qn, [C] * B, W)
        assert torch.equal(a_o, b_o) and torch.equal(a_l, b_l)
        assert rows.cpu().tolist() == [plain.rows] * B
    # impossible states: a window start right of what the first query sees, more rows than the queries' slab, a
    # negative position; the good sequence in between is still served, the others' outputs stay as they were
    kc, vc = ragged.current()
    qn = qd[:, :, L - C:].contiguous()
    dev = lambda x: torch.tensor(x, dtype=torch.int32, device="cuda")
    out = torch.full((B, Hq, C, D), 7.0, dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, C), 7.0, device="cuda")
    rows = torch.zeros(B, dtype=torch.int32, device="cuda")
    s_ok = L - C - W + 1
    p0, n, s0 = dev([L - C, L - C, -5]), dev([C, C, C]), dev([s_ok + 1, s_ok, s_ok])  # kept alive across the call
    st = u.unigist_prefill_chunk_ragged(qn.data_ptr(), kc.data_ptr(), vc.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                        B, Hq, Hkv, C, D, r, W, 0, 0, p0.data_ptr(), n.data_ptr(), s0.data_ptr(), L,
                                        rows.data_ptr(), 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert st == 0
    assert rows.cpu().tolist() == [-1, u.unigist_cache_rows(s_ok, L - 1, r), -1]
    assert torch.equal(out[1], b_o[1]) and torch.equal(lse[1], b_l[1])
    assert bool((out[0] == 7.0).all()) and bool((out[2] == 7.0).all()) and bool((lse[0] == 7.0).all())
    # n > C and a cache too small for the state
    p0, n, s0 = dev([L - C, 0, L - C]), dev([C + 1, 0, C]), dev([s_ok, 0, s_ok])
    st = u.unigist_prefill_chunk_ragged(qn.data_ptr(), kc.data_ptr(), vc.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                        B, Hq, Hkv, C, D, r, W, 0, 0, p0.data_ptr(), n.data_ptr(), s0.data_ptr(), 100,
                                        rows.data_ptr(), 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert st == 0 and rows.cpu().tolist() == [-1, 0, -1]


def test_prefill_on_row_slices_equals_prefill_on_copies():
    # chunks passed as slices along the row axis of the full tensors (no copies): same bits as with contiguous
    # chunks, and nothing outside the chunk's rows is written
    B, Hq, Hkv, D, r, W, C, L = 2, 4, 2, 128, 4, 60, 300, 1000
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, L, D, seed=29)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    a, b = u.KVCache(B, Hkv, L, D, r), u.KVCache(B, Hkv, L, D, r)
    out = torch.full((B, Hq, L, D), 7.0, dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, L), 7.0, device="cuda")
    for p0 in range(0, L, C):
        n = min(C, L - p0)
        s = max(0, p0 - W + 1)
        a.update(kd[:, :, p0:p0 + n].contiguous(), vd[:, :, p0:p0 + n].contiguous(), s)
        b.update(kd[:, :, p0:p0 + n], vd[:, :, p0:p0 + n], s)
        assert torch.equal(a.kc[:, :, :a.rows], b.kc[:, :, :b.rows]) and torch.equal(a.vc[:, :, :a.rows], b.vc[:, :, :b.rows])
        o, l = u.prefill_chunk(qd[:, :, p0:p0 + n].contiguous(), a, r, W, p0)
        u.prefill_chunk(qd[:, :, p0:p0 + n], b, r, W, p0, out=out[:, :, p0:p0 + n], lse=lse[:, :, p0:p0 + n])
        assert torch.equal(out[:, :, p0:p0 + n], o) and torch.equal(lse[:, :, p0:p0 + n], l)
        assert bool((out[:, :, p0 + n:] == 7.0).all()) and bool((lse[:, :, p0 + n:] == 7.0).all())
    with pytest.raises(u.UnigistError):
        u.prefill_chunk(qd[:, :, 0:C], b, r, W, 0, out=out[:, :, 0:C].contiguous(), lse=lse[:, :, 0:C])


def _sorted_rows(kr, vr):
    """rows of K and V side by side ([n, D] each), as raw 16-bit words, sorted: the cache's content as a multiset"""
    x = np.concatenate([kr.contiguous().view(torch.int16).numpy(), vr.contiguous().view(torch.int16).numpy()], axis=1)
    return x[np.lexsort(x.T[::-1])]


@pytest.mark.parametrize("sinks,units,W,r", [(0, False, 48, 4), (7, False, 48, 4), (9, True, 6, 4), (0, True, 2, 2),
                                             (40, True, 1, 7)])
def test_ring_cache_token_by_token_then_back(sinks, units, W, r):
    # Decoding loop on the ring layout: after every appended token each sequence's slab holds exactly the positions
    # the oracle says the next query sees (as a multiset of (K row, V row) pairs -- decode ignores the order), the
    # reported rows are their number, and decode on the slab matches the oracle.  Sequences pause at random.  At the
    # end the ring is turned back into the ordered layout and must be the exact gather of those positions.
    B, Hq, Hkv, D = 4, 8, 2, 128
    mask = dict(sinks=sinks, units=units)
    prompt = [130, 3, 60, 47]
    steps = 140
    Lmax = max(prompt) + steps
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, Lmax, D, seed=30)
    kd, vd = k.cuda(), v.cuda()
    rag = u.RaggedKVCache(B, Hkv, Lmax, D, r, sinks=sinks)
    for b, n in enumerate(prompt):
        rag.update(b, kd[b, :, :n].contiguous(), vd[b, :, :n].contiguous(), _window_start(n - 1, r, W, sinks, units))
    rag.gathered()
    ring = u.RingKVCache(rag, W, window_mode=int(units))
    torch.cuda.synchronize()
    t = [n - 1 for n in prompt]

    def check_content(when):
        rows = ring.rows.cpu().tolist()
        kc, vc = ring.kc.cpu(), ring.vc.cpu()
        for b in range(B):
            pos = oracle.compressed_cache_positions(t[b], r, W, **mask)
            assert rows[b] == len(pos) == u.unigist_cache_ring_rows(t[b], r, W, sinks, int(units)), (when, b)
            for h in range(Hkv):
                assert np.array_equal(_sorted_rows(kc[b, h, :rows[b]], vc[b, h, :rows[b]]),
                                      _sorted_rows(k[b, h][pos], v[b, h][pos])), (when, b, h)

    check_content("converted")
    rng = np.random.default_rng(12)
    for step in range(steps):
        act = [int(rng.random() < 0.8) for _ in range(B)]
        kn = torch.stack([kd[b, :, t[b] + 1:t[b] + 2] for b in range(B)]).contiguous()
        vn = torch.stack([vd[b, :, t[b] + 1:t[b] + 2] for b in range(B)]).contiguous()
        ring.append(kn, vn, torch.tensor(act, dtype=torch.int32, device="cuda"))
        t = [t[b] + act[b] for b in range(B)]
        if step % 9 == 0 or step % 9 == 4 or step == steps - 1:
            check_content(step)
        if step % 35 == 0 or step == steps - 1:
            qt = torch.stack([q[b, :, t[b]] for b in range(B)]).contiguous()
            out, lse = u.decode(qt.cuda(), ring.kc, ring.vc, ring.rows)
            for b in range(B):
                pos = oracle.compressed_cache_positions(t[b], r, W, **mask)
                o, l = oracle.decode(to_np(qt[b:b + 1]), to_np(k[b:b + 1][:, :, pos]), to_np(v[b:b + 1][:, :, pos]))
                # over a handful of keys an output is nearly a raw V value, which can exceed 2: the common bound
                assert out_ok(to_np(out[b]), o[0])
                assert max_abs(to_np(lse[b]), l[0]) <= TOL_LSE_BF16
    assert ring.t.cpu().tolist() == t
    rows = ring.to_ragged(rag).cpu().tolist()
    kc, vc = rag.current()
    for b in range(B):
        pos = oracle.compressed_cache_positions(t[b], r, W, **mask)
        assert rows[b] == len(pos)
        assert torch.equal(kc[b, :, :len(pos)].cpu(), k[b][:, pos]) and torch.equal(vc[b, :, :len(pos)].cpu(), v[b][:, pos])


def test_ring_cache_reports_impossible_states():
    B, Hkv, D, r, W, cap = 3, 2, 64, 4, 16, 40
    kc = torch.zeros(B, Hkv, cap, D, dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    kn = torch.ones(B, Hkv, 1, D, dtype=torch.bfloat16, device="cuda")
    dev = lambda x: torch.tensor(x, dtype=torch.int32, device="cuda")
    rows = torch.zeros(B, dtype=torch.int32, device="cuda")
    # t_old = -2 is no state; 150 positions need 16 + 27 rows > cap; the middle sequence is fine and not active
    t_old, act = dev([-2, 20, 150]), dev([1, 0, 1])
    st = u.unigist_cache_ring_append(kc.data_ptr(), vc.data_ptr(), kn.data_ptr(), kn.data_ptr(), 1, t_old.data_ptr(),
                                     act.data_ptr(), cap, rows.data_ptr(), B, Hkv, D, r, W, 0, 0, 0,
                                     torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert st == 0 and rows.cpu().tolist() == [-1, u.unigist_cache_ring_rows(20, r, W, 0, 0), -1]
    assert not bool(kc.any()) and not bool(vc.any())
    # conversion: the window start must be exactly the first position of the last query's window
    out_k, out_v = torch.zeros_like(kc), torch.zeros_like(kc)
    s, t = dev([3, 5, 0]), dev([20, 20, -1])
    st = u.unigist_cache_to_ring(kc.data_ptr(), vc.data_ptr(), s.data_ptr(), t.data_ptr(), cap, out_k.data_ptr(),
                                 out_v.data_ptr(), cap, rows.data_ptr(), B, Hkv, D, r, W, 0, 0, 0,
                                 torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert st == 0 and rows.cpu().tolist() == [-1, 16 + 1, 0]


@pytest.mark.parametrize("sinks,units,W", [(0, False, 40), (9, True, 5)], ids=["sliding", "sinks_units"])
def test_serving_loop_prefill_then_token_by_token(sinks, units, W):
    # The whole inference path of Sec. 4.3 on a batch of sequences of different lengths: ragged chunk-wise prefill,
    # eviction down to each last token's visible set, the ring layout, then token-by-token decoding with the O(1)
    # append.  Every output row, prefilled or decoded, must equal that row of the one-pass attention over the
    # sequence so far (the oracle never sees a cache).
    B, Hq, Hkv, D, r, C = 3, 8, 2, 128, 4, 128
    prompt, steps = [300, 41, 190], 60
    Lmax = max(prompt) + steps
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, Lmax, D, seed=31)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    cache = u.RaggedKVCache(B, Hkv, Lmax, D, r, sinks=sinks)
    got = [torch.zeros(Hq, n + steps, D, dtype=torch.bfloat16) for n in prompt]
    while any(cache.t[b] < prompt[b] - 1 for b in range(B)):
        n_new = [min(C, prompt[b] - 1 - cache.t[b]) for b in range(B)]
        p0 = [cache.t[b] + 1 for b in range(B)]
        kn = torch.zeros(B, Hkv, C, D, dtype=kd.dtype, device="cuda")
        vn, qn = torch.zeros_like(kn), torch.zeros(B, Hq, C, D, dtype=qd.dtype, device="cuda")
        for b in range(B):
            kn[b, :, :n_new[b]] = kd[b, :, p0[b]:p0[b] + n_new[b]]
            vn[b, :, :n_new[b]] = vd[b, :, p0[b]:p0[b] + n_new[b]]
            qn[b, :, :n_new[b]] = qd[b, :, p0[b]:p0[b] + n_new[b]]
        s_new = [max(cache.s[b], _window_start(p0[b], r, W, sinks, units)) if n_new[b] else cache.s[b] for b in range(B)]
        cache.update_batch(kn, vn, n_new, s_new)
        out, _, rows = cache.prefill_batch(qn, n_new, W, window_mode=int(units))
        assert min(rows.cpu().tolist()) >= 0
        for b in range(B):
            got[b][:, p0[b]:p0[b] + n_new[b]] = out[b, :, :n_new[b]].cpu()
    # evict down to what the last prompt token sees, switch layouts
    empty = torch.zeros(B, Hkv, 1, D, dtype=kd.dtype, device="cuda")
    cache.update_batch(empty, empty, [0] * B, [_window_start(prompt[b] - 1, r, W, sinks, units) for b in range(B)])
    ring = u.RingKVCache(cache, W, window_mode=int(units))
    t = [n - 1 for n in prompt]
    for _ in range(steps):
        kn = torch.stack([kd[b, :, t[b] + 1:t[b] + 2] for b in range(B)]).contiguous()
        vn = torch.stack([vd[b, :, t[b] + 1:t[b] + 2] for b in range(B)]).contiguous()
        rows = ring.append(kn, vn)
        t = [x + 1 for x in t]
        qt = torch.stack([qd[b, :, t[b]] for b in range(B)]).contiguous()
        out, _ = u.decode(qt, ring.kc, ring.vc, rows)
        for b in range(B):
            got[b][:, t[b]] = out[b].cpu()
    torch.cuda.synchronize()
    for b in range(B):
        n = prompt[b] + steps
        rows = np.unique(np.concatenate([[0, prompt[b] - 1, prompt[b], n - 1], np.random.default_rng(b).integers(0, n, 16)]))
        for h in (0, Hq - 1):
            g = h // (Hq // Hkv)
            o, _ = oracle.attn_fwd_rows(to_np(q[b, h, :n]), to_np(k[b, g, :n]), to_np(v[b, g, :n]), rows, r, W,
                                        sinks=sinks, units=units)
            assert out_ok(to_np(got[b][h])[rows], o), (b, h)


def test_ring_cache_moves_one_byte_rows_bit_exactly():
    # the ring calls are copies of rows of any element size: a cache of E4M3 codes (random bytes here) through
    # conversion, 90 appended tokens and the conversion back
    B, Hkv, D, r, W, sinks = 2, 2, 64, 4, 24, 3
    prompt, steps = [70, 5], 90
    Lmax = max(prompt) + steps
    g = torch.Generator().manual_seed(5)
    k = torch.randint(0, 256, (B, Hkv, Lmax, D), dtype=torch.uint8, generator=g)
    v = torch.randint(0, 256, (B, Hkv, Lmax, D), dtype=torch.uint8, generator=g)
    kd, vd = k.cuda(), v.cuda()
    rag = u.RaggedKVCache(B, Hkv, Lmax, D, r, dtype=torch.uint8, sinks=sinks)
    for b, n in enumerate(prompt):
        rag.update(b, kd[b, :, :n].contiguous(), vd[b, :, :n].contiguous(), max(0, n - 1 - W + 1))
    rag.gathered()
    ring = u.RingKVCache(rag, W)
    t = [n - 1 for n in prompt]
    for step in range(steps):
        kn = torch.stack([kd[b, :, t[b] + 1:t[b] + 2] for b in range(B)]).contiguous()
        vn = torch.stack([vd[b, :, t[b] + 1:t[b] + 2] for b in range(B)]).contiguous()
        ring.append(kn, vn)
        t = [x + 1 for x in t]
        if step % 7 == 0 or step == steps - 1:
            rows = ring.rows.cpu().tolist()
            kc, vc = ring.kc.cpu(), ring.vc.cpu()
            for b in range(B):
                pos = oracle.compressed_cache_positions(t[b], r, W, sinks=sinks)
                assert rows[b] == len(pos)
                for h in range(Hkv):
                    assert np.array_equal(_sorted_rows(kc[b, h, :rows[b]], vc[b, h, :rows[b]]),
                                          _sorted_rows(k[b, h][pos], v[b, h][pos])), (step, b, h)
    ring.to_ragged(rag)
    kc, vc = rag.current()
    for b in range(B):
        pos = oracle.compressed_cache_positions(t[b], r, W, sinks=sinks)
        assert torch.equal(kc[b, :, :len(pos)].cpu(), k[b][:, pos]) and torch.equal(vc[b, :, :len(pos)].cpu(), v[b][:, pos])


@pytest.mark.parametrize("D", [128, 96])
def test_prefill_on_projection_layout_equals_prefill_on_copies(D):
    # q as a projection layer leaves it, [B, C, Hq, D], passed as its transposed view: out comes back in the same
    # layout, same bits as with a contiguous [B, Hq, C, D] copy; a row slice without out= / lse= takes the same path
    B, Hq, Hkv, r, W, C, L = 2, 4, 2, 4, 60, 300, 900
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, L, D, seed=32)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    cache = u.KVCache(B, Hkv, L, D, r)
    for p0 in range(0, L, C):
        cache.update(kd[:, :, p0:p0 + C], vd[:, :, p0:p0 + C], max(0, p0 - W + 1))
        want_o, want_l = u.prefill_chunk(qd[:, :, p0:p0 + C].contiguous(), cache, r, W, p0)
        q_blhd = qd[:, :, p0:p0 + C].transpose(1, 2).contiguous()          # [B, C, Hq, D] in memory
        o, l = u.prefill_chunk(q_blhd.transpose(1, 2), cache, r, W, p0)
        assert o.stride() == q_blhd.transpose(1, 2).stride() and torch.equal(o, want_o) and torch.equal(l, want_l)
        o2, l2 = u.prefill_chunk(qd[:, :, p0:p0 + C], cache, r, W, p0)     # a row slice of the [B, Hq, L, D] tensor
        assert torch.equal(o2, want_o) and torch.equal(l2, want_l)
