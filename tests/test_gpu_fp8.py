"""GPU parity of the 8-bit (E4M3) storage of the compressed cache against the oracle: the quantiser bit for bit, the
decode over quantised caches within the decode tolerances (both sides read the same codes), the cache maintenance
on one-byte rows bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth
from _parity import TOL_LSE_BF16, TOL_OUT_BF16, max_abs, out_ok, to_np

pytestmark = pytest.mark.gpu


def special_values():
    """binary32 values around everything the rounding has to get right: every representable magnitude, every midpoint
    between neighbours, values a hair to either side, the subnormal range, the clamp."""
    grid = oracle.e4m3_decode(np.arange(0x00, 0x7F, dtype=np.uint8))
    mids = (grid[:-1] + grid[1:]) / 2
    eps = (grid[1:] - grid[:-1]) / 64
    extra = np.array([0.0, 2.0 ** -10, 2.0 ** -10 * (1 + 2.0 ** -20), 2.0 ** -11, 1e-30, 448.0, 449.0, 463.9, 464.0, 480.0, 1e5, 3e38])
    x = np.concatenate([grid, mids, mids - eps, mids + eps, extra])
    x = np.concatenate([x, -x]).astype(np.float32)
    pad = (-len(x)) % 128
    return np.concatenate([x, np.zeros(pad, np.float32)])


@pytest.mark.parametrize("D", [64, 128, 32])
def test_quantiser_is_bit_exact_on_the_special_values(D):
    x = special_values().reshape(1, 1, -1, D)
    for c in (1.0, 0.75, 1.1, 0.013):
        scale = np.float32([c])
        xs = (x.astype(np.float64) * float(scale[0])).astype(np.float32)        # so that x / c lands on or near the special values
        got = u.quantize_e4m3(torch.from_numpy(xs).cuda(), torch.from_numpy(scale).cuda()).cpu().numpy()
        want = oracle.quantize_e4m3(xs, scale)
        bad = np.flatnonzero(got.ravel() != want.ravel())
        assert bad.size == 0, (c, xs.ravel()[bad[:8]], got.ravel()[bad[:8]], want.ravel()[bad[:8]])


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32], ids=["bf16", "f32"])
@pytest.mark.parametrize("B,H,n,D", [(2, 3, 517, 128), (1, 8, 64, 64), (3, 1, 1, 128), (1, 2, 0, 64), (2, 2, 77, 96),
                                     (1, 3, 130, 48)])
def test_quantiser_is_bit_exact_on_cache_rows(B, H, n, D, dtype):
    _, k, v, _ = synth.attn_inputs(B, H, H, max(n, 1), D, dtype=dtype, seed=51)
    k = (k[:, :, :n] * 1.7).to(dtype).contiguous()      # wider than the scales assume: some values saturate
    ks, _ = synth.e4m3_scales(H, seed=5)
    got = u.quantize_e4m3(k.cuda(), ks.cuda()).cpu().numpy()
    want = oracle.quantize_e4m3(k.to(torch.float32).numpy(), ks.numpy())
    assert got.shape == want.shape and np.array_equal(got, want)
    if n:
        assert (want & 0x7F).max() == 0x7E or n < 64     # the clamp was exercised


CASES = [
    (3, 8, 2, 1000, 128, False), (3, 8, 2, 1000, 128, True), (2, 4, 4, 257, 64, True), (1, 32, 8, 5000, 128, False),
    (2, 6, 2, 300, 128, True), (1, 1, 1, 1, 64, False), (5, 16, 2, 77, 64, True),
    (2, 8, 2, 300, 64, True), (1, 4, 1, 2100, 64, False), (64, 4, 1, 40, 128, True),
    (2, 4, 2, 500, 128, True), (1, 8, 1, 700, 128, False), (3, 16, 2, 129, 64, True), (1, 32, 1, 300, 128, False),
    (2, 16, 1, 200, 64, True), (2, 15, 1, 333, 128, True), (1, 12, 4, 1000, 128, False),
    # other head dimensions (multiples of 16 for one-byte codes): matrix-core kernel and, for a group of 16, the vector kernel
    (2, 8, 2, 700, 96, True), (1, 4, 1, 300, 80, False), (3, 4, 4, 129, 32, True), (1, 16, 1, 300, 112, False),
]


@pytest.mark.parametrize("B,Hq,Hkv,Lk,D,ragged", CASES)
def test_decode_over_codes_matches_oracle(B, Hq, Hkv, Lk, D, ragged):
    print("case", B, Hq, Hkv, Lk, D, ragged, flush=True)
    q, kc, vc = synth.decode_inputs(B, Hq, Hkv, Lk, D, seed=52)
    ks, vs = synth.e4m3_scales(Hkv, seed=6)
    # the codes are inputs of both sides: quantised by the oracle
    kq = oracle.quantize_e4m3(kc.to(torch.float32).numpy(), ks.numpy())
    vq = oracle.quantize_e4m3(vc.to(torch.float32).numpy(), vs.numpy())
    sl = synth.ragged_seqlens(B, Lk, seed=2) if ragged else None
    out, lse = u.decode_e4m3(q.cuda(), torch.from_numpy(kq).cuda(), torch.from_numpy(vq).cuda(), ks.cuda(), vs.cuda(),
                             None if sl is None else sl.cuda())
    torch.cuda.synchronize()
    o, l = oracle.decode_e4m3(to_np(q), kq, vq, ks.numpy(), vs.numpy(), None if sl is None else sl.numpy())
    eo, el = max_abs(to_np(out), o), max_abs(to_np(lse), l)
    print(f"  out {eo:.3e} lse {el:.3e}", flush=True)
    # a sequence of a few keys returns values of v themselves (up to 448 * scale, about 4.8): the common bound
    assert out_ok(to_np(out), o) and el <= TOL_LSE_BF16


def test_quantised_cache_through_updates_then_decode():
    # append and evict on one-byte rows: the cache equals a gather of the oracle's codes, and decode on it matches
    B, Hq, Hkv, D, r, W, L = 2, 8, 2, 128, 4, 64, 700
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, L, D, seed=53)
    ks, vs = synth.e4m3_scales(Hkv, seed=7)
    kq = oracle.quantize_e4m3(k.to(torch.float32).numpy(), ks.numpy())
    vq = oracle.quantize_e4m3(v.to(torch.float32).numpy(), vs.numpy())
    cache = u.KVCache(B, Hkv, L, D, r, dtype=torch.uint8, k_scale=ks.cuda(), v_scale=vs.cuda())
    kd, vd = k.cuda(), v.cuda()
    rng = np.random.default_rng(8)
    while cache.t < L - 1:
        n = int(min(L - 1 - cache.t, rng.choice([1, 3, 64, 200])))
        lo, hi = cache.t + 1, cache.t + 1 + n
        cache.update(kd[:, :, lo:hi].contiguous(), vd[:, :, lo:hi].contiguous(), max(0, hi - 1 - W + 1))
        pos = oracle.cache_positions(cache.s, cache.t, r)
        assert cache.rows == len(pos)
        assert np.array_equal(cache.kc[:, :, :cache.rows].cpu().numpy(), kq[:, :, pos])
        assert np.array_equal(cache.vc[:, :, :cache.rows].cpu().numpy(), vq[:, :, pos])
    t = L - 1
    pos = oracle.compressed_cache_positions(t, r, W)
    assert np.array_equal(pos, oracle.cache_positions(cache.s, cache.t, r))
    sl = torch.full((B,), cache.rows, dtype=torch.int32, device="cuda")
    out, lse = u.decode_e4m3(q[:, :, t].contiguous().cuda(), cache.kc, cache.vc, cache.k_scale, cache.v_scale, sl)
    o, l = oracle.decode_e4m3(to_np(q[:, :, t]), kq[:, :, pos], vq[:, :, pos], ks.numpy(), vs.numpy())
    assert max_abs(to_np(out), o) <= TOL_OUT_BF16 and max_abs(to_np(lse), l) <= TOL_LSE_BF16
    # and the 8-bit cache is a faithful stand-in for the 16-bit one at these scales
    o16, _ = oracle.decode(to_np(q[:, :, t]), to_np(k[:, :, pos]), to_np(v[:, :, pos]))
    assert max_abs(o, o16) < 0.05


@pytest.mark.parametrize("Hq,Hkv,D,L,C,r,W,sinks,units", [
    (8, 2, 128, 1500, 400, 4, 64, 0, False),
    (4, 1, 64, 900, 256, 4, 5, 40, True),       # sinks and a window of whole units, D = 64, ragged last chunk
    (4, 2, 96, 1100, 300, 4, 64, 0, False),     # head dimension 96
])
def test_chunkwise_prefill_over_codes(Hq, Hkv, D, L, C, r, W, sinks, units):
    # the prompt goes through a cache of one-byte rows chunk by chunk: every chunk's rows equal attention over the
    # dequantised keys and values (the oracle's codes times the scales, in fp64), and the last row agrees with decode
    B = 2
    q, k, v, _ = synth.attn_inputs(B, Hq, Hkv, L, D, seed=54)
    ks, vs = synth.e4m3_scales(Hkv, seed=8)
    kq = oracle.quantize_e4m3(k.to(torch.float32).numpy(), ks.numpy())
    vq = oracle.quantize_e4m3(v.to(torch.float32).numpy(), vs.numpy())
    kdq, vdq = oracle.dequantize_e4m3(kq, ks.numpy()), oracle.dequantize_e4m3(vq, vs.numpy())
    cache = u.KVCache(B, Hkv, L, D, r, dtype=torch.uint8, k_scale=ks.cuda(), v_scale=vs.cuda(), sinks=sinks)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()

    def wstart(i):
        if not units:
            return max(0, i - W + 1)
        return i if i < sinks else sinks + max(0, (i - sinks) // (r + 1) - W) * (r + 1)

    outs, lses = [], []
    for p0 in range(0, L, C):
        n = min(C, L - p0)
        cache.update(kd[:, :, p0:p0 + n].contiguous(), vd[:, :, p0:p0 + n].contiguous(), wstart(p0))
        o, l = u.prefill_chunk(qd[:, :, p0:p0 + n].contiguous(), cache, r, W, p0, window_mode=int(units))
        outs.append(o)
        lses.append(l)
    out, lse = torch.cat(outs, dim=2), torch.cat(lses, dim=2)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, max(sinks - 1, 0), sinks, C - 1, C, L - 1], np.random.default_rng(3).integers(0, L, 20)]))
    for b, h in [(0, 0), (B - 1, Hq - 1)]:
        g = h // (Hq // Hkv)
        o, l = oracle.attn_fwd_rows(to_np(q[b, h]), kdq[b, g], vdq[b, g], rows, r, W, sinks=sinks, units=units)
        assert max_abs(to_np(out[b, h])[rows], o) <= TOL_OUT_BF16, (b, h)
        assert max_abs(to_np(lse[b, h])[rows], l) <= TOL_LSE_BF16, (b, h)
    t = L - 1
    cache.update(None, None, wstart(t))
    sl = torch.full((B,), cache.rows, dtype=torch.int32, device="cuda")
    o2, l2 = u.decode_e4m3(qd[:, :, t].contiguous(), cache.kc, cache.vc, cache.k_scale, cache.v_scale, sl)
    assert max_abs(to_np(o2), to_np(out[:, :, t])) <= 2 * TOL_OUT_BF16
    assert max_abs(to_np(l2), to_np(lse[:, :, t])) <= 2 * TOL_LSE_BF16


def test_full_size_decode_over_codes_sampled():
    # the serving shape, cache bytes halved: sampled (batch, head) pairs against the oracle on the same codes
    w = synth.WORKLOADS["cfg5_decode"]
    B, Hq, Hkv, Lk, D = w["B"], w["Hq"], w["Hkv"], w["Lk"], w["D"]
    q, kc, vc = synth.decode_inputs(B, Hq, Hkv, Lk, D, seed=0, device="cuda")
    ks, vs = synth.e4m3_scales(Hkv, seed=0, device="cuda")
    kq, vq = u.quantize_e4m3(kc, ks), u.quantize_e4m3(vc, vs)
    sl = synth.ragged_seqlens(B, Lk, seed=3).cuda()
    out, lse = u.decode_e4m3(q, kq, vq, ks, vs, sl)
    torch.cuda.synchronize()
    G = Hq // Hkv
    for b, h in [(0, 0), (17, 13), (B - 1, Hq - 1)]:
        g = h // G
        n = int(sl[b])
        # the GPU quantiser's codes for this head must be the oracle's; then both sides decode the same codes
        want_k = oracle.quantize_e4m3(kc[b, g].to(torch.float32).cpu().numpy()[None], ks[g:g + 1].cpu().numpy())[0]
        want_v = oracle.quantize_e4m3(vc[b, g].to(torch.float32).cpu().numpy()[None], vs[g:g + 1].cpu().numpy())[0]
        assert np.array_equal(kq[b, g].cpu().numpy(), want_k) and np.array_equal(vq[b, g].cpu().numpy(), want_v)
        o, l = oracle.decode_e4m3(to_np(q[b:b + 1, h:h + 1]), want_k[None, None, :n], want_v[None, None, :n],
                                  ks[g:g + 1].cpu().numpy(), vs[g:g + 1].cpu().numpy())
        assert max_abs(to_np(out[b, h]), o[0, 0]) <= TOL_OUT_BF16 and abs(float(lse[b, h]) - l[0, 0]) <= TOL_LSE_BF16
