"""GPU parity: unigist_decode (through the C ABI) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_15763_amd as u
from paper_2509_15763_amd import synth
from _parity import TOL_F32, TOL_LSE_BF16, TOL_OUT_BF16, max_abs, out_ok, to_np

pytestmark = pytest.mark.gpu

# B, Hq, Hkv, Lk, D, ragged
CASES = [
    (3, 8, 2, 1000, 128, False), (3, 8, 2, 1000, 128, True), (2, 4, 4, 257, 64, True), (1, 32, 8, 5000, 128, False),
    (2, 6, 2, 300, 128, True), (1, 1, 1, 1, 64, False), (5, 16, 2, 77, 64, True),
    (2, 8, 2, 300, 64, True), (1, 4, 1, 2100, 64, False), (64, 4, 1, 40, 128, True),
    (2, 4, 2, 500, 128, True), (1, 8, 1, 700, 128, False), (3, 16, 2, 129, 64, True), (1, 32, 1, 300, 128, False),
    (2, 16, 1, 200, 64, True), (2, 15, 1, 333, 128, True), (1, 12, 4, 1000, 128, False),
    # other head dimensions: the matrix-core kernel (groups up to 15 heads) and the vector kernel (fp32; larger groups)
    (2, 8, 2, 700, 96, True), (1, 4, 1, 300, 80, False), (3, 4, 4, 129, 32, True), (1, 32, 1, 300, 96, False),
    (2, 16, 1, 200, 48, True), (1, 8, 2, 2100, 112, False),
]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("B,Hq,Hkv,Lk,D,ragged", CASES)
def test_decode_matches_oracle(B, Hq, Hkv, Lk, D, ragged, dtype):
    print("case", B, Hq, Hkv, Lk, D, ragged, dtype, flush=True)
    q, kc, vc = synth.decode_inputs(B, Hq, Hkv, Lk, D, dtype=dtype, seed=1)
    sl = synth.ragged_seqlens(B, Lk, seed=2) if ragged else None
    out, lse = u.decode(q.cuda(), kc.cuda(), vc.cuda(), None if sl is None else sl.cuda())
    torch.cuda.synchronize()
    o, l = oracle.decode(to_np(q), to_np(kc), to_np(vc), None if sl is None else sl.numpy())
    eo, el = max_abs(to_np(out), o), max_abs(to_np(lse), l)
    print(f"  out {eo:.3e} lse {el:.3e}", flush=True)
    if dtype == torch.float32:
        assert eo <= TOL_F32 and el <= TOL_F32
    else:
        # sequences of a few keys give outputs of size 2 and more: the common bound (1e-2 below 2, the stored
        # result's half-ulp on top from there)
        assert out_ok(to_np(out), o) and el <= TOL_LSE_BF16


def test_decode_equals_last_row_of_the_training_kernel():
    # the cache a generation loop would hold at position t, fed to decode, must give row t of the forward
    L, D, r, W = 2000, 128, 8, 100
    q, k, v, _ = synth.attn_inputs(1, 4, 1, L, D, seed=7)
    out, lse = u.attn_fwd(q.cuda(), k.cuda(), v.cuda(), r, W)
    t = L - 1
    pos = torch.from_numpy(oracle.compressed_cache_positions(t, r, W))
    kc, vc = k[:, :, pos].contiguous(), v[:, :, pos].contiguous()
    o2, l2 = u.decode(q[:, :, t].contiguous().cuda(), kc.cuda(), vc.cuda())
    assert max_abs(to_np(o2), to_np(out[:, :, t])) <= 1e-2
    assert max_abs(to_np(l2), to_np(lse[:, :, t])) <= 1e-3


def test_a_sequence_of_zero_keys_gives_the_empty_sum():
    # outside the contract (seqlens are >= 1), but it must not poison the batch with NaN
    B, Hq, Hkv, Lk, D = 3, 8, 2, 300, 128
    q, kc, vc = synth.decode_inputs(B, Hq, Hkv, Lk, D, seed=5)
    sl = torch.tensor([300, 0, 17], dtype=torch.int32)
    out, lse = u.decode(q.cuda(), kc.cuda(), vc.cuda(), sl.cuda())
    torch.cuda.synchronize()
    assert torch.equal(out[1].cpu(), torch.zeros_like(out[1].cpu())) and torch.isinf(lse[1]).all() and (lse[1] < 0).all()
    keep = [0, 2]
    o, l = oracle.decode(to_np(q[keep]), to_np(kc[keep]), to_np(vc[keep]), sl[keep].numpy())
    assert max_abs(to_np(out[keep]), o) <= 2e-2 and max_abs(to_np(lse[keep]), l) <= TOL_LSE_BF16


@pytest.mark.parametrize("codes", [False, True], ids=["bf16", "e4m3"])
def test_decode_over_a_million_keys(codes):
    # one sequence whose cache holds 2^20 rows (64 slices of 16 384 keys per kv head), bf16 and E4M3 storage
    B, Hq, Hkv, Lk, D = 1, 4, 2, 1 << 20, 128
    q, kc, vc = synth.decode_inputs(B, Hq, Hkv, Lk, D, seed=9, device="cuda")
    if codes:
        ks, vs = synth.e4m3_scales(Hkv, seed=9, device="cuda")
        k8, v8 = u.quantize_e4m3(kc, ks), u.quantize_e4m3(vc, vs)
        out, lse = u.decode_e4m3(q, k8, v8, ks, vs)
        torch.cuda.synchronize()
        o, l = oracle.decode_e4m3(to_np(q.cpu()), k8.cpu().numpy(), v8.cpu().numpy(), ks.cpu().numpy(), vs.cpu().numpy())
    else:
        out, lse = u.decode(q, kc, vc)
        torch.cuda.synchronize()
        o, l = oracle.decode(to_np(q.cpu()), to_np(kc.cpu()), to_np(vc.cpu()))
    assert max_abs(to_np(out.cpu()), o) <= TOL_OUT_BF16 and max_abs(to_np(lse.cpu()), l) <= TOL_LSE_BF16
