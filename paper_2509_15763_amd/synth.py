"""Seeded synthetic inputs and the workload table.

Holds no attention arithmetic: only shapes and random draws.  Both the HIP
path's tests/bench and the CPU oracle's tests read their inputs from here.

The workloads stand in for the attention layer of a Llama-3-8B-shaped model
trained on 32K-token gist-interleaved sequences (Sec. 5.1 and App. C of the
paper: 32 heads, head dim 128, lengths 16K-128K).  Attention cost does not
depend on the data, so q, k, v and dout are i.i.d. N(0, 1).
"""
from __future__ import annotations

import torch

# name -> dict(B, Hq, Hkv, L, D, r, W); "decode" entries carry Lk instead of L/r/W.
WORKLOADS = {
    "cfg1_tiny": dict(B=1, Hq=1, Hkv=1, L=1024, D=64, r=4, W=128),
    "cfg2_llama8b_32k": dict(B=1, Hq=32, Hkv=8, L=32768, D=128, r=4, W=1024),
    "cfg3_long_128k": dict(B=1, Hq=32, Hkv=8, L=131072, D=128, r=8, W=2048),
    "cfg4_ratio_sweep": dict(B=4, Hq=32, Hkv=8, L=16384, D=128, r=(2, 4, 8, 16, 32), W=1024),
    "cfg5_decode": dict(B=64, Hq=32, Hkv=8, Lk=17408, D=128, gists=16384, window=1024),
}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def attn_inputs(B, Hq, Hkv, L, D, dtype=torch.bfloat16, seed=0, device="cpu"):
    """q, dout [B,Hq,L,D] and k, v [B,Hkv,L,D], drawn in fp32 in the order
    q, k, v, dout from one generator, then rounded to `dtype`."""
    g = _gen(seed, device)
    q = torch.randn(B, Hq, L, D, generator=g, device=device, dtype=torch.float32).to(dtype)
    k = torch.randn(B, Hkv, L, D, generator=g, device=device, dtype=torch.float32).to(dtype)
    v = torch.randn(B, Hkv, L, D, generator=g, device=device, dtype=torch.float32).to(dtype)
    dout = torch.randn(B, Hq, L, D, generator=g, device=device, dtype=torch.float32).to(dtype)
    return q, k, v, dout


def decode_inputs(B, Hq, Hkv, Lk, D, dtype=torch.bfloat16, seed=0, device="cpu"):
    """q [B,Hq,D] and kcache, vcache [B,Hkv,Lk,D], order q, k, v.  The caches are
    drawn one batch entry at a time so that the fp32 staging stays small."""
    g = _gen(seed, device)
    q = torch.randn(B, Hq, D, generator=g, device=device, dtype=torch.float32).to(dtype)
    kc = torch.empty(B, Hkv, Lk, D, device=device, dtype=dtype)
    vc = torch.empty(B, Hkv, Lk, D, device=device, dtype=dtype)
    for b in range(B):
        kc[b] = torch.randn(Hkv, Lk, D, generator=g, device=device, dtype=torch.float32).to(dtype)
    for b in range(B):
        vc[b] = torch.randn(Hkv, Lk, D, generator=g, device=device, dtype=torch.float32).to(dtype)
    return q, kc, vc


def ragged_seqlens(B, Lk, seed=0):
    """Per-sequence cache lengths in [1, Lk], with the extremes present."""
    g = _gen(seed, "cpu")
    s = torch.randint(1, Lk + 1, (B,), generator=g, dtype=torch.int32)
    if B >= 2:
        s[0] = Lk
        s[1] = 1
    return s


def e4m3_scales(H, seed=0, device="cpu"):
    """One positive scale per kv head for K and one for V (float32 [H] each): about amax / 448 of unit-variance
    data, different per head and not powers of two, so that the division has to round."""
    g = _gen(seed, "cpu")
    ks = (0.0093 + 0.004 * torch.rand(H, generator=g)).to(torch.float32)
    vs = (0.0107 + 0.004 * torch.rand(H, generator=g)).to(torch.float32)
    return ks.to(device), vs.to(device)
