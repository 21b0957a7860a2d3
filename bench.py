#!/usr/bin/env python3
"""Benchmark of libunigist on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one forward plus one backward of gist-masked attention on the 32K-token GQA
workload (B=1, Hq=32, Hkv=8, D=128, L=32768, r=4, W=1024, bf16, synthetic N(0,1) inputs
already resident in HBM).  The headline value is TFLOP/s counted over the visible
(query, key) pairs only: 4*D flops per pair forward, 10*D backward, recompute not counted.
The backward is issued one stage at a time with HIP events between the stages (all on
torch's current stream, which is the stream the kernels run on), so every kernel's
duration is measured live inside the timed region.  The decode op (a serving-path call on
a different workload: 64 sequences x 17 408 cached keys) is timed in its own region and
reported beside it with its HBM roofline.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import paper_2509_15763_amd as u  # noqa: E402
from paper_2509_15763_amd import synth  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, vendor figure
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, vendor figure
WORKLOAD = "cfg2_llama8b_32k"

# HBM bytes per launch measured offline with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by
# what the same counters read for a plain copy); see profiles/.  None = not measured yet.
TRAFFIC_BYTES = {"fwd": 1038100000, "dkdv_gist": 2257700000, "dkdv_window": 1473500000, "dq": 1408400000,
                 "decode": 4669700000, "decode_e4m3": 2285100000}


def pair_counts(L, r, W):
    """Visible pairs per head, split the way the dK/dV pass splits them: a 64-row query chunk
    c reaches the gists left of far(c) = floor(max(0, 64c - W + 1) / 128) * 128 in the gist
    phase and everything else in the window phase."""
    nvis = u.n_vis(L, r, W)
    rp1 = r + 1 if r < L else L + 1
    far_pairs = 0
    for c in range((L + 63) // 64):
        rows = min(L, 64 * c + 64) - 64 * c
        far = (max(0, 64 * c - min(W, L) + 1) // 128) * 128
        far_pairs += rows * (far // rp1)
    return nvis, far_pairs


def time_shape(B, Hq, Hkv, L, D, r, W, steps=3, warmup=1, seed=0):
    """Forward and backward (all stages in one call) of one more shape, each in its own event-timed region."""
    q, k, v, dout = synth.attn_inputs(B, Hq, Hkv, L, D, seed=seed, device="cuda")
    ws = torch.empty(u.unigist_attn_bwd_workspace(B, Hq, Hkv, L, D, r, W, u.UNIGIST_BF16), device="cuda", dtype=torch.uint8)
    grads = (torch.empty_like(q), torch.empty_like(k), torch.empty_like(v))
    out, lse = u.attn_fwd(q, k, v, r, W)
    res = {}
    for name, fn in (("fwd", lambda: u.attn_fwd(q, k, v, r, W)),
                     ("bwd", lambda: u.attn_bwd(q, k, v, out, lse, dout, r, W, workspace=ws, grads=grads))):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        res[name] = e0.elapsed_time(e1) / steps
    nvis = u.n_vis(L, r, W)
    bm, bn = u.unigist_tile_sizes(D, u.UNIGIST_BF16)
    m = u.unigist_blockmap_build(L, r, W, bm, bn)
    tf = lambda per_pair, ms: per_pair * D * nvis * B * Hq / ms / 1e9
    return {"fwd_ms": res["fwd"], "bwd_ms": res["bwd"],
            "fwd_pct_of_peak": 100.0 * tf(4.0, res["fwd"]) / PEAK_BF16_TFLOPS,
            "bwd_pct_of_peak": 100.0 * tf(10.0, res["bwd"]) / PEAK_BF16_TFLOPS,
            "tflops": tf(14.0, res["fwd"] + res["bwd"]),
            "live_tile_fraction": m["live_tiles"] / m["causal_tiles"],
            "visible_fraction": nvis / (L * (L + 1) / 2),
            "bwd_workspace_mb": ws.numel() / 1e6}


def cpu_baseline(cfg, budget_s=15.0):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload: blocks of 512
    query rows spread over the sequence, forward and backward, head after head, until about
    `budget_s` seconds of CPU work are done.  Its cost per row does not depend on the row (every
    key is scored), so the sample is representative."""
    import numpy as np
    import oracle
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    L, D, r, W, G = cfg["L"], cfg["D"], cfg["r"], cfg["W"], cfg["Hq"] // cfg["Hkv"]
    q, k, v, do = synth.attn_inputs(1, G, 1, L, D, seed=0)
    kn, vn = k[0, 0].double().numpy(), v[0, 0].double().numpy()
    starts = [int(x) for x in np.linspace(0, L - 512, 12)]
    pairs = nblocks = 0
    t0 = time.perf_counter()
    for h in range(G):
        qn, don = q[0, h].double().numpy(), do[0, h].double().numpy()
        for s0 in starts:
            rows = np.arange(s0, s0 + 512)
            oracle.attn_fwd_rows(qn, kn, vn, rows, r, W)
            oracle.attn_bwd_head(qn, kn, vn, don, r, W, block=512, row_lo=s0, row_hi=s0 + 512)
            pairs += int(np.sum(np.minimum(rows + 1, W) + np.maximum(0, (rows - W + 1) // (r + 1))))
            nblocks += 1
            if time.perf_counter() - t0 > budget_s:
                break
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    return {"value": 14.0 * D * pairs / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{nblocks} blocks of 512 query rows spread over the {L} positions of up to {G} query heads "
                      f"(one kv group), fwd+bwd, dense fp64 numpy, {dt:.1f} s of CPU work; flops counted on "
                      f"visible pairs only (4*D fwd + 10*D bwd per pair)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--no-prefill", action="store_true",
                    help="skip the chunk-wise prefill region and the packed-documents region (profiling runs: the first "
                         "launches the forward kernel under the same name at a smaller size)")
    ap.add_argument("--no-probe", action="store_true",
                    help="skip the matrix-core rate probe (profiling runs: its kernel would top the kernel statistics)")
    ap.add_argument("--no-other-shapes", action="store_true",
                    help="skip the 128K-token shape and the compression-ratio sweep (profiling runs)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy, so that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                         "can be scaled by what they read for a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU (no collectives, no sharding); run with --gpus 1")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; libunigist has no CPU path")

    cfg = dict(synth.WORKLOADS[WORKLOAD])
    B, Hq, Hkv, L, D, r, W = (cfg[n] for n in ("B", "Hq", "Hkv", "L", "D", "r", "W"))
    dev = "cuda"
    q, k, v, dout = synth.attn_inputs(B, Hq, Hkv, L, D, seed=0, device=dev)
    nvis, far_pairs = pair_counts(L, r, W)
    flops_fwd = 4.0 * D * nvis * B * Hq
    flops_bwd = 10.0 * D * nvis * B * Hq
    ws = torch.empty(u.unigist_attn_bwd_workspace(B, Hq, Hkv, L, D, r, W, u.UNIGIST_BF16), device=dev, dtype=torch.uint8)
    grads = (torch.empty_like(q), torch.empty_like(k), torch.empty_like(v))
    stage_names = ["delta", "dkdv_gist", "gist_reduce", "dkdv_window", "dq"]

    def step(events=None):
        if events is not None:
            events[0].record()
        out, lse = u.attn_fwd(q, k, v, r, W)
        if events is not None:
            events[1].record()
        for n, name in enumerate(stage_names):
            u.attn_bwd(q, k, v, out, lse, dout, r, W, workspace=ws, stages=u.BWD_STAGES[name], grads=grads)
            if events is not None:
                events[2 + n].record()

    if args.copy_calibration:
        src = torch.empty(1 << 30, device=dev, dtype=torch.uint8).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(7)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    names = ["fwd"] + stage_names
    ms = {n: sum(e[i].elapsed_time(e[i + 1]) for e in evs) / args.steps for i, n in enumerate(names)}
    fwd_ms = ms["fwd"]
    bwd_ms = sum(ms[n] for n in stage_names)
    step_ms = evs[0][0].elapsed_time(evs[-1][6]) / args.steps

    # dominant kernel and its roofline: algorithmic flops of that launch / its measured duration.
    # dK/dV kernels: S, dP, dV, dK = 8*D per pair they own; dQ kernel: only dQ is new work (2*D per
    # pair), its recomputed S and dP are overhead and not counted.
    alg = {"fwd": flops_fwd, "dkdv_gist": 8.0 * D * far_pairs * B * Hq,
           "dkdv_window": 8.0 * D * (nvis - far_pairs) * B * Hq, "dq": 2.0 * D * nvis * B * Hq}
    # Dominant = the launch that carries most of the step's algorithmic FLOPs (the gist-phase dK/dV kernel: 43 % of
    # the step's 14*D per pair on this workload).  It and the dQ kernel take the same time to within a percent,
    # so "the longest" would flip from box to box; every kernel's own figure is in `kernels` beside it.
    dom = max(alg, key=lambda n: alg[n])
    achieved = alg[dom] / ms[dom] / 1e9
    roofline = {"kernel": dom, "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_BF16_TFLOPS, "traffic": TRAFFIC_BYTES.get(dom),
                "avg_ms": ms[dom], "alg_flops_per_launch": alg[dom],
                "kernels": {n: {"avg_ms": ms[n], "alg_flops_per_launch": alg[n],
                                "frac": alg[n] / ms[n] / 1e9 / PEAK_BF16_TFLOPS,
                                # the dQ kernel executes three contractions (S, dP, dQ) to count one
                                "executed_frac": (3.0 if n == "dq" else 1.0) * alg[n] / ms[n] / 1e9 / PEAK_BF16_TFLOPS,
                                "traffic": TRAFFIC_BYTES.get(n)} for n in alg}}

    # what the matrix cores sustain on register-resident operands, outside the timed region: the chip is
    # power-limited, so the rate with operands like the workload's (random) is below the published peak
    g = torch.Generator(device="cpu").manual_seed(0)
    probe = {}
    for name, ops in (("random_operands", torch.randn(16384, generator=g)), ("constant_operands", torch.ones(16384))):
        if args.no_probe:
            break
        tf, mhz = u.probe_mfma_rate(ops.to(torch.bfloat16).to(dev))
        probe[name] = {"tflops": tf, "clock_mhz": mhz}
    if probe:
        roofline["frac_of_sustained_random_operand_rate"] = achieved / probe["random_operands"]["tflops"]

    # decode on its own workload, its own timed region
    dc = synth.WORKLOADS["cfg5_decode"]
    dq_, dk_, dv_ = synth.decode_inputs(dc["B"], dc["Hq"], dc["Hkv"], dc["Lk"], dc["D"], seed=0, device=dev)
    dws = torch.empty(u.unigist_decode_workspace(dc["B"], dc["Hq"], dc["Hkv"], dc["Lk"], dc["D"], u.UNIGIST_BF16),
                      device=dev, dtype=torch.uint8)
    for _ in range(3):
        u.decode(dq_, dk_, dv_, workspace=dws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    nd = 20
    e0.record()
    for _ in range(nd):
        u.decode(dq_, dk_, dv_, workspace=dws)
    e1.record()
    torch.cuda.synchronize()
    dec_ms = e0.elapsed_time(e1) / nd
    dec_bytes = 2.0 * dc["B"] * dc["Hkv"] * dc["Lk"] * dc["D"] * 2
    # a decoding step = the new token's K/V written into the cache (ring layout: one or two rows per sequence and
    # kv head) + decode; the cache is in the state whose window and gists fill the cfg5 rows
    t_ring = (dc["Lk"] - W) * (r + 1) - 64
    i32 = lambda x: torch.full((dc["B"],), x, dtype=torch.int32, device=dev)
    rt, ract, rrows = i32(t_ring), i32(1), i32(0)
    knew = dk_[:, :, :1].contiguous()
    def decode_step():
        u.unigist_cache_ring_append(dk_.data_ptr(), dv_.data_ptr(), knew.data_ptr(), knew.data_ptr(), 1, rt.data_ptr(),
                                    ract.data_ptr(), dc["Lk"], rrows.data_ptr(), dc["B"], dc["Hkv"], dc["D"], r, W, 0,
                                    u.UNIGIST_WINDOW_SLIDING, u.UNIGIST_BF16, torch.cuda.current_stream().cuda_stream)
        u.decode(dq_, dk_, dv_, rrows, workspace=dws)
    for _ in range(3):
        decode_step()
    torch.cuda.synchronize()
    assert int(rrows[0]) == u.unigist_cache_ring_rows(t_ring + 1, r, W, 0, 0) <= dc["Lk"]
    e0.record()
    for _ in range(nd):
        decode_step()
    e1.record()
    torch.cuda.synchronize()
    dec_step_ms = e0.elapsed_time(e1) / nd
    dec_gbs = dec_bytes / dec_ms / 1e6
    # what a kernel that only reads a buffer of that size reaches on this machine: the ceiling the memory system delivers
    stream_gbs = None
    if not args.no_probe:
        stream_gbs = max(u.probe_read_rate(int(dec_bytes) // 16 * 16, blocks=nb) for nb in (2048, 4096, 8192, 16384))
    # the same cache stored as E4M3 codes (one byte per element, per-kv-head scales): half the bytes to stream
    ks_, vs_ = synth.e4m3_scales(dc["Hkv"], seed=0, device=dev)
    k8_, v8_ = u.quantize_e4m3(dk_, ks_), u.quantize_e4m3(dv_, vs_)
    del dk_, dv_
    for _ in range(3):
        u.decode_e4m3(dq_, k8_, v8_, ks_, vs_, workspace=dws)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(nd):
        u.decode_e4m3(dq_, k8_, v8_, ks_, vs_, workspace=dws)
    e1.record()
    torch.cuda.synchronize()
    dec8_ms = e0.elapsed_time(e1) / nd
    dec8_bytes = dec_bytes / 2
    dec8_gbs = dec8_bytes / dec8_ms / 1e6
    del dq_, k8_, v8_, dws

    # chunk-wise prefill of the same 32K sequence through the compressed cache (4096-token chunks), own region
    C = 4096
    cache = u.KVCache(B, Hkv, min(L, W + C) + L // (r + 1) + 8, D, r)
    pout, plse = torch.empty_like(q), torch.empty(B, Hq, L, device=dev, dtype=torch.float32)
    def prefill_pass():  # the chunks are row slices of q, k, v, out and lse: nothing is copied out
        cache.cur, cache.s, cache.t = 0, 0, -1
        for p0 in range(0, L, C):
            n = min(C, L - p0)
            cache.update(k[:, :, p0:p0 + n], v[:, :, p0:p0 + n], max(0, p0 - W + 1))
            u.prefill_chunk(q[:, :, p0:p0 + n], cache, r, W, p0, out=pout[:, :, p0:p0 + n], lse=plse[:, :, p0:p0 + n])
    prefill_ms = None
    if not args.no_prefill:
        prefill_pass()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            prefill_pass()
        e1.record()
        torch.cuda.synchronize()
        prefill_ms = e0.elapsed_time(e1) / 3

    bm, bn = u.unigist_tile_sizes(D, u.UNIGIST_BF16)
    m = u.unigist_blockmap_build(L, r, W, bm, bn)
    # the same 32K tokens as a pack of five documents (attention confined to each), own region
    pack = None
    if not args.no_prefill:
        lens = [8192, 4100, 12288, 1020, 7168]
        cu = [0]
        for n in lens:
            cu.append(cu[-1] + n)
        q1, k1, v1, d1 = q[0], k[0], v[0], dout[0]
        po, pl_ = u.attn_fwd_varlen(q1, k1, v1, r, W, cu)
        pws = torch.empty(u.unigist_attn_bwd_varlen_workspace(Hq, Hkv, L, D, r, W, cu, u.UNIGIST_BF16), dtype=torch.uint8,
                          device="cuda")
        pack_nvis = sum(u.n_vis(n, r, W) for n in lens)
        pack = {"workload": f"{WORKLOAD} as a pack of documents of {lens} tokens"}
        for name, fn, fl in (("fwd", lambda: u.attn_fwd_varlen(q1, k1, v1, r, W, cu), 4.0),
                             ("bwd", lambda: u.attn_bwd_varlen(q1, k1, v1, po, pl_, d1, r, W, cu, workspace=pws), 10.0)):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                fn()
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) / 10
            tf = fl * D * pack_nvis * Hq / t / 1e9
            pack[name] = {"ms": t, "tflops": tf, "pct_of_peak": 100.0 * tf / PEAK_BF16_TFLOPS}
        del po, pl_, pws

    value = (flops_fwd + flops_bwd) / step_ms / 1e9
    res = {
        "metric": "gist-attn fwd+bwd TFLOP/s (unmasked) @32K GQA; % of bf16 MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": step_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOAD, "B": B, "Hq": Hq, "Hkv": Hkv, "L": L, "D": D, "r": r, "W": W,
                   "visible_pairs_per_head": nvis, "live_tile_fraction": m["live_tiles"] / m["causal_tiles"]},
        "pct_of_bf16_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "fwd": {"ms": fwd_ms, "tflops": flops_fwd / fwd_ms / 1e9, "pct_of_peak": flops_fwd / fwd_ms / 1e9 / PEAK_BF16_TFLOPS * 100},
        "bwd": {"ms": bwd_ms, "tflops": flops_bwd / bwd_ms / 1e9, "pct_of_peak": flops_bwd / bwd_ms / 1e9 / PEAK_BF16_TFLOPS * 100,
                "stage_ms": {n: ms[n] for n in stage_names}},
        "wall_ms_per_step": wall_ms,
        "roofline": roofline,
        "mfma_sustained": probe or None,
        "decode": {"workload": "cfg5_decode", "ms": dec_ms, "roofline": {
            "bound": "hbm", "achieved": dec_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": dec_gbs / PEAK_HBM_GBS,
            "traffic": TRAFFIC_BYTES.get("decode"), "alg_bytes_per_launch": dec_bytes,
            "measured_streaming_read_gbs": stream_gbs,
            "frac_of_measured_streaming_read": dec_gbs / stream_gbs if stream_gbs else None},
            "step_ms_with_cache_append": dec_step_ms},
        "decode_e4m3": {"workload": "cfg5_decode, cache stored as E4M3 codes", "ms": dec8_ms, "roofline": {
            "bound": "hbm", "achieved": dec8_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": dec8_gbs / PEAK_HBM_GBS,
            "traffic": TRAFFIC_BYTES.get("decode_e4m3"), "alg_bytes_per_launch": dec8_bytes}},
    }
    if pack is not None:
        res["packed_documents"] = pack
    if prefill_ms is not None:
        res["prefill"] = {"workload": f"{WORKLOAD} in {C}-token chunks through the compressed cache", "ms": prefill_ms,
                          "tflops": flops_fwd / prefill_ms / 1e9,
                          "note": "includes the cache updates; the chunks are row slices, nothing is copied out"}
    if not args.no_other_shapes:
        del q, k, v, dout, ws, grads, pout, plse, cache
        torch.cuda.empty_cache()
        c3 = synth.WORKLOADS["cfg3_long_128k"]
        res["cfg3_long_128k"] = dict(B=c3["B"], Hq=c3["Hq"], Hkv=c3["Hkv"], L=c3["L"], D=c3["D"], r=c3["r"], W=c3["W"],
                                     **time_shape(c3["B"], c3["Hq"], c3["Hkv"], c3["L"], c3["D"], c3["r"], c3["W"]))
        c4 = synth.WORKLOADS["cfg4_ratio_sweep"]
        res["cfg4_ratio_sweep"] = {"B": c4["B"], "Hq": c4["Hq"], "Hkv": c4["Hkv"], "L": c4["L"], "D": c4["D"], "W": c4["W"],
                                   "per_r": {str(rr): time_shape(c4["B"], c4["Hq"], c4["Hkv"], c4["L"], c4["D"], rr, c4["W"],
                                                                 steps=5) for rr in c4["r"]}}
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
