"""ctypes binding of libunigist.so.  Same names as the C ABI (include/unigist.h);
argument marshalling only.  Tensors are torch tensors on the GPU; nothing here
computes anything and there is no CPU fallback."""
from __future__ import annotations

import ctypes as C
import os

import torch

UNIGIST_BF16 = 0
UNIGIST_F32 = 1
BWD_STAGES = {"delta": 1, "dkdv_gist": 2, "gist_reduce": 4, "dkdv_window": 8, "dq": 16}
UNIGIST_BWD_ALL = 31
UNIGIST_E4M3 = 2  # storage type of the compressed cache only (uint8 tensors here)
UNIGIST_WINDOW_SLIDING = 0
UNIGIST_WINDOW_UNITS = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = [
    "unigist_status_str", "unigist_attn_fwd", "unigist_attn_bwd", "unigist_attn_bwd_stages",
    "unigist_attn_bwd_workspace",
    "unigist_decode", "unigist_decode_workspace", "unigist_blockmap_build", "unigist_blockmap_free",
    "unigist_tile_sizes", "unigist_cache_rows", "unigist_cache_update", "unigist_prefill_chunk",
    "unigist_attn_fwd_ex", "unigist_attn_bwd_ex", "unigist_attn_bwd_workspace_ex", "unigist_blockmap_build_ex",
    "unigist_attn_fwd_varlen", "unigist_attn_bwd_varlen", "unigist_attn_bwd_varlen_workspace",
    "unigist_cache_rows_ex", "unigist_cache_update_ex", "unigist_prefill_chunk_ex",
    "unigist_probe_mfma_rate", "unigist_quantize_e4m3", "unigist_decode_e4m3", "unigist_cache_update_ragged",
    "unigist_prefill_chunk_ragged", "unigist_prefill_chunk_e4m3", "unigist_prefill_chunk_e4m3_workspace",
    "unigist_attn_fwd_varlen_ex", "unigist_attn_bwd_varlen_ex", "unigist_attn_bwd_varlen_workspace_ex",
    "unigist_prefill_chunk_view", "unigist_prefill_chunk_strided", "unigist_attn_fwd_strided", "unigist_attn_bwd_strided",
    "unigist_attn_fwd_varlen_strided", "unigist_attn_bwd_varlen_strided",
    "unigist_cache_ring_rows", "unigist_cache_to_ring", "unigist_cache_from_ring", "unigist_cache_ring_append",
    "unigist_decode_noalloc", "unigist_decode_noalloc_scratch_bytes", "unigist_debug_force_plain_alu",
    "unigist_window_start", "unigist_plan_row_tile", "unigist_bwd_plan_build", "unigist_plan_key_tile", "unigist_plan_gist_unit",
    "unigist_probe_read_rate",
]


class UnigistError(RuntimeError):
    pass


class _BlockMap(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("L", "r", "W", "Bm", "Bn", "n_qtiles", "n_ktiles", "n_gists", "n_gtiles")] + \
               [(n, C.POINTER(C.c_int)) for n in ("win_first", "win_last", "n_far_gists", "n_full", "qt_first",
                                                   "qt_last", "gist_qt_first")] + \
               [(n, C.c_int64) for n in ("live_tiles", "masked_tiles", "causal_tiles", "n_vis")] + \
               [(n, C.c_int) for n in ("sinks", "window_mode")]


class _RowTilePlan(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("Bm", "Bn", "rows_per_wave", "wstart", "nfar", "n_gist_steps", "n_window_steps")]


class _BwdPlan(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("key_tile", "chunk_rows", "n_chunks", "n_key_tiles", "n_gist_tiles", "seg_chunks",
                                       "n_segs")] + [("slot0", C.c_int * 33)] + \
               [(n, C.c_size_t) for n in ("partial_bytes", "reduced_bytes", "workspace_bytes")]


def lib_path() -> str:
    """The in-tree library, or the one UNIGIST_LIB points at (for comparing builds)."""
    return os.environ.get("UNIGIST_LIB") or os.path.join(_HERE, "libunigist.so")


def load():
    """Load libunigist.so (once).  Raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise UnigistError(f"{path} is missing: build it with `python -m paper_2509_15763_amd.build` "
                           "(there is no fallback implementation)")
    lib = C.CDLL(path)
    vp, ip, sz, fp = C.c_void_p, C.c_int, C.c_size_t, C.c_void_p
    lib.unigist_status_str.restype = C.c_char_p
    lib.unigist_status_str.argtypes = [ip]
    lib.unigist_attn_fwd.restype = ip
    lib.unigist_attn_fwd.argtypes = [vp, vp, vp, vp, fp] + [ip] * 7 + [ip, vp]
    lib.unigist_attn_bwd.restype = ip
    lib.unigist_attn_bwd.argtypes = [vp] * 9 + [ip] * 7 + [ip, vp, sz, vp]
    lib.unigist_attn_bwd_stages.restype = ip
    lib.unigist_attn_bwd_stages.argtypes = [vp] * 9 + [ip] * 7 + [ip, vp, sz, C.c_uint, vp]
    lib.unigist_attn_bwd_workspace.restype = sz
    lib.unigist_attn_bwd_workspace.argtypes = [ip] * 7 + [ip]
    lib.unigist_attn_fwd_ex.restype = ip
    lib.unigist_attn_fwd_ex.argtypes = [vp, vp, vp, vp, fp] + [ip] * 9 + [ip, vp]
    lib.unigist_attn_bwd_ex.restype = ip
    lib.unigist_attn_bwd_ex.argtypes = [vp] * 9 + [ip] * 9 + [ip, vp, sz, C.c_uint, vp]
    lib.unigist_attn_bwd_workspace_ex.restype = sz
    lib.unigist_attn_bwd_workspace_ex.argtypes = [ip] * 9 + [ip]
    lib.unigist_blockmap_build_ex.restype = ip
    lib.unigist_blockmap_build_ex.argtypes = [ip] * 7 + [C.POINTER(C.POINTER(_BlockMap))]
    cup = C.POINTER(C.c_int)
    lib.unigist_attn_fwd_varlen.restype = ip
    lib.unigist_attn_fwd_varlen.argtypes = [vp, vp, vp, vp, fp] + [ip] * 6 + [cup, ip, ip, vp]
    lib.unigist_attn_bwd_varlen.restype = ip
    lib.unigist_attn_bwd_varlen.argtypes = [vp] * 9 + [ip] * 6 + [cup, ip, ip, vp, sz, vp]
    lib.unigist_attn_bwd_varlen_workspace.restype = sz
    lib.unigist_attn_bwd_varlen_workspace.argtypes = [ip] * 6 + [cup, ip, ip]
    lib.unigist_attn_fwd_varlen_ex.restype = ip
    lib.unigist_attn_fwd_varlen_ex.argtypes = [vp, vp, vp, vp, fp] + [ip] * 8 + [cup, ip, ip, vp]
    lib.unigist_attn_bwd_varlen_ex.restype = ip
    lib.unigist_attn_bwd_varlen_ex.argtypes = [vp] * 9 + [ip] * 8 + [cup, ip, ip, vp, sz, vp]
    lib.unigist_attn_bwd_varlen_workspace_ex.restype = sz
    lib.unigist_attn_bwd_varlen_workspace_ex.argtypes = [ip] * 8 + [cup, ip, ip]
    lib.unigist_decode.restype = ip
    lib.unigist_decode.argtypes = [vp, vp, vp, vp, fp, ip, ip, ip, ip, vp, ip, ip, vp, sz, vp]
    lib.unigist_decode_noalloc.restype = ip
    lib.unigist_decode_noalloc.argtypes = [vp, vp, vp, vp, fp, ip, ip, ip, ip, vp, ip, ip, vp]
    lib.unigist_plan_row_tile.restype = ip
    lib.unigist_plan_row_tile.argtypes = [ip] * 7 + [C.POINTER(_RowTilePlan), ip, vp]
    lib.unigist_bwd_plan_build.restype = ip
    lib.unigist_bwd_plan_build.argtypes = [ip] * 9 + [C.POINTER(_BwdPlan)]
    lib.unigist_plan_gist_unit.restype = ip
    lib.unigist_plan_gist_unit.argtypes = [ip] * 10 + [C.POINTER(ip), C.POINTER(ip)]
    lib.unigist_plan_key_tile.restype = ip
    lib.unigist_plan_key_tile.argtypes = [ip] * 12 + [C.POINTER(ip), C.POINTER(ip), ip, vp, vp]
    lib.unigist_window_start.restype = ip
    lib.unigist_window_start.argtypes = [ip] * 5
    lib.unigist_debug_force_plain_alu.restype = ip
    lib.unigist_debug_force_plain_alu.argtypes = [ip]
    lib.unigist_decode_noalloc_scratch_bytes.restype = sz
    lib.unigist_decode_noalloc_scratch_bytes.argtypes = []
    lib.unigist_quantize_e4m3.restype = ip
    lib.unigist_quantize_e4m3.argtypes = [vp, vp, vp, ip, ip, ip, ip, ip, vp]
    lib.unigist_decode_e4m3.restype = ip
    lib.unigist_decode_e4m3.argtypes = [vp, vp, vp, vp, vp, vp, fp, ip, ip, ip, ip, vp, ip, vp, sz, vp]
    lib.unigist_decode_workspace.restype = sz
    lib.unigist_decode_workspace.argtypes = [ip] * 5 + [ip]
    lib.unigist_blockmap_build.restype = ip
    lib.unigist_blockmap_build.argtypes = [ip] * 5 + [C.POINTER(C.POINTER(_BlockMap))]
    lib.unigist_blockmap_free.restype = None
    lib.unigist_blockmap_free.argtypes = [C.POINTER(_BlockMap)]
    lib.unigist_cache_rows_ex.restype = ip
    lib.unigist_cache_rows_ex.argtypes = [ip, ip, ip, ip]
    lib.unigist_cache_update_ex.restype = ip
    lib.unigist_cache_update_ex.argtypes = [vp, vp, ip, ip, ip, vp, vp, ip, ip, vp, vp, ip, ip, ip, ip, ip, ip, ip, ip, vp]
    lib.unigist_cache_update_ragged.restype = ip
    lib.unigist_cache_update_ragged.argtypes = [vp, vp, vp, vp, ip, vp, vp, vp, ip, vp, vp, vp, ip, vp] + [ip] * 6 + [vp]
    lib.unigist_prefill_chunk_ex.restype = ip
    lib.unigist_prefill_chunk_ex.argtypes = [vp, vp, vp, vp, fp] + [ip] * 13 + [vp]
    lib.unigist_cache_ring_rows.restype = ip
    lib.unigist_cache_ring_rows.argtypes = [ip] * 5
    for fn in (lib.unigist_cache_to_ring, lib.unigist_cache_from_ring):
        fn.restype = ip
        fn.argtypes = [vp, vp, vp, vp, ip, vp, vp, ip, vp] + [ip] * 8 + [vp]
    lib.unigist_cache_ring_append.restype = ip
    lib.unigist_cache_ring_append.argtypes = [vp, vp, vp, vp, ip, vp, vp, ip, vp] + [ip] * 8 + [vp]
    lib.unigist_attn_fwd_varlen_strided.restype = ip
    lib.unigist_attn_fwd_varlen_strided.argtypes = [vp, vp, vp, vp, fp] + [ip] * 8 + [cup, ip] + [C.c_longlong] * 2 + [ip, vp]
    lib.unigist_attn_bwd_varlen_strided.restype = ip
    lib.unigist_attn_bwd_varlen_strided.argtypes = [vp] * 9 + [ip] * 8 + [cup, ip] + [C.c_longlong] * 2 + [ip, vp, sz, vp]
    lib.unigist_attn_fwd_strided.restype = ip
    lib.unigist_attn_fwd_strided.argtypes = [vp, vp, vp, vp, fp] + [ip] * 9 + [C.c_longlong] * 3 + [ip, vp]
    lib.unigist_attn_bwd_strided.restype = ip
    lib.unigist_attn_bwd_strided.argtypes = [vp] * 9 + [ip] * 9 + [C.c_longlong] * 3 + [ip, vp, sz, vp]
    lib.unigist_prefill_chunk_strided.restype = ip
    lib.unigist_prefill_chunk_strided.argtypes = [vp, vp, vp, vp, fp] + [ip] * 12 + [C.c_longlong] * 3 + [ip, vp]
    lib.unigist_prefill_chunk_view.restype = ip
    lib.unigist_prefill_chunk_view.argtypes = [vp, vp, vp, vp, fp] + [ip] * 14 + [vp]
    lib.unigist_prefill_chunk_ragged.restype = ip
    lib.unigist_prefill_chunk_ragged.argtypes = [vp, vp, vp, vp, fp] + [ip] * 9 + [vp, vp, vp, ip, vp, ip, vp]
    lib.unigist_prefill_chunk_e4m3_workspace.restype = sz
    lib.unigist_prefill_chunk_e4m3_workspace.argtypes = [ip] * 7
    lib.unigist_prefill_chunk_e4m3.restype = ip
    lib.unigist_prefill_chunk_e4m3.argtypes = [vp, vp, vp, vp, vp, vp, fp] + [ip] * 12 + [vp, sz, vp]
    lib.unigist_cache_rows.restype = ip
    lib.unigist_cache_rows.argtypes = [ip, ip, ip]
    lib.unigist_cache_update.restype = ip
    lib.unigist_cache_update.argtypes = [vp, vp, ip, ip, ip, vp, vp, ip, ip, vp, vp, ip, ip, ip, ip, ip, ip, ip, vp]
    lib.unigist_prefill_chunk.restype = ip
    lib.unigist_prefill_chunk.argtypes = [vp, vp, vp, vp, fp] + [ip] * 10 + [ip, vp]
    lib.unigist_probe_read_rate.restype = ip
    lib.unigist_probe_read_rate.argtypes = [vp, sz, vp, ip, vp]
    lib.unigist_probe_mfma_rate.restype = ip
    lib.unigist_probe_mfma_rate.argtypes = [vp, vp, vp, ip, ip, vp]
    lib.unigist_tile_sizes.restype = None
    lib.unigist_tile_sizes.argtypes = [ip, ip, C.POINTER(ip), C.POINTER(ip)]
    _LIB = lib
    return lib


def _check(st: int, what: str):
    if st != 0:
        raise UnigistError(f"{what}: {unigist_status_str(st)} (status {st})")


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return UNIGIST_BF16
    if t.dtype == torch.float32:
        return UNIGIST_F32
    raise UnigistError(f"unsupported dtype {t.dtype}")


def _dev(*ts):
    for t in ts:
        if t is None:
            continue
        if not t.is_cuda:
            raise UnigistError("libunigist takes device tensors only (no CPU path)")
        if not t.is_contiguous():
            raise UnigistError("tensors must be contiguous [B,H,L,D]")


def _head_rows(t: torch.Tensor, lead: int) -> int:
    """Rows between consecutive heads of t [..., H, n, D] (lead dims in front of H), which may be a slice along the
    row axis of a larger contiguous tensor; raises for any other layout."""
    if not t.is_cuda:
        raise UnigistError("libunigist takes device tensors only (no CPU path)")
    n, D = t.shape[-2], t.shape[-1]
    st = t.stride()
    rows = st[-3] // D if D and st[-3] % D == 0 else -1
    ok = st[-1] == 1 and st[-2] == D and rows >= n
    for i in range(lead):  # the dims in front of H must be laid out densely over heads of `rows` rows
        ok = ok and (t.shape[i] == 1 or st[i] == st[i + 1] * t.shape[i + 1])
    if not ok:
        raise UnigistError("tensor must be contiguous or a slice along the row axis of a contiguous [.., H, rows, D] tensor")
    return rows


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


# ---------------------------------------------------------------- raw ABI, same names
def unigist_status_str(st: int) -> str:
    return load().unigist_status_str(int(st)).decode()


def unigist_attn_fwd(q, k, v, out, lse, B, Hq, Hkv, L, D, r, W, dt, stream=None) -> int:
    return load().unigist_attn_fwd(q, k, v, out, lse, B, Hq, Hkv, L, D, r, W, dt, stream)


def unigist_attn_bwd(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, L, D, r, W, dt, ws, ws_bytes, stream=None) -> int:
    return load().unigist_attn_bwd(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, L, D, r, W, dt, ws, ws_bytes,
                                   stream)


def unigist_attn_bwd_stages(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, L, D, r, W, dt, ws, ws_bytes, stages,
                            stream=None) -> int:
    return load().unigist_attn_bwd_stages(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, L, D, r, W, dt, ws,
                                          ws_bytes, stages, stream)


def unigist_attn_bwd_workspace(B, Hq, Hkv, L, D, r, W, dt) -> int:
    return load().unigist_attn_bwd_workspace(B, Hq, Hkv, L, D, r, W, dt)


def unigist_attn_fwd_ex(q, k, v, out, lse, B, Hq, Hkv, L, D, r, W, sinks, window_mode, dt, stream=None) -> int:
    return load().unigist_attn_fwd_ex(q, k, v, out, lse, B, Hq, Hkv, L, D, r, W, sinks, window_mode, dt, stream)


def unigist_attn_bwd_ex(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, L, D, r, W, sinks, window_mode, dt, ws,
                        ws_bytes, stages, stream=None) -> int:
    return load().unigist_attn_bwd_ex(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, L, D, r, W, sinks,
                                      window_mode, dt, ws, ws_bytes, stages, stream)


def unigist_attn_bwd_workspace_ex(B, Hq, Hkv, L, D, r, W, sinks, window_mode, dt) -> int:
    return load().unigist_attn_bwd_workspace_ex(B, Hq, Hkv, L, D, r, W, sinks, window_mode, dt)


def _cu(cu_seqlens):
    """Host int array for the *_varlen calls (None stays a null pointer) and its document count."""
    if cu_seqlens is None:
        return None, 0
    vals = [int(x) for x in cu_seqlens]
    return (C.c_int * len(vals))(*vals), len(vals) - 1


def unigist_attn_fwd_varlen(q, k, v, out, lse, Hq, Hkv, T, D, r, W, cu_seqlens, dt, stream=None) -> int:
    cu, nd = _cu(cu_seqlens)
    return load().unigist_attn_fwd_varlen(q, k, v, out, lse, Hq, Hkv, T, D, r, W, cu, nd, dt, stream)


def unigist_attn_bwd_varlen(q, k, v, out, lse, dout, dq, dk, dv, Hq, Hkv, T, D, r, W, cu_seqlens, dt, ws, ws_bytes,
                            stream=None) -> int:
    cu, nd = _cu(cu_seqlens)
    return load().unigist_attn_bwd_varlen(q, k, v, out, lse, dout, dq, dk, dv, Hq, Hkv, T, D, r, W, cu, nd, dt, ws,
                                          ws_bytes, stream)


def unigist_attn_fwd_varlen_ex(q, k, v, out, lse, Hq, Hkv, T, D, r, W, sinks, window_mode, cu_seqlens, dt,
                               stream=None) -> int:
    cu, nd = _cu(cu_seqlens)
    return load().unigist_attn_fwd_varlen_ex(q, k, v, out, lse, Hq, Hkv, T, D, r, W, sinks, window_mode, cu, nd, dt, stream)


def unigist_attn_bwd_varlen_ex(q, k, v, out, lse, dout, dq, dk, dv, Hq, Hkv, T, D, r, W, sinks, window_mode, cu_seqlens,
                               dt, ws, ws_bytes, stream=None) -> int:
    cu, nd = _cu(cu_seqlens)
    return load().unigist_attn_bwd_varlen_ex(q, k, v, out, lse, dout, dq, dk, dv, Hq, Hkv, T, D, r, W, sinks, window_mode,
                                             cu, nd, dt, ws, ws_bytes, stream)


def unigist_attn_bwd_varlen_workspace_ex(Hq, Hkv, T, D, r, W, sinks, window_mode, cu_seqlens, dt) -> int:
    cu, nd = _cu(cu_seqlens)
    return load().unigist_attn_bwd_varlen_workspace_ex(Hq, Hkv, T, D, r, W, sinks, window_mode, cu, nd, dt)


def unigist_attn_bwd_varlen_workspace(Hq, Hkv, T, D, r, W, cu_seqlens, dt) -> int:
    cu, nd = _cu(cu_seqlens)
    return load().unigist_attn_bwd_varlen_workspace(Hq, Hkv, T, D, r, W, cu, nd, dt)


def unigist_decode(q, kc, vc, out, lse, B, Hq, Hkv, Lk, seqlens, D, dt, ws, ws_bytes, stream=None) -> int:
    return load().unigist_decode(q, kc, vc, out, lse, B, Hq, Hkv, Lk, seqlens, D, dt, ws, ws_bytes, stream)


def unigist_decode_noalloc(q, kc, vc, out, lse, B, Hq, Hkv, Lk, seqlens, D, dt, stream=None) -> int:
    return load().unigist_decode_noalloc(q, kc, vc, out, lse, B, Hq, Hkv, Lk, seqlens, D, dt, stream)


UNIGIST_WALK_FWD, UNIGIST_WALK_DQ = 0, 1


def unigist_plan_row_tile(L, r, W, sinks, window_mode, kernel, tile) -> dict:
    """The forward (kernel = UNIGIST_WALK_FWD) or dQ walk of query tile `tile`, as a dict; "kind" is an int8 numpy
    array [waves, steps] (0 skipped, 1 no mask, 2 masked)."""
    import numpy as np
    p = _RowTilePlan()
    _check(load().unigist_plan_row_tile(L, r, W, sinks, window_mode, kernel, tile, C.byref(p), 0, None),
           "unigist_plan_row_tile")
    nw, ns = p.Bm // p.rows_per_wave, p.n_gist_steps + p.n_window_steps
    kind = np.zeros((nw, ns), dtype=np.int8)
    _check(load().unigist_plan_row_tile(L, r, W, sinks, window_mode, kernel, tile, C.byref(p), kind.size,
                                        kind.ctypes.data), "unigist_plan_row_tile")
    d = {n: getattr(p, n) for n, _ in _RowTilePlan._fields_}
    d["kind"] = kind
    return d


def unigist_bwd_plan_build(B, Hq, Hkv, L, D, r, W, sinks=0, window_mode=UNIGIST_WINDOW_SLIDING) -> dict:
    p = _BwdPlan()
    _check(load().unigist_bwd_plan_build(B, Hq, Hkv, L, D, r, W, sinks, window_mode, C.byref(p)), "unigist_bwd_plan_build")
    d = {n: getattr(p, n) for n, _ in _BwdPlan._fields_ if n != "slot0"}
    d["slot0"] = list(p.slot0)[: p.n_segs + 1]
    return d


def unigist_plan_gist_unit(B, Hq, Hkv, L, D, r, W, sinks, window_mode, unit) -> tuple:
    """-> (segment, compact tile) of the gist-phase workgroup `unit` in launch order."""
    seg, tile = C.c_int(0), C.c_int(0)
    _check(load().unigist_plan_gist_unit(B, Hq, Hkv, L, D, r, W, sinks, window_mode, unit, C.byref(seg), C.byref(tile)),
           "unigist_plan_gist_unit")
    return seg.value, tile.value


def unigist_plan_key_tile(B, Hq, Hkv, L, D, r, W, sinks, window_mode, gist_phase, tile, seg=0) -> dict:
    """One dK/dV workgroup: {"c_lo", "c_hi", "nfar": int32 [chunks], "kind": int8 [4 waves, chunks, 2 row blocks]}."""
    import numpy as np
    lo, hi = C.c_int(0), C.c_int(-1)
    args = (B, Hq, Hkv, L, D, r, W, sinks, window_mode, int(bool(gist_phase)), tile, seg)
    _check(load().unigist_plan_key_tile(*args, C.byref(lo), C.byref(hi), 0, None, None), "unigist_plan_key_tile")
    n = max(0, hi.value - lo.value + 1)
    nfar = np.zeros(max(n, 1), dtype=np.int32)
    kind = np.zeros((4, max(n, 1), 2), dtype=np.int8)
    _check(load().unigist_plan_key_tile(*args, C.byref(lo), C.byref(hi), n, nfar.ctypes.data, kind.ctypes.data),
           "unigist_plan_key_tile")
    return {"c_lo": lo.value, "c_hi": hi.value, "nfar": nfar[:n], "kind": kind[:, :n]}


def unigist_window_start(t, r, W, sinks=0, window_mode=UNIGIST_WINDOW_SLIDING) -> int:
    return load().unigist_window_start(int(t), int(r), int(W), int(sinks), int(window_mode))


def unigist_debug_force_plain_alu(on) -> int:
    return load().unigist_debug_force_plain_alu(int(bool(on)))


def unigist_decode_noalloc_scratch_bytes() -> int:
    return load().unigist_decode_noalloc_scratch_bytes()


def unigist_quantize_e4m3(x, y, scale, B, H, n, D, dt_in, stream=None) -> int:
    return load().unigist_quantize_e4m3(x, y, scale, B, H, n, D, dt_in, stream)


def unigist_decode_e4m3(q, kc, vc, k_scale, v_scale, out, lse, B, Hq, Hkv, Lk, seqlens, D, ws, ws_bytes, stream=None) -> int:
    return load().unigist_decode_e4m3(q, kc, vc, k_scale, v_scale, out, lse, B, Hq, Hkv, Lk, seqlens, D, ws, ws_bytes, stream)


def unigist_decode_workspace(B, Hq, Hkv, Lk, D, dt) -> int:
    return load().unigist_decode_workspace(B, Hq, Hkv, Lk, D, dt)


def unigist_cache_rows(s, t, r) -> int:
    return load().unigist_cache_rows(s, t, r)


def unigist_cache_update(kc_in, vc_in, s_old, t_old, cap_in, k_new, v_new, n_new, new_rows, kc_out, vc_out, s_new,
                         cap_out, B, Hkv, D, r, dt, stream=None) -> int:
    return load().unigist_cache_update(kc_in, vc_in, s_old, t_old, cap_in, k_new, v_new, n_new, new_rows, kc_out,
                                       vc_out, s_new, cap_out, B, Hkv, D, r, dt, stream)


def unigist_cache_rows_ex(s, t, r, sinks) -> int:
    return load().unigist_cache_rows_ex(s, t, r, sinks)


def unigist_cache_update_ex(kc_in, vc_in, s_old, t_old, cap_in, k_new, v_new, n_new, new_rows, kc_out, vc_out, s_new,
                            cap_out, B, Hkv, D, r, sinks, dt, stream=None) -> int:
    return load().unigist_cache_update_ex(kc_in, vc_in, s_old, t_old, cap_in, k_new, v_new, n_new, new_rows, kc_out,
                                          vc_out, s_new, cap_out, B, Hkv, D, r, sinks, dt, stream)


def unigist_prefill_chunk_ex(q, kc, vc, out, lse, B, Hq, Hkv, C, D, r, W, sinks, window_mode, p0, s, cap, dt,
                             stream=None) -> int:
    return load().unigist_prefill_chunk_ex(q, kc, vc, out, lse, B, Hq, Hkv, C, D, r, W, sinks, window_mode, p0, s,
                                           cap, dt, stream)


def unigist_cache_update_ragged(kc_in, vc_in, s_old, t_old, cap_in, k_new, v_new, n_new, new_rows, kc_out, vc_out, s_new,
                                cap_out, rows_out, B, Hkv, D, r, sinks, dt, stream=None) -> int:
    return load().unigist_cache_update_ragged(kc_in, vc_in, s_old, t_old, cap_in, k_new, v_new, n_new, new_rows, kc_out,
                                              vc_out, s_new, cap_out, rows_out, B, Hkv, D, r, sinks, dt, stream)


def unigist_cache_ring_rows(t, r, W, sinks=0, window_mode=UNIGIST_WINDOW_SLIDING) -> int:
    return load().unigist_cache_ring_rows(t, r, W, sinks, window_mode)


def unigist_cache_to_ring(kc_in, vc_in, s, t, cap_in, kc_out, vc_out, cap_out, rows_out, B, Hkv, D, r, W, sinks,
                          window_mode, dt, stream=None) -> int:
    return load().unigist_cache_to_ring(kc_in, vc_in, s, t, cap_in, kc_out, vc_out, cap_out, rows_out, B, Hkv, D, r, W,
                                        sinks, window_mode, dt, stream)


def unigist_cache_from_ring(kc_in, vc_in, s, t, cap_in, kc_out, vc_out, cap_out, rows_out, B, Hkv, D, r, W, sinks,
                            window_mode, dt, stream=None) -> int:
    return load().unigist_cache_from_ring(kc_in, vc_in, s, t, cap_in, kc_out, vc_out, cap_out, rows_out, B, Hkv, D, r, W,
                                          sinks, window_mode, dt, stream)


def unigist_cache_ring_append(kc, vc, k_new, v_new, new_rows, t_old, n_new, cap, rows_out, B, Hkv, D, r, W, sinks,
                              window_mode, dt, stream=None) -> int:
    return load().unigist_cache_ring_append(kc, vc, k_new, v_new, new_rows, t_old, n_new, cap, rows_out, B, Hkv, D, r, W,
                                            sinks, window_mode, dt, stream)


def unigist_prefill_chunk_view(q, kc, vc, out, lse, B, Hq, Hkv, C, q_rows, D, r, W, sinks, window_mode, p0, s, cap, dt,
                               stream=None) -> int:
    return load().unigist_prefill_chunk_view(q, kc, vc, out, lse, B, Hq, Hkv, C, q_rows, D, r, W, sinks, window_mode, p0,
                                             s, cap, dt, stream)


def unigist_attn_fwd_varlen_strided(q, k, v, out, lse, Hq, Hkv, T, D, r, W, sinks, window_mode, cu_seqlens, q_hs, q_rs, dt,
                                    stream=None) -> int:
    cu, nd = _cu(cu_seqlens)
    return load().unigist_attn_fwd_varlen_strided(q, k, v, out, lse, Hq, Hkv, T, D, r, W, sinks, window_mode, cu, nd, q_hs,
                                                  q_rs, dt, stream)


def unigist_attn_bwd_varlen_strided(q, k, v, out, lse, dout, dq, dk, dv, Hq, Hkv, T, D, r, W, sinks, window_mode,
                                    cu_seqlens, q_hs, q_rs, dt, ws, ws_bytes, stream=None) -> int:
    cu, nd = _cu(cu_seqlens)
    return load().unigist_attn_bwd_varlen_strided(q, k, v, out, lse, dout, dq, dk, dv, Hq, Hkv, T, D, r, W, sinks,
                                                  window_mode, cu, nd, q_hs, q_rs, dt, ws, ws_bytes, stream)


def unigist_attn_fwd_strided(q, k, v, out, lse, B, Hq, Hkv, L, D, r, W, sinks, window_mode, q_bs, q_hs, q_rs, dt,
                             stream=None) -> int:
    return load().unigist_attn_fwd_strided(q, k, v, out, lse, B, Hq, Hkv, L, D, r, W, sinks, window_mode, q_bs, q_hs, q_rs,
                                           dt, stream)


def unigist_attn_bwd_strided(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, L, D, r, W, sinks, window_mode, q_bs, q_hs,
                             q_rs, dt, ws, ws_bytes, stream=None) -> int:
    return load().unigist_attn_bwd_strided(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, L, D, r, W, sinks, window_mode,
                                           q_bs, q_hs, q_rs, dt, ws, ws_bytes, stream)


def unigist_prefill_chunk_strided(q, kc, vc, out, lse, B, Hq, Hkv, C, D, r, W, sinks, window_mode, p0, s, cap, q_bs, q_hs,
                                  q_rs, dt, stream=None) -> int:
    return load().unigist_prefill_chunk_strided(q, kc, vc, out, lse, B, Hq, Hkv, C, D, r, W, sinks, window_mode, p0, s,
                                                cap, q_bs, q_hs, q_rs, dt, stream)


def unigist_prefill_chunk_e4m3_workspace(B, Hkv, D, s, t, r, sinks) -> int:
    return load().unigist_prefill_chunk_e4m3_workspace(B, Hkv, D, s, t, r, sinks)


def unigist_prefill_chunk_e4m3(q, kc, vc, k_scale, v_scale, out, lse, B, Hq, Hkv, C, D, r, W, sinks, window_mode, p0, s,
                               cap, ws, ws_bytes, stream=None) -> int:
    return load().unigist_prefill_chunk_e4m3(q, kc, vc, k_scale, v_scale, out, lse, B, Hq, Hkv, C, D, r, W, sinks,
                                             window_mode, p0, s, cap, ws, ws_bytes, stream)


def unigist_prefill_chunk_ragged(q, kc, vc, out, lse, B, Hq, Hkv, C, D, r, W, sinks, window_mode, p0, n, s, cap,
                                 rows_out, dt, stream=None) -> int:
    return load().unigist_prefill_chunk_ragged(q, kc, vc, out, lse, B, Hq, Hkv, C, D, r, W, sinks, window_mode, p0, n,
                                               s, cap, rows_out, dt, stream)


def unigist_prefill_chunk(q, kc, vc, out, lse, B, Hq, Hkv, C, D, r, W, p0, s, cap, dt, stream=None) -> int:
    return load().unigist_prefill_chunk(q, kc, vc, out, lse, B, Hq, Hkv, C, D, r, W, p0, s, cap, dt, stream)


def unigist_probe_mfma_rate(operands, clocks, sink, blocks, iters, stream=None) -> int:
    return load().unigist_probe_mfma_rate(operands, clocks, sink, blocks, iters, stream)


def unigist_probe_read_rate(buf, nbytes, sink, blocks, stream=None) -> int:
    return load().unigist_probe_read_rate(buf, nbytes, sink, blocks, stream)


def probe_read_rate(nbytes=4 << 30, blocks=2048, reps=5):
    """GB/s of a kernel that only reads an nbytes buffer (allocated here), best of `reps` launches."""
    buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    sink = torch.zeros(2, dtype=torch.int32, device="cuda")
    run = lambda: _check(unigist_probe_read_rate(buf.data_ptr(), nbytes, sink.data_ptr(), blocks, _stream()),
                         "unigist_probe_read_rate")
    run()
    best = float("inf")
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1))
    return nbytes / best / 1e6


def probe_mfma_rate(operands, blocks=512, iters=100000):
    """operands: 32 KiB of bf16 on the GPU -> (TFLOP/s, clock in MHz) of a register-resident MFMA loop."""
    _dev(operands)
    if operands.dtype != torch.bfloat16 or operands.numel() != 16384 or not operands.is_contiguous():
        raise UnigistError("operands must be 16384 contiguous bf16 values")
    clocks = torch.zeros(2 * blocks, dtype=torch.int64, device=operands.device)
    sink = torch.zeros(1, dtype=torch.float32, device=operands.device)
    run = lambda: _check(unigist_probe_mfma_rate(operands.data_ptr(), clocks.data_ptr(), sink.data_ptr(), blocks, iters,
                                                 _stream()), "unigist_probe_mfma_rate")
    run()  # lets the clock settle under this load
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    run()
    e1.record()
    torch.cuda.synchronize()
    flops = blocks * 4 * iters * 8 * 2.0 * 32 * 32 * 16
    c = clocks.view(blocks, 2).sum(0).tolist()
    return flops / e0.elapsed_time(e1) / 1e9, 100.0 * c[0] / max(c[1], 1)


def unigist_tile_sizes(D, dt):
    bm, bn = C.c_int(0), C.c_int(0)
    load().unigist_tile_sizes(D, dt, C.byref(bm), C.byref(bn))
    return bm.value, bn.value


def unigist_blockmap_build(L, r, W, Bm, Bn) -> dict:
    """Host block map as a dict of python lists / ints (the C object is freed before returning)."""
    p = C.POINTER(_BlockMap)()
    _check(load().unigist_blockmap_build(L, r, W, Bm, Bn, C.byref(p)), "unigist_blockmap_build")
    return _blockmap_dict(p)


def unigist_blockmap_build_ex(L, r, W, sinks, window_mode, Bm, Bn) -> dict:
    p = C.POINTER(_BlockMap)()
    _check(load().unigist_blockmap_build_ex(L, r, W, sinks, window_mode, Bm, Bn, C.byref(p)),
           "unigist_blockmap_build_ex")
    return _blockmap_dict(p)


def _blockmap_dict(p) -> dict:
    try:
        m = p.contents
        d = {n: getattr(m, n) for n in ("L", "r", "W", "Bm", "Bn", "n_qtiles", "n_ktiles", "n_gists", "n_gtiles",
                                        "live_tiles", "masked_tiles", "causal_tiles", "n_vis", "sinks",
                                        "window_mode")}
        for n in ("win_first", "win_last", "n_far_gists", "n_full"):
            d[n] = [getattr(m, n)[i] for i in range(m.n_qtiles)]
        for n in ("qt_first", "qt_last"):
            d[n] = [getattr(m, n)[i] for i in range(m.n_ktiles)]
        d["gist_qt_first"] = [m.gist_qt_first[i] for i in range(m.n_gtiles)]
        return d
    finally:
        load().unigist_blockmap_free(p)


def n_vis(L, r, W, sinks=0, window_mode=UNIGIST_WINDOW_SLIDING) -> int:
    """Visible (query, key) pairs of one head: the unit the FLOP counts are quoted in."""
    return unigist_blockmap_build_ex(L, r, W, sinks, window_mode, 128, 128)["n_vis"]


# ---------------------------------------------------------------- conveniences (allocate outputs, check status)
def _q_strided(q) -> bool:
    """Is q a bf16 view with a contiguous last axis but not contiguous as a whole (e.g. the transposed view of a
    [B, L, Hq, D] or [T, Hq, D] projection output)?  Such a q goes through the *_strided entry points without a copy."""
    return (q.dtype == torch.bfloat16 and q.is_cuda and not q.is_contiguous() and q.stride(-1) == 1
            and all(s % 8 == 0 for s in q.stride()[:-1]) and q.stride(-2) >= q.shape[-1])


def attn_fwd(q, k, v, r, W, sinks=0, window_mode=UNIGIST_WINDOW_SLIDING):
    """q [B,Hq,L,D], k/v [B,Hkv,L,D] on the GPU -> out [B,Hq,L,D], lse [B,Hq,L] fp32.  A bf16 q that is a strided view
    (see _q_strided) is taken as it is and out gets the same strides."""
    B, Hq, L, D = q.shape
    Hkv = k.shape[1]
    if k.shape != (B, Hkv, L, D) or v.shape != k.shape or k.dtype != q.dtype or v.dtype != q.dtype:
        raise UnigistError("q/k/v shapes or dtypes disagree")
    if _q_strided(q):
        _dev(k, v)
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
        lse = torch.empty(B, Hq, L, device=q.device, dtype=torch.float32)
        _check(unigist_attn_fwd_strided(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                        B, Hq, Hkv, L, D, int(r), int(W), int(sinks), int(window_mode), q.stride(0),
                                        q.stride(1), q.stride(2), _dt(q), _stream()),
               "unigist_attn_fwd_strided")
        return out, lse
    _dev(q, k, v)
    out = torch.empty_like(q)
    lse = torch.empty(B, Hq, L, device=q.device, dtype=torch.float32)
    _check(unigist_attn_fwd_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                               B, Hq, Hkv, L, D, int(r), int(W), int(sinks), int(window_mode), _dt(q), _stream()),
           "unigist_attn_fwd_ex")
    return out, lse


def attn_bwd(q, k, v, out, lse, dout, r, W, workspace=None, stages=UNIGIST_BWD_ALL, grads=None, sinks=0,
             window_mode=UNIGIST_WINDOW_SLIDING):
    """-> dq [B,Hq,L,D], dk, dv [B,Hkv,L,D].  `stages`/`grads` let a caller run the backward one
    stage at a time into the same output tensors (per-kernel timing).  A strided bf16 q (see attn_fwd) with out of
    the same strides takes the strided entry point: dq gets q's strides, dout is brought to them if it differs."""
    B, Hq, L, D = q.shape
    Hkv = k.shape[1]
    dt = _dt(q)
    if out.shape != q.shape or dout.shape != q.shape or lse.shape != (B, Hq, L) or lse.dtype != torch.float32:
        raise UnigistError("out/dout/lse shapes or dtypes disagree")
    if k.shape != (B, Hkv, L, D) or v.shape != k.shape or len({t.dtype for t in (q, k, v, out, dout)}) != 1:
        raise UnigistError("q/k/v/out/dout shapes or dtypes disagree")
    if _q_strided(q) and out.stride() == q.stride() and stages == UNIGIST_BWD_ALL and grads is None:
        _dev(k, v, lse)
        if dout.stride() != q.stride():
            dout = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device).copy_(dout)
        need = unigist_attn_bwd_workspace_ex(B, Hq, Hkv, L, D, int(r), int(W), int(sinks), int(window_mode), dt)
        if need == 0:
            raise UnigistError("unigist_attn_bwd_workspace_ex: invalid or unsupported shape")
        if workspace is None:
            workspace = torch.empty(need, device=q.device, dtype=torch.uint8)
        dq = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
        dk, dv = torch.empty_like(k), torch.empty_like(v)
        _check(unigist_attn_bwd_strided(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                        dout.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), B, Hq, Hkv, L, D,
                                        int(r), int(W), int(sinks), int(window_mode), q.stride(0), q.stride(1),
                                        q.stride(2), dt, workspace.data_ptr(),
                                        workspace.numel() * workspace.element_size(), _stream()),
               "unigist_attn_bwd_strided")
        return dq, dk, dv
    _dev(q, k, v, out, lse, dout)
    need = unigist_attn_bwd_workspace_ex(B, Hq, Hkv, L, D, int(r), int(W), int(sinks), int(window_mode), dt)
    if need == 0:
        raise UnigistError("unigist_attn_bwd_workspace_ex: invalid or unsupported shape")
    if workspace is None:
        workspace = torch.empty(need, device=q.device, dtype=torch.uint8)
    dq, dk, dv = grads if grads is not None else (torch.empty_like(q), torch.empty_like(k), torch.empty_like(v))
    _check(unigist_attn_bwd_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                               dout.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), B, Hq, Hkv, L, D,
                               int(r), int(W), int(sinks), int(window_mode), dt, workspace.data_ptr(),
                               workspace.numel() * workspace.element_size(), int(stages), _stream()),
           "unigist_attn_bwd_ex")
    return dq, dk, dv


def attn_fwd_varlen(q, k, v, r, W, cu_seqlens, sinks=0, window_mode=UNIGIST_WINDOW_SLIDING):
    """Packed documents: q [Hq,T,D], k/v [Hkv,T,D] on the GPU, cu_seqlens a host sequence -> out, lse [Hq,T].  A bf16 q
    that is a strided view (e.g. of a [T, Hq, D] tensor) is taken as it is and out gets the same strides."""
    Hq, T, D = q.shape
    Hkv = k.shape[0]
    if k.shape != (Hkv, T, D) or v.shape != k.shape or k.dtype != q.dtype or v.dtype != q.dtype:
        raise UnigistError("q/k/v shapes or dtypes disagree")
    if _q_strided(q):
        _dev(k, v)
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
        lse = torch.empty(Hq, T, device=q.device, dtype=torch.float32)
        _check(unigist_attn_fwd_varlen_strided(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                               Hq, Hkv, T, D, int(r), int(W), int(sinks), int(window_mode), cu_seqlens,
                                               q.stride(0), q.stride(1), _dt(q), _stream()),
               "unigist_attn_fwd_varlen_strided")
        return out, lse
    _dev(q, k, v)
    out = torch.empty_like(q)
    lse = torch.empty(Hq, T, device=q.device, dtype=torch.float32)
    _check(unigist_attn_fwd_varlen_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                      Hq, Hkv, T, D, int(r), int(W), int(sinks), int(window_mode), cu_seqlens, _dt(q),
                                      _stream()),
           "unigist_attn_fwd_varlen_ex")
    return out, lse


def attn_bwd_varlen(q, k, v, out, lse, dout, r, W, cu_seqlens, workspace=None, sinks=0,
                    window_mode=UNIGIST_WINDOW_SLIDING):
    """-> dq [Hq,T,D], dk, dv [Hkv,T,D] for packed documents (dq with q's strides if q is a strided view)."""
    Hq, T, D = q.shape
    Hkv = k.shape[0]
    dt = _dt(q)
    if _q_strided(q) and out.stride() == q.stride() and out.shape == q.shape and dout.shape == q.shape:
        _dev(k, v, lse)
        if dout.stride() != q.stride():
            dout = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device).copy_(dout)
        need = unigist_attn_bwd_varlen_workspace_ex(Hq, Hkv, T, D, int(r), int(W), int(sinks), int(window_mode), cu_seqlens, dt)
        if need == 0:
            raise UnigistError("unigist_attn_bwd_varlen_workspace_ex: invalid shape or document bounds")
        if workspace is None:
            workspace = torch.empty(need, device=q.device, dtype=torch.uint8)
        dq = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
        dk, dv = torch.empty_like(k), torch.empty_like(v)
        _check(unigist_attn_bwd_varlen_strided(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                               dout.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), Hq, Hkv, T, D,
                                               int(r), int(W), int(sinks), int(window_mode), cu_seqlens, q.stride(0),
                                               q.stride(1), dt, workspace.data_ptr(),
                                               workspace.numel() * workspace.element_size(), _stream()),
               "unigist_attn_bwd_varlen_strided")
        return dq, dk, dv
    _dev(q, k, v, out, lse, dout)
    if out.shape != q.shape or dout.shape != q.shape or lse.shape != (Hq, T) or lse.dtype != torch.float32:
        raise UnigistError("out/dout/lse shapes or dtypes disagree")
    if k.shape != (Hkv, T, D) or v.shape != k.shape or len({t.dtype for t in (q, k, v, out, dout)}) != 1:
        raise UnigistError("q/k/v/out/dout shapes or dtypes disagree")
    need = unigist_attn_bwd_varlen_workspace_ex(Hq, Hkv, T, D, int(r), int(W), int(sinks), int(window_mode), cu_seqlens, dt)
    if need == 0:
        raise UnigistError("unigist_attn_bwd_varlen_workspace: invalid shape or document bounds")
    if workspace is None:
        workspace = torch.empty(need, device=q.device, dtype=torch.uint8)
    # cu_seqlens covers 0 .. T (the library checks it), so every row belongs to a document and is written
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    _check(unigist_attn_bwd_varlen_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                      dout.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), Hq, Hkv, T, D,
                                      int(r), int(W), int(sinks), int(window_mode), cu_seqlens, dt, workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), _stream()),
           "unigist_attn_bwd_varlen_ex")
    return dq, dk, dv


def decode(q, kcache, vcache, seqlens=None, want_lse=True, workspace=None):
    """q [B,Hq,D], kcache/vcache [B,Hkv,Lk,D], seqlens int32 [B] on the GPU or None -> out [B,Hq,D], lse [B,Hq]."""
    _dev(q, kcache, vcache, seqlens)
    B, Hq, D = q.shape
    Hkv, Lk = kcache.shape[1], kcache.shape[2]
    dt = _dt(q)
    if kcache.shape != (B, Hkv, Lk, D) or vcache.shape != kcache.shape or kcache.dtype != q.dtype or vcache.dtype != q.dtype:
        raise UnigistError("q/kcache/vcache shapes or dtypes disagree")
    if seqlens is not None and (seqlens.dtype != torch.int32 or seqlens.shape != (B,)):
        raise UnigistError("seqlens must be int32 [B]")
    need = unigist_decode_workspace(B, Hq, Hkv, Lk, D, dt)
    if need == 0:
        raise UnigistError("unigist_decode_workspace: invalid or unsupported shape")
    if workspace is None:
        workspace = torch.empty(need, device=q.device, dtype=torch.uint8)
    out = torch.empty_like(q)
    lse = torch.empty(B, Hq, device=q.device, dtype=torch.float32) if want_lse else None
    _check(unigist_decode(q.data_ptr(), kcache.data_ptr(), vcache.data_ptr(), out.data_ptr(),
                          lse.data_ptr() if want_lse else None, B, Hq, Hkv, Lk,
                          seqlens.data_ptr() if seqlens is not None else None, D, dt,
                          workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream()),
           "unigist_decode")
    return out, lse


def _scales(t, H):
    _dev(t)
    if t.dtype != torch.float32 or t.shape != (H,):
        raise UnigistError("scales must be float32 [H] on the GPU")


def quantize_e4m3(x, scale):
    """x [B,H,n,D] bf16/fp32, scale float32 [H] on the GPU -> uint8 E4M3 codes of x / scale[h], same shape."""
    _dev(x)
    B, H, n, D = x.shape
    _scales(scale, H)
    y = torch.empty(x.shape, device=x.device, dtype=torch.uint8)
    _check(unigist_quantize_e4m3(x.data_ptr(), y.data_ptr(), scale.data_ptr(), B, H, n, D, _dt(x), _stream()),
           "unigist_quantize_e4m3")
    return y


def decode_e4m3(q, kcache, vcache, k_scale, v_scale, seqlens=None, want_lse=True, workspace=None):
    """decode() over a cache of E4M3 codes (uint8 [B,Hkv,Lk,D]) with per-kv-head scales; q and out bf16."""
    _dev(q, kcache, vcache, seqlens)
    B, Hq, D = q.shape
    Hkv, Lk = kcache.shape[1], kcache.shape[2]
    if q.dtype != torch.bfloat16 or kcache.dtype != torch.uint8 or vcache.dtype != torch.uint8:
        raise UnigistError("decode_e4m3 takes bf16 queries and uint8 caches")
    if kcache.shape != (B, Hkv, Lk, D) or vcache.shape != kcache.shape:
        raise UnigistError("q/kcache/vcache shapes disagree")
    if seqlens is not None and (seqlens.dtype != torch.int32 or seqlens.shape != (B,)):
        raise UnigistError("seqlens must be int32 [B]")
    _scales(k_scale, Hkv)
    _scales(v_scale, Hkv)
    need = unigist_decode_workspace(B, Hq, Hkv, Lk, D, UNIGIST_BF16)
    if need == 0:
        raise UnigistError("unigist_decode_workspace: invalid or unsupported shape")
    if workspace is None:
        workspace = torch.empty(need, device=q.device, dtype=torch.uint8)
    out = torch.empty_like(q)
    lse = torch.empty(B, Hq, device=q.device, dtype=torch.float32) if want_lse else None
    _check(unigist_decode_e4m3(q.data_ptr(), kcache.data_ptr(), vcache.data_ptr(), k_scale.data_ptr(), v_scale.data_ptr(),
                               out.data_ptr(), lse.data_ptr() if want_lse else None, B, Hq, Hkv, Lk,
                               seqlens.data_ptr() if seqlens is not None else None, D,
                               workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream()),
           "unigist_decode_e4m3")
    return out, lse


class KVCache:
    """Two ping-pong [B, Hkv, cap, D] buffers and the state (s, t) of the compressed cache; thin host-side
    bookkeeping around unigist_cache_update (no arithmetic).  With dtype=torch.uint8 the cache holds E4M3 codes:
    k_scale / v_scale (float32 [Hkv] on the GPU) are then required and update() quantises the rows it is given."""

    def __init__(self, B, Hkv, cap, D, r, dtype=torch.bfloat16, device="cuda", sinks=0, k_scale=None, v_scale=None):
        self.B, self.Hkv, self.cap, self.D, self.r, self.sinks = B, Hkv, cap, D, int(r), int(sinks)
        self.k_scale, self.v_scale = k_scale, v_scale
        if dtype == torch.uint8:
            _scales(k_scale, Hkv)
            _scales(v_scale, Hkv)
        self.k = [torch.empty(B, Hkv, cap, D, device=device, dtype=dtype) for _ in range(2)]
        self.v = [torch.empty(B, Hkv, cap, D, device=device, dtype=dtype) for _ in range(2)]
        self.cur, self.s, self.t = 0, 0, -1

    @property
    def rows(self) -> int:
        return unigist_cache_rows_ex(self.s, self.t, self.r, self.sinks)

    @property
    def kc(self):
        return self.k[self.cur]

    @property
    def vc(self):
        return self.v[self.cur]

    def update(self, k_new=None, v_new=None, s_new=None):
        """Append k_new/v_new ([B, Hkv, n, D], the next n positions; may be slices along the row axis of larger
        tensors) and move the window start to s_new."""
        n = 0 if k_new is None else k_new.shape[2]
        rows = n
        if n:
            if self.k[0].dtype == torch.uint8 and k_new.dtype != torch.uint8:
                k_new, v_new = k_new.contiguous(), v_new.contiguous()
                k_new, v_new = quantize_e4m3(k_new, self.k_scale), quantize_e4m3(v_new, self.v_scale)
            rows = _head_rows(k_new, 1)
            if _head_rows(v_new, 1) != rows or v_new.shape != k_new.shape:
                raise UnigistError("k_new and v_new must have the same shape and layout")
        s_new = self.s if s_new is None else int(s_new)
        nxt = 1 - self.cur
        _check(unigist_cache_update_ex(self.k[self.cur].data_ptr(), self.v[self.cur].data_ptr(), self.s, self.t,
                                       self.cap, k_new.data_ptr() if n else None, v_new.data_ptr() if n else None, n, rows,
                                       self.k[nxt].data_ptr(), self.v[nxt].data_ptr(), s_new, self.cap,
                                       self.B, self.Hkv, self.D, self.r, self.sinks,
                                       UNIGIST_E4M3 if self.k[0].dtype == torch.uint8 else _dt(self.k[0]), _stream()),
               "unigist_cache_update_ex")
        self.cur, self.s, self.t = nxt, s_new, self.t + n


class RaggedKVCache:
    """A batch of compressed caches whose sequences are in different states (s_b, t_b): one [B, Hkv, cap, D] buffer
    pair as unigist_decode wants it, maintained one sequence at a time with unigist_cache_update_ex on that
    sequence's slab (B = 1).  Host-side bookkeeping only; `seqlens()` is the int32 device vector decode takes."""

    def __init__(self, B, Hkv, cap, D, r, dtype=torch.bfloat16, device="cuda", sinks=0):
        self.B, self.Hkv, self.cap, self.D, self.r, self.sinks = B, Hkv, cap, D, int(r), int(sinks)
        self.k = [torch.empty(B, Hkv, cap, D, device=device, dtype=dtype) for _ in range(2)]
        self.v = [torch.empty(B, Hkv, cap, D, device=device, dtype=dtype) for _ in range(2)]
        self.cur = [0] * B           # which of the two buffers holds sequence b
        self.s, self.t = [0] * B, [-1] * B

    def rows(self, b) -> int:
        return unigist_cache_rows_ex(self.s[b], self.t[b], self.r, self.sinks)

    def update(self, b, k_new=None, v_new=None, s_new=None):
        """Sequence b: append k_new/v_new ([Hkv, n, D], its next n positions), move its window start to s_new."""
        n = 0 if k_new is None else k_new.shape[1]
        if n:
            _dev(k_new, v_new)
        s_new = self.s[b] if s_new is None else int(s_new)
        cur, nxt = self.cur[b], 1 - self.cur[b]
        _check(unigist_cache_update_ex(self.k[cur][b].data_ptr(), self.v[cur][b].data_ptr(), self.s[b], self.t[b], self.cap,
                                       k_new.data_ptr() if n else None, v_new.data_ptr() if n else None, n, n,
                                       self.k[nxt][b].data_ptr(), self.v[nxt][b].data_ptr(), s_new, self.cap,
                                       1, self.Hkv, self.D, self.r, self.sinks,
                                       UNIGIST_E4M3 if self.k[0].dtype == torch.uint8 else _dt(self.k[0]), _stream()),
               "unigist_cache_update_ex")
        self.cur[b], self.s[b], self.t[b] = nxt, s_new, self.t[b] + n

    def update_batch(self, k_new, v_new, n_new, s_new):
        """All sequences in one launch (unigist_cache_update_ragged): k_new/v_new [B, Hkv, new_rows, D] (sequence b
        uses its first n_new[b] rows), n_new and s_new sequences of B ints.  -> rows in use per sequence, int32 [B] on
        the GPU (-1 where a state was invalid).  Every sequence must currently sit in the same buffer."""
        if len(set(self.cur)) != 1:
            raise UnigistError("update_batch needs all sequences in the same buffer: call gathered() first")
        _dev(k_new, v_new)
        dev = self.k[0].device
        as_dev = lambda x: torch.tensor([int(v) for v in x], dtype=torch.int32).to(dev)
        so, to, nn, sn = as_dev(self.s), as_dev(self.t), as_dev(n_new), as_dev(s_new)
        rows = torch.empty(self.B, dtype=torch.int32, device=dev)
        cur, nxt = self.cur[0], 1 - self.cur[0]
        _check(unigist_cache_update_ragged(self.k[cur].data_ptr(), self.v[cur].data_ptr(), so.data_ptr(), to.data_ptr(),
                                           self.cap, k_new.data_ptr(), v_new.data_ptr(), nn.data_ptr(), k_new.shape[2],
                                           self.k[nxt].data_ptr(), self.v[nxt].data_ptr(), sn.data_ptr(), self.cap,
                                           rows.data_ptr(), self.B, self.Hkv, self.D, self.r, self.sinks,
                                           UNIGIST_E4M3 if self.k[0].dtype == torch.uint8 else _dt(self.k[0]), _stream()),
               "unigist_cache_update_ragged")
        self.cur = [nxt] * self.B
        self.s = [int(v) for v in s_new]
        self.t = [t + int(n) for t, n in zip(self.t, n_new)]
        return rows

    def prefill_batch(self, q, n, W, window_mode=UNIGIST_WINDOW_SLIDING, out=None, lse=None):
        """All sequences in one launch (unigist_prefill_chunk_ragged), after update_batch appended the chunk's keys:
        q [B, Hq, C, D], sequence b's queries are its first n[b] rows, at the last n[b] positions of its cache.
        -> out, lse (rows past n[b] untouched) and the rows in use per sequence, int32 [B] on the GPU (-1 where a
        state was invalid)."""
        kc, vc = self.current()
        _dev(q)
        B, Hq, C, D = q.shape
        dev = q.device
        as_dev = lambda x: torch.tensor([int(v) for v in x], dtype=torch.int32).to(dev)
        p0, nn, ss = as_dev([t + 1 - int(nb) for t, nb in zip(self.t, n)]), as_dev(n), as_dev(self.s)
        out = torch.empty_like(q) if out is None else out
        lse = torch.empty(B, Hq, C, device=dev, dtype=torch.float32) if lse is None else lse
        rows = torch.empty(B, dtype=torch.int32, device=dev)
        _check(unigist_prefill_chunk_ragged(q.data_ptr(), kc.data_ptr(), vc.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                            B, Hq, self.Hkv, C, D, self.r, int(W), self.sinks, int(window_mode),
                                            p0.data_ptr(), nn.data_ptr(), ss.data_ptr(), self.cap,
                                            rows.data_ptr(), _dt(q), _stream()),
               "unigist_prefill_chunk_ragged")
        return out, lse, rows

    def current(self):
        """-> kc, vc of the buffer all sequences sit in (after update_batch)."""
        if len(set(self.cur)) != 1:
            raise UnigistError("sequences sit in different buffers: call gathered()")
        return self.k[self.cur[0]], self.v[self.cur[0]]

    def gathered(self):
        """-> kc, vc [B, Hkv, cap, D] with every sequence's current slab in one buffer (sequences sitting in the
        other buffer are moved over with an empty update), and seqlens int32 [B] on the GPU."""
        for b in range(self.B):
            if self.cur[b] != 0:
                self.update(b)
        sl = torch.tensor([self.rows(b) for b in range(self.B)], dtype=torch.int32).to(self.k[0].device)
        return self.k[0], self.v[0], sl


class RingKVCache:
    """The cache of a batch in the ring layout for token-by-token decoding: appending a token writes a row or two
    per (sequence, kv head) instead of gathering the cache.  Built from a RaggedKVCache whose sequences have their
    window start at the first position of the window of their last position t; `t` (int32 [B] on the GPU) is each
    sequence's last position and `rows` the rows in use -- the seqlens of decode.  Bookkeeping only."""

    def __init__(self, ragged: "RaggedKVCache", W, window_mode=UNIGIST_WINDOW_SLIDING):
        kc, vc = ragged.current()
        self.B, self.Hkv, self.cap, self.D, self.r, self.sinks, self.W = (ragged.B, ragged.Hkv, ragged.cap, ragged.D,
                                                                         ragged.r, ragged.sinks, int(W))
        self.mode = int(window_mode)
        dev = kc.device
        self.dt = UNIGIST_E4M3 if kc.dtype == torch.uint8 else _dt(kc)
        self.kc, self.vc = torch.empty_like(kc), torch.empty_like(vc)
        self.t = torch.tensor(ragged.t, dtype=torch.int32).to(dev)
        s = torch.tensor(ragged.s, dtype=torch.int32).to(dev)
        self.rows = torch.empty(self.B, dtype=torch.int32, device=dev)
        _check(unigist_cache_to_ring(kc.data_ptr(), vc.data_ptr(), s.data_ptr(), self.t.data_ptr(), self.cap,
                                     self.kc.data_ptr(), self.vc.data_ptr(), self.cap, self.rows.data_ptr(), self.B,
                                     self.Hkv, self.D, self.r, self.W, self.sinks, self.mode, self.dt, _stream()),
               "unigist_cache_to_ring")

    def append(self, k_new, v_new, active=None):
        """k_new/v_new [B, Hkv, 1, D]: the next position of every sequence (of those with active[b] = 1, int32 [B] on
        the GPU).  -> rows in use per sequence (int32 [B] on the GPU, -1 for a sequence that does not fit)."""
        _dev(k_new, v_new, active)
        if active is None:
            active = torch.ones(self.B, dtype=torch.int32, device=self.kc.device)
        _check(unigist_cache_ring_append(self.kc.data_ptr(), self.vc.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                         k_new.shape[2], self.t.data_ptr(), active.data_ptr(), self.cap,
                                         self.rows.data_ptr(), self.B, self.Hkv, self.D, self.r, self.W, self.sinks,
                                         self.mode, self.dt, _stream()),
               "unigist_cache_ring_append")
        # in place, stream-ordered behind the kernel's read of t (the call can be captured in a graph); a sequence
        # that did not fit (rows = -1) was left alone and does not advance
        self.t.add_(active * (self.rows >= 0))
        return self.rows

    def to_ragged(self, ragged: "RaggedKVCache"):
        """Back to the layout prefill wants, into `ragged`'s buffers: every sequence in state (first position of the
        window of t, t)."""
        t = self.t.cpu().tolist()  # RaggedKVCache keeps its states on the host: a change of phase, not a per-token step
        s = [unigist_window_start(x, self.r, self.W, self.sinks, self.mode) for x in t]
        dev = self.kc.device
        sd = torch.tensor(s, dtype=torch.int32).to(dev)
        rows = torch.empty(self.B, dtype=torch.int32, device=dev)
        _check(unigist_cache_from_ring(self.kc.data_ptr(), self.vc.data_ptr(), sd.data_ptr(), self.t.data_ptr(), self.cap,
                                       ragged.k[0].data_ptr(), ragged.v[0].data_ptr(), ragged.cap, rows.data_ptr(),
                                       self.B, self.Hkv, self.D, self.r, self.W, self.sinks, self.mode, self.dt, _stream()),
               "unigist_cache_from_ring")
        ragged.cur, ragged.s, ragged.t = [0] * self.B, s, t
        return rows


def prefill_chunk(q, cache: "KVCache", r, W, p0, window_mode=UNIGIST_WINDOW_SLIDING, workspace=None, out=None, lse=None):
    """q [B, Hq, C, D]: queries at positions p0 .. p0+C-1; cache already holds their keys.  -> out, lse.
    A cache of E4M3 codes goes through unigist_prefill_chunk_e4m3 (workspace: a uint8 tensor to reuse, optional).
    q may be a slice along the row axis of a [B, Hq, L, D] tensor if out and lse are given as the same slice of
    tensors [B, Hq, L, D] and [B, Hq, L] (unigist_prefill_chunk_view: no copies of the chunk).  Without out/lse, a q
    of any strides with a contiguous last axis (e.g. the transposed view of a [B, C, Hq, D] projection output) gets
    an out of the same strides (unigist_prefill_chunk_strided)."""
    B, Hq, C, D = q.shape
    if out is None and lse is None and not q.is_contiguous() and cache.kc.dtype != torch.uint8:
        if not q.is_cuda:
            raise UnigistError("libunigist takes device tensors only (no CPU path)")
        st = q.stride()
        if st[3] != 1:
            raise UnigistError("the last axis of q must be contiguous")
        out = torch.empty_strided(q.shape, st, dtype=q.dtype, device=q.device)
        lse = torch.empty(B, Hq, C, device=q.device, dtype=torch.float32)
        _check(unigist_prefill_chunk_strided(q.data_ptr(), cache.kc.data_ptr(), cache.vc.data_ptr(), out.data_ptr(),
                                             lse.data_ptr(), B, Hq, cache.Hkv, C, D, int(r), int(W), cache.sinks,
                                             int(window_mode), int(p0), cache.s, cache.cap, st[0], st[1], st[2], _dt(q),
                                             _stream()),
               "unigist_prefill_chunk_strided")
        return out, lse
    if out is not None or lse is not None or not q.is_contiguous():
        if out is None or lse is None or cache.kc.dtype == torch.uint8:
            raise UnigistError("a sliced q needs out= and lse= slices of the same layout (bf16 caches only)")
        rows = _head_rows(q, 1)
        lrows = lse.stride(1) if lse.dim() == 3 and lse.stride(2) == 1 and lse.is_cuda else -1
        if _head_rows(out, 1) != rows or lrows != rows or out.shape != q.shape or lse.shape != (B, Hq, C) or \
                (B > 1 and lse.stride(0) != Hq * rows) or out.dtype != q.dtype or lse.dtype != torch.float32:
            raise UnigistError("q, out and lse must be the same row slice of tensors with equal rows per head")
        _check(unigist_prefill_chunk_view(q.data_ptr(), cache.kc.data_ptr(), cache.vc.data_ptr(), out.data_ptr(),
                                          lse.data_ptr(), B, Hq, cache.Hkv, C, rows, D, int(r), int(W), cache.sinks,
                                          int(window_mode), int(p0), cache.s, cache.cap, _dt(q), _stream()),
               "unigist_prefill_chunk_view")
        return out, lse
    _dev(q)
    out = torch.empty_like(q)
    lse = torch.empty(B, Hq, C, device=q.device, dtype=torch.float32)
    if cache.kc.dtype == torch.uint8:
        need = unigist_prefill_chunk_e4m3_workspace(B, cache.Hkv, D, cache.s, int(p0) + C - 1, int(r), cache.sinks)
        if workspace is None or workspace.numel() < need:
            workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
        _check(unigist_prefill_chunk_e4m3(q.data_ptr(), cache.kc.data_ptr(), cache.vc.data_ptr(),
                                          cache.k_scale.data_ptr(), cache.v_scale.data_ptr(), out.data_ptr(),
                                          lse.data_ptr(), B, Hq, cache.Hkv, C, D, int(r), int(W), cache.sinks,
                                          int(window_mode), int(p0), cache.s, cache.cap, workspace.data_ptr(),
                                          workspace.numel(), _stream()),
               "unigist_prefill_chunk_e4m3")
        return out, lse
    _check(unigist_prefill_chunk_ex(q.data_ptr(), cache.kc.data_ptr(), cache.vc.data_ptr(), out.data_ptr(),
                                    lse.data_ptr(), B, Hq, cache.Hkv, C, D, int(r), int(W), cache.sinks,
                                    int(window_mode), int(p0), cache.s, cache.cap, _dt(q), _stream()),
           "unigist_prefill_chunk_ex")
    return out, lse
