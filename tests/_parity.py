"""Helpers for the GPU parity tests: run the oracle on the same seeded tensors and
measure the errors the tolerances are stated in."""
import numpy as np
import torch

import oracle

# Tolerances:
#   bf16 inputs, fp32 accumulation: max-abs error on out <= 1e-2, relative L2 error on
#   dq/dk/dv <= 2e-2; fp32 debug build: <= 1e-5 for all of them.
#   lse is fp32 on both builds: 1e-4 on the bf16 build (measured <= 4e-6; a key dropped or added among several
#   thousand moves it by about 1e-4).
TOL_OUT_BF16 = 1e-2
TOL_LSE_BF16 = 1e-4
TOL_GRAD_BF16 = 2e-2
TOL_F32 = 1e-5


def out_bound(want) -> np.ndarray:
    """The one bound used for bf16 `out` wherever an output can leave the range of an average of many values
    (full-size samples, rows or caches of a few keys): 1e-2 as stated where |out| < 2; from |out| >= 2 on the
    rounding of the *stored* bf16 result alone -- half an ulp, 2^(e-8) for |out| in [2^e, 2^(e+1)), i.e. 7.8e-3 in
    [2, 4) -- is allowed on top, since it is not an error of the arithmetic being checked."""
    w = np.abs(np.asarray(want, dtype=np.float64))
    half_ulp = np.where(w >= 2.0, 2.0 ** (np.floor(np.log2(np.maximum(w, 1e-30))) - 8), 0.0)
    return TOL_OUT_BF16 + half_ulp


def out_ok(got, want) -> bool:
    return bool((np.abs(np.asarray(got, dtype=np.float64) - np.asarray(want, dtype=np.float64)) <= out_bound(want)).all())


def to_np(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a (bf16 or fp32) tensor to float64 on the host."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def max_abs(a, b) -> float:
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)))) if np.size(a) else 0.0


def rel_l2(a, b) -> float:
    """||a - b|| / ||b|| with b the oracle."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = float(np.linalg.norm(b))
    num = float(np.linalg.norm(a - b))
    return num / den if den > 0 else num


def oracle_fwd_bwd(q, k, v, dout, r, W, **mask):
    qn, kn, vn, don = (to_np(t) for t in (q, k, v, dout))
    out, lse = oracle.attn_fwd(qn, kn, vn, r, W, **mask)
    dq, dk, dv = oracle.attn_bwd(qn, kn, vn, don, r, W, **mask)
    return out, lse, dq, dk, dv
