"""8-bit floating point storage of the compressed cache (E4M3), CPU reference.

THIS IS TEST INFRASTRUCTURE, like the rest of this package: it shares no code with the HIP
kernels and must never be imported by the product package.

The paper does not quantise the cache; this is an extension of its decode step (Sec. 4.3) whose
arithmetic is fixed here, by the published format and by three choices:

* Format: E4M3 of the OCP 8-bit floating point specification -- 1 sign, 4 exponent (bias 7) and
  3 mantissa bits, subnormals at exponent field 0, no infinities, S.1111.111 is NaN, so the largest
  finite magnitude is S.1111.110 = 1.75 * 2^8 = 448.
* Quantisation of a cache element x with the scale c of its kv head: y = x / c in IEEE binary32
  (x widened exactly, one correctly rounded division), y clamped to [-448, 448], then rounded to
  the nearest representable value, ties to the even mantissa.  The rounding decision is thus taken
  on a binary32 number on both sides.
* Decode on a quantised cache is the plain decode on the dequantised values code * c, in fp64.
"""
import numpy as np

E4M3_MAX = 448.0


def e4m3_decode(codes):
    """uint8 codes -> float64 values (exact)."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = c & 0x7
    mag = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    mag = np.where((e == 15) & (m == 7), np.nan, mag)
    return sign * mag


def e4m3_encode(y):
    """binary32 values -> uint8 codes: clamp to +-448, round to nearest, ties to even."""
    y = np.asarray(y, dtype=np.float32)
    a = np.minimum(np.abs(y.astype(np.float64)), E4M3_MAX)      # exact: binary32 fits in binary64
    nan = np.isnan(a)
    a = np.where(nan, 0.0, a)
    # spacing of the representable values around a: 2^-9 below 2^-6, else 2^(floor(log2 a) - 3)
    _, ex = np.frexp(a)                                          # a = f * 2^ex, f in [0.5, 1)
    binade = np.maximum(ex - 1, -6)
    q = np.exp2((binade - 3).astype(np.float64))
    n = np.rint(a / q)                                           # a / q is exact; rint rounds halves to even
    v = n * q                                                    # the rounded magnitude (may reach the next binade)
    _, ex2 = np.frexp(v)
    normal = v >= 2.0 ** -6
    efield = np.where(normal, ex2 - 1 + 7, 0)
    mant = np.where(normal, np.rint((v / np.exp2((ex2 - 1).astype(np.float64)) - 1.0) * 8.0), np.rint(v * 2.0 ** 9))
    code = (efield.astype(np.int64) << 3) | mant.astype(np.int64)
    code = np.where(nan, 0x7F, code)
    code = code | np.where(np.signbit(y), 0x80, 0)
    return code.astype(np.uint8)


def quantize_e4m3(x, scale):
    """x [..., H, n, D] (any float dtype whose values fit binary32 exactly), scale [H] -> uint8 codes."""
    x32 = np.asarray(x).astype(np.float32)
    s32 = np.asarray(scale, dtype=np.float32).reshape((-1, 1, 1))
    with np.errstate(over="ignore"):
        y = (x32 / s32).astype(np.float32)
    return e4m3_encode(y)


def dequantize_e4m3(codes, scale):
    """uint8 codes [..., H, n, D], scale [H] -> float64 values code * scale."""
    s = np.asarray(scale, dtype=np.float32).astype(np.float64).reshape((-1, 1, 1))
    return e4m3_decode(codes) * s


def decode_e4m3(q, kcodes, vcodes, k_scale, v_scale, seqlens=None):
    """Decode (Sec. 4.3) over a cache stored as E4M3 codes with one scale per kv head:
    q [B,Hq,D]; kcodes, vcodes uint8 [B,Hkv,Lk,D]; k_scale, v_scale [Hkv] -> out [B,Hq,D], lse [B,Hq]."""
    from .unigist_oracle import decode
    return decode(q, dequantize_e4m3(kcodes, k_scale), dequantize_e4m3(vcodes, v_scale), seqlens)
