"""FP8 E4M3 reference for the fp8 variant of the block-prefill step.  TEST INFRASTRUCTURE ONLY.

The paper computes attention in 16-bit floating point; the fp8 variant is this build's extension of
its block-prefill step (Sec. "Formulations", Eq. 3-4) and is defined here, in plain numpy:

  * the 8-bit format is OCP "E4M3" (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no
    infinities, the all-ones exponent-and-mantissa pattern is NaN, largest finite value 448,
    subnormals m * 2^-9);
  * a tensor is stored as codes x a power-of-two scale 2^e, where e is the smallest integer with
    amax * 2^-e <= 448 (amax = largest magnitude the scale covers; e = 0 for amax = 0; e is kept
    within [-100, 100]).  Multiplying by a power of two is exact, so the code of a value does not
    depend on the precision the scaling is carried out in;
  * codes are rounded to nearest, ties to the even mantissa, magnitudes above 448 saturate;
  * Q has one scale per (token, query head), K and V one scale per KV head over all tokens;
  * what is quantised of Q is q * f, f = softmax factor * log2(e) as a float32 number and the product
    rounded once to float32 (the scores of the quantised operands are then base-2 exponents);
  * the attention itself is Eq. 3-4 evaluated exactly (fp64) on the de-quantised tensors (Q divided
    by f again).

Nothing here is shared with the HIP path.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0
EXP_LIMIT = 100


def decode_table() -> np.ndarray:
    """Value of each of the 256 codes (float64; NaN for 0x7f and 0xff), from the bit fields."""
    out = np.empty(256, np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e, m = (code >> 3) & 0xF, code & 0x7
        if e == 0xF and m == 0x7:
            out[code] = np.nan
        elif e == 0:
            out[code] = sign * m * 2.0 ** -9          # subnormal: 0.m * 2^(1 - bias)
        else:
            out[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return out


_TABLE = decode_table()
_POS = _TABLE[:127]  # codes 0 .. 126: the non-negative finite values, increasing


def decode(codes: np.ndarray) -> np.ndarray:
    return _TABLE[np.asarray(codes, np.uint8)]


def encode(x: np.ndarray) -> np.ndarray:
    """Nearest code (ties to the even mantissa = even code), saturating at +-448.  x finite."""
    x = np.asarray(x, np.float64)
    a = np.minimum(np.abs(x), E4M3_MAX)
    hi = np.searchsorted(_POS, a, side="left")          # first value >= a
    hi = np.minimum(hi, 126)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - _POS[lo], _POS[hi] - a
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return np.where(np.signbit(x), code | 0x80, code).astype(np.uint8)


def scale_exponent(amax: np.ndarray) -> np.ndarray:
    """Smallest integer e with amax * 2^-e <= 448, 0 for amax == 0, clipped to [-100, 100]."""
    amax = np.asarray(amax, np.float64)
    with np.errstate(divide="ignore"):
        e = np.ceil(np.log2(amax / E4M3_MAX))
    e = np.where(amax > 0, e, 0.0).astype(np.int64)
    # log2 in floating point may be off by one at exact powers of two: settle it with exact arithmetic
    e = np.where((amax > 0) & (np.ldexp(amax, -(e - 1)) <= E4M3_MAX), e - 1, e)
    e = np.where((amax > 0) & (np.ldexp(amax, -e) > E4M3_MAX), e + 1, e)
    return np.clip(e, -EXP_LIMIT, EXP_LIMIT).astype(np.int32)


def quantise(x: np.ndarray, axes) -> tuple[np.ndarray, np.ndarray]:
    """Codes of x and the exponents of the scales, one scale per slice along `axes` (those axes are
    reduced: the exponent array keeps them with length 1)."""
    x = np.asarray(x, np.float64)
    amax = np.max(np.abs(x), axis=axes, keepdims=True) if x.size else np.zeros([1] * x.ndim)
    e = scale_exponent(amax)
    return encode(np.ldexp(x, -e)), e


def dequantise(codes: np.ndarray, e: np.ndarray) -> np.ndarray:
    return np.ldexp(decode(codes), e)


def q_factor(softmax_scale: float, head_dim: int) -> np.float32:
    """f = softmax factor * log2(e) in float32 (softmax_scale <= 0: the default 1/sqrt(head_dim))."""
    scale = np.float32(softmax_scale) if softmax_scale > 0 else np.float32(1.0 / np.sqrt(np.float64(head_dim)))
    return np.float32(scale * np.float32(1.4426950408889634))


def quantise_qkv(q: np.ndarray, k: np.ndarray, v: np.ndarray, factor: np.float32):
    """q [T, Hq, D], k and v [T, Hkv, D] (values exactly representable in float32) -> dict of codes and
    scale exponents as the fp8 variant stores them: Q * factor per (token, head), K and V per head."""
    q = (np.asarray(q, np.float32) * np.float32(factor)).astype(np.float64)  # one float32 rounding per element
    qc, qe = quantise(q, axes=(2,))
    kc, ke = quantise(k, axes=(0, 2))
    vc, ve = quantise(v, axes=(0, 2))
    return dict(q_codes=qc, q_exp=qe[:, :, 0], k_codes=kc, k_exp=ke[0, :, 0], v_codes=vc, v_exp=ve[0, :, 0])


def dequantised_qkv(q: np.ndarray, k: np.ndarray, v: np.ndarray, factor: np.float32):
    """The tensors the fp8 variant attends over, as float64 (Q with the factor taken out again, so that
    the plain attention with the same softmax factor applies)."""
    z = quantise_qkv(q, k, v, factor)
    return (np.ldexp(decode(z["q_codes"]), z["q_exp"][:, :, None]) / np.float64(factor),
            np.ldexp(decode(z["k_codes"]), z["k_exp"][None, :, None]),
            np.ldexp(decode(z["v_codes"]), z["v_exp"][None, :, None]))
