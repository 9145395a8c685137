"""FP8 (OCP E4M3) quantisation and the FP8 projection product, numpy (test infrastructure only).

An extension beyond the paper (it states no numeric precision; Sec. "Evaluation" names only the software
stack): the forward-only frozen components (Sec. 2.1) run their projections on 8-bit operands.  The format is
the published OCP 8-bit floating point E4M3: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits; exponent
field 0 holds the subnormals m / 8 * 2^-6; the largest finite value is 448 (exponent field 15 with mantissa
111 is NaN, there are no infinities).  Conversion is to the nearest representable value, ties to the one with
an even mantissa, after clamping to +-448.

Where floating point decides an integer (the 8-bit code), the decision is taken in the precision the
kernel uses: x (bf16, exact in fp32) times 1 / scale (fp32) rounded to fp32, then converted.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """uint8 codes -> float64 values, straight from the format's definition (NaN codes are not produced here)."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e, m = (c >> 3) & 0xF, c & 0x7
    return sign * np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7.0))


def e4m3_round(v: np.ndarray):
    """Nearest E4M3 value (ties to even mantissa) of float values already inside [-448, 448]: returns (values, codes)."""
    v = np.asarray(v, dtype=np.float64)
    a = np.abs(v)
    # spacing of the representable values around a: 2^-9 below 2^-6 (subnormals), else 2^(floor(log2 a) - 3)
    ex = np.floor(np.log2(np.maximum(a, 2.0 ** -6)))
    step = 2.0 ** (ex - 3.0)
    k = np.rint(a / step)                      # numpy rounds halves to even: with step a power of two this is ties-to-even mantissa
    q = k * step                               # may have carried into the next binade: still representable (448 is the cap)
    q = np.minimum(q, E4M3_MAX)
    qe = np.floor(np.log2(np.maximum(q, 2.0 ** -6)))
    sub = q < 2.0 ** -6
    mant = np.where(sub, np.rint(q / 2.0 ** -9), np.rint((q / 2.0 ** qe - 1.0) * 8.0)).astype(np.int64)
    expf = np.where(sub, 0, (qe + 7).astype(np.int64))
    codes = ((np.signbit(v).astype(np.int64) << 7) | (expf << 3) | mant).astype(np.uint8)
    return np.copysign(q, v), codes


def quantize(x: np.ndarray, scale: float):
    """x: values representable in bf16.  Returns (values, codes) of e4m3(clamp(fp32(x) * fp32(1 / scale), +-448))."""
    inv = np.float32(1.0) / np.float32(scale)
    prod = (np.asarray(x, dtype=np.float32) * inv).astype(np.float32)          # one fp32 rounding, as in the kernel
    return e4m3_round(np.clip(prod.astype(np.float64), -E4M3_MAX, E4M3_MAX))


def gemm(a_vals: np.ndarray, b_vals: np.ndarray, out_scale: float, bias=None) -> np.ndarray:
    """C = out_scale * A B^T (+ bias) on the decoded operand values, in float64."""
    c = float(np.float32(out_scale)) * (a_vals @ b_vals.T)
    return c if bias is None else c + bias
