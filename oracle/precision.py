"""Storage formats of the offloaded projection and what they cost in accuracy (a CPU-side study).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (see gelo_oracle.py).  The paper's Conclusion asks to
"characterize numerical stability under common inference precisions and quantization
(BF16/FP16/FP8/INT8)"; Table 1 reports only that the method is exact up to floating point.  The
rounding functions below are written from the formats' public definitions (IEEE 754 binary16,
bfloat16 = the upper half of binary32, OCP 8-bit floating point E4M3 / E5M2, symmetric INT8 with
an absolute-maximum scale) in float64 numpy and pinned in tests/test_precision_study.py by
enumerating every code of the 8-bit formats, hand-computed ties, and library casts as checkers.
`chain_error` runs the oracle's chain with the accelerator's operands U and W (and optionally its
result Y) stored in a format, everything else exact: the error of Z it returns is the format's alone.
"""
from __future__ import annotations

import numpy as np

from oracle import gelo_oracle as o


def round_to_float_format(x, exponent_bits, mantissa_bits, max_finite):
    """Round-to-nearest-even onto a binary floating-point grid with `mantissa_bits` stored fraction
    bits, bias 2^(exponent_bits-1) - 1, gradual underflow, and saturation at +-max_finite (the 8-bit
    formats of the OCP specification have no use for infinities in a GEMM operand)."""
    x = np.asarray(x, dtype=np.float64)
    bias = (1 << (exponent_bits - 1)) - 1
    e_min = 1 - bias                                      # exponent of the smallest normal number
    mag = np.abs(x)
    e = np.floor(np.log2(np.where(mag > 0, mag, 1.0)))
    e = np.maximum(e, e_min)                              # subnormals share the spacing of the smallest binade
    step = np.exp2(e - mantissa_bits)
    q = np.round(mag / step) * step                       # numpy rounds halves to even
    q = np.minimum(q, max_finite)
    return np.sign(x) * q


def round_to_e4m3(x):
    """OCP FP8 E4M3: 4 exponent bits (bias 7), 3 fraction bits, largest finite value 448, no infinity."""
    return round_to_float_format(x, 4, 3, 448.0)


def round_to_e5m2(x):
    """OCP FP8 E5M2: 5 exponent bits (bias 15), 2 fraction bits, largest finite value 57344."""
    return round_to_float_format(x, 5, 2, 57344.0)


def round_to_bf16(x):
    return round_to_float_format(x, 8, 7, 3.3895313892515355e38)


def round_to_fp16(x):
    return round_to_float_format(x, 5, 10, 65504.0)


def quantize_scaled(x, rounder, max_finite, axis=None):
    """x -> scale * rounder(x / scale) with scale = absmax / max_finite over `axis` (None: the whole
    tensor): the usual way an 8-bit float operand is brought into range."""
    x = np.asarray(x, dtype=np.float64)
    amax = np.max(np.abs(x), axis=axis, keepdims=axis is not None)
    scale = np.where(amax > 0, amax / max_finite, 1.0)
    return rounder(x / scale) * scale


def quantize_int8(x, axis=None):
    """Symmetric INT8: x -> scale * clip(round(x / scale), -127, 127), scale = absmax / 127 over `axis`."""
    x = np.asarray(x, dtype=np.float64)
    amax = np.max(np.abs(x), axis=axis, keepdims=axis is not None)
    scale = np.where(amax > 0, amax / 127.0, 1.0)
    return np.clip(np.round(x / scale), -127, 127) * scale


FORMATS = {
    "bf16": (lambda u: round_to_bf16(u), lambda w: round_to_bf16(w)),
    "fp16": (lambda u: round_to_fp16(u), lambda w: round_to_fp16(w)),
    # 8-bit floats: one scale per row of U (per token) and per column of W (per output channel)
    "e4m3": (lambda u: quantize_scaled(u, round_to_e4m3, 448.0, axis=1), lambda w: quantize_scaled(w, round_to_e4m3, 448.0, axis=0)),
    "e5m2": (lambda u: quantize_scaled(u, round_to_e5m2, 57344.0, axis=1), lambda w: quantize_scaled(w, round_to_e5m2, 57344.0, axis=0)),
    "int8": (lambda u: quantize_int8(u, axis=1), lambda w: quantize_int8(w, axis=0)),
}


def chain_error(fmt, H, W, A, S=None, round_y_to_bf16=False):
    """Relative Frobenius error of Z = A^-1 (q(U) q(W)) against H W when the accelerator stores U and W
    in `fmt` (a key of FORMATS) and accumulates exactly; mixing and unmixing are exact (A orthogonal:
    A^-1 = A^T)."""
    qu, qw = FORMATS[fmt]
    n_data = H.shape[0]
    U = o.mix(A, H, S)
    Y = qu(U) @ qw(np.asarray(W, dtype=np.float64))
    if round_y_to_bf16:
        Y = round_to_bf16(Y)
    Z = o.unmix(A.T, Y, n_data)
    return o.rel_frobenius(Z, o.plain_projection(H, W))
