"""Oracle: the 8-bit floating-point (E4M3) convolution variant (test infrastructure).

Not from the paper, which runs its models inside an inference engine and says nothing about number formats
(Sec. III-A, step 4): this is the reduced-precision variant of the model-execution kernel.  What it computes is fixed
here by two public definitions:

  * the E4M3 format of the OCP 8-bit floating point specification: 1 sign bit, 4 exponent bits with bias 7, 3 mantissa
    bits; exponent field 0 holds the subnormals q * 2^-9; there are no infinities; S.1111.111 is NaN, so the largest
    finite value is S.1111.110 = 1.75 * 2^8 = 448;
  * conversion to it: round to nearest, ties to even, saturating (|x| > 448 gives +-448), NaN gives NaN (0x7F here);
  * the convolution itself is `nn.direct_conv` / `nn.conv2d` on the decoded values in fp64:
        y_real = act(scale[k] * sum x_val * w_val + bias[k] (+ res_val * res_scale)),
    and, where the output is stored in E4M3, code = encode(fp32(y_real * y_inv_scale)).

The encoder works on fp64 numbers that are exactly the fp32 inputs (scaling by powers of two is exact), so it is an
exact statement of the rounding rule, not an approximation of it.
"""
from __future__ import annotations

import numpy as np

from . import nn

E4M3_MAX = 448.0


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """uint8 codes -> fp64 values (NaN for 0x7F / 0xFF)."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    ex = (c >> 3) & 15
    q = (c & 7).astype(np.float64)
    mag = np.where(ex == 0, q * 2.0 ** -9, (1.0 + q / 8.0) * np.exp2((ex - 7).astype(np.float64)))
    out = sign * mag
    return np.where((ex == 15) & ((c & 7) == 7), np.nan, out)


def _rne(x: np.ndarray) -> np.ndarray:
    """nearest integer, ties to even, for non-negative x"""
    f = np.floor(x)
    d = x - f
    up = (d > 0.5) | ((d == 0.5) & (np.mod(f, 2.0) == 1.0))
    return f + up


def e4m3_encode(x) -> np.ndarray:
    """fp32 values -> uint8 codes: nearest representable value, ties to the even mantissa, saturating at +-448."""
    x32 = np.asarray(x, dtype=np.float32)
    a = np.minimum(np.abs(x32.astype(np.float64)), E4M3_MAX)
    nan = np.isnan(x32)
    a = np.where(nan, 0.0, a)
    # the spacing of representable values around a: 2^-9 below the first normal 2^-6, else 2^(floor(log2 a) - 3)
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    # log2 of a float just below a power of two can round up to that power; fix the exponent so that 2^e <= a
    e = np.where(np.exp2(e) > a, e - 1, e)
    e = np.maximum(e, -6.0)
    step = np.exp2(e - 3.0)
    n = _rne(a / step)                       # a in units of the spacing: 0..8 for subnormals, 8..16 for normals
    val = n * step                           # the rounded magnitude (16 * step = the next binade's first value)
    # value -> code
    ev = np.floor(np.log2(np.where(val > 0, val, 1.0)))
    ev = np.where(np.exp2(ev) > val, ev - 1, ev)
    sub = val < 2.0 ** -6
    field = np.where(sub, 0, ev + 7).astype(np.int64)
    mant = np.where(sub, val * 2.0 ** 9, (val / np.exp2(ev) - 1.0) * 8.0).astype(np.int64)
    code = (field << 3) | mant
    code = np.where(np.signbit(x32), code | 0x80, code)
    return np.where(nan, 0x7F, code).astype(np.uint8)


def conv_e4m3(x_codes: np.ndarray, w_codes: np.ndarray, scale: np.ndarray, bias: np.ndarray, stride: int, pad: int, act: int,
              res_codes: np.ndarray = None, res_scale: float = 0.0, res_mode: int = nn.RES_NONE) -> np.ndarray:
    """fp64 result before it is stored.  x_codes [N][H][W][C], w_codes [K][R][S][C], scale / bias [K]."""
    acc = nn.conv2d(e4m3_decode(x_codes), e4m3_decode(w_codes), stride, pad)
    y = acc * np.asarray(scale, np.float64) + np.asarray(bias, np.float64)
    if res_mode == nn.RES_BEFORE_ACT:
        return nn.activation(y + e4m3_decode(res_codes) * float(res_scale), act)
    if res_mode == nn.RES_AFTER_ACT:
        return nn.activation(y, act) + e4m3_decode(res_codes) * float(res_scale)
    return nn.activation(y, act)


def store_e4m3(y_real: np.ndarray, y_inv_scale: float) -> np.ndarray:
    """What the path stores: the fp32 product y * y_inv_scale, encoded."""
    return e4m3_encode(np.asarray(y_real, np.float64).astype(np.float32) * np.float32(y_inv_scale))
