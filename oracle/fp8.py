"""Oracle of the 8-bit storage format of the fp8 KV slots (test infrastructure only).

The format is the OCP 8-bit floating point "E4M3" (1 sign, 4 exponent bits with bias 7, 3 mantissa
bits; no infinities; the all-ones exponent with all-ones mantissa is NaN; largest finite value
448; subnormals m * 2^-9).  Storing a key or value rounds it to the nearest representable number,
ties to the even mantissa, values beyond +-448 saturate to +-448, NaN stays NaN.  Written from
the format's definition with exact arithmetic on float64 (every bf16 / fp32 input is exact in
float64), no table shared with the GPU side.
"""
import numpy as np

E4M3_MAX = 448.0


def decode_e4m3(codes):
    """uint8 codes -> float64 values."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = c & 0x7
    val = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * 2.0 ** (e - 7.0))
    val = np.where((e == 15) & (m == 7), np.nan, val)
    return sign * val


def encode_e4m3(x):
    """float values -> uint8 codes: round to nearest, ties to even, saturating at +-448."""
    x = np.asarray(x, dtype=np.float64)
    out = np.zeros(x.shape, np.uint8)
    sign = np.signbit(x)
    a = np.minimum(np.abs(np.where(np.isnan(x), 0.0, x)), E4M3_MAX)      # NaN handled at the end
    # spacing of the format around a: 2^-9 below 2^-6 (subnormals and the first binade), else 2^(floor(log2 a) - 3)
    with np.errstate(divide="ignore", invalid="ignore"):
        ex = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    ex = np.maximum(ex, -6.0)
    step = 2.0 ** (ex - 3.0)
    q = np.rint(a / step)                      # numpy rounds halves to even; a / step is exact (power of two)
    r = q * step                               # the rounded magnitude, may have carried into the next binade
    with np.errstate(divide="ignore", invalid="ignore"):
        ex2 = np.floor(np.log2(np.where(r > 0, r, 1.0)))
    normal = r >= 2.0 ** -6
    e_field = np.where(normal, ex2 + 7.0, 0.0)
    m_field = np.where(normal, r / 2.0 ** ex2 * 8.0 - 8.0, r * 2.0 ** 9)
    code = (e_field.astype(np.int64) << 3) | m_field.astype(np.int64)
    code = np.where(np.isnan(x), 0x7F, code)
    out = (code | np.where(sign, 0x80, 0)).astype(np.uint8)
    return out


def round_e4m3(x):
    """The value a key/value element has after it was stored: float64."""
    return decode_e4m3(encode_e4m3(x))
