"""Software rounding to the 8-bit floating-point format E4M3 (test infrastructure only).

The format (OCP 8-bit floating point, "E4M3": 1 sign bit, 4 exponent bits with bias 7, 3 mantissa
bits, subnormals, no infinities, the single code S.1111.111 is NaN): a normal number is
(-1)^s 2^(e-7) (1 + m/8) for e = 1..15 (without e = 15, m = 7), a subnormal one (-1)^s 2^-6 (m/8);
the largest magnitude is 448, the smallest positive one 2^-9.

round_to_e4m3(x) returns, as binary32 values, the E4M3 numbers nearest to x, ties to the even
mantissa code, magnitudes beyond 448 clamped to 448 (the emulation's choice: nothing in this
repository feeds it such values).  decode_all() lists the value of every code straight from the
bit fields; the tests use it to check the rounding function exhaustively.
"""
import numpy as np

E4M3_MAX = 448.0


def decode(code):
    """Value of one 8-bit code (NaN for 0x7F / 0xFF)."""
    code = int(code)
    s = -1.0 if code & 0x80 else 1.0
    e = (code >> 3) & 0xF
    m = code & 0x7
    if e == 15 and m == 7:
        return float("nan")
    if e == 0:
        return s * (m / 8.0) * 2.0 ** -6
    return s * (1.0 + m / 8.0) * 2.0 ** (e - 7)


def decode_all():
    return np.array([decode(c) for c in range(256)], dtype=np.float64)


def round_to_e4m3(x):
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    # spacing of the format around |x|: 2^-9 below 2^-6 (subnormals), else 2^(floor(log2|x|) - 3)
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.maximum(e, -6.0)
    q = 2.0 ** (e - 3.0)
    r = np.rint(a / q) * q                 # rint: ties to even, which is the even mantissa code
    r = np.minimum(r, E4M3_MAX)
    out = np.where(np.isnan(x), np.nan, np.sign(x) * r)
    return out.astype(np.float32)
