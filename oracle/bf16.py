"""Software bfloat16 rounding for the CPU oracle (test infrastructure only).

bfloat16 = 1 sign bit, 8 exponent bits, 7 fraction bits: the top half of an IEEE
binary32 word (Sec. 2.1 and Appendix B of the paper).  Converting binary32 to
bfloat16 keeps the upper 16 bits and rounds on the lower 16 with
round-to-nearest, ties-to-even (the rounding stage of the addition procedure in Appendix B).
"""
import numpy as np


def bf16_bits(x):
    """binary32 array -> uint16 array of bfloat16 bit patterns (RNE).

    Appendix B, rounding stage: the discarded part is compared with half of the last kept
    bit; above half rounds away, below half truncates, exactly half goes to the
    neighbour whose last kept bit is 0.  NaNs are returned as a quiet NaN.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    kept = u >> np.uint64(16)
    dropped = u & np.uint64(0xFFFF)
    half = np.uint64(0x8000)
    last_kept_is_odd = (kept & np.uint64(1)) == np.uint64(1)
    round_away = (dropped > half) | ((dropped == half) & last_kept_is_odd)
    out = kept + round_away.astype(np.uint64)          # a carry may ripple into the exponent: correct
    is_nan = np.isnan(x)
    out = np.where(is_nan, np.uint64(0x7FC0), out)
    return out.astype(np.uint16)


def bits_to_float32(b):
    """uint16 bfloat16 bit patterns -> the binary32 values they denote (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x):
    """Round binary32 values to the nearest bfloat16 (ties to even); result held as binary32."""
    x = np.asarray(x, dtype=np.float32)
    return bits_to_float32(bf16_bits(x)).reshape(x.shape)


def is_bf16_valued(x):
    """True when every entry of x is exactly representable in bfloat16."""
    x32 = np.asarray(x, dtype=np.float32)
    if not np.array_equal(x32.astype(np.float64), np.asarray(x, dtype=np.float64)):
        return False
    return bool(np.all((x32.view(np.uint32) & np.uint32(0xFFFF)) == 0))
