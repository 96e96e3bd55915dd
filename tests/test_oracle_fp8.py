"""Exhaustive pins of the E4M3 rounding emulation against the format's bit-field definition."""
import numpy as np

from oracle.fp8 import decode, decode_all, round_to_e4m3, E4M3_MAX


def test_code_table_landmarks():
    assert decode(0x00) == 0.0 and decode(0x01) == 2.0 ** -9 and decode(0x08) == 2.0 ** -6
    assert decode(0x38) == 1.0 and decode(0x37) == 0.9375 and decode(0x39) == 1.125
    assert decode(0x7E) == E4M3_MAX and np.isnan(decode(0x7F)) and decode(0xB8) == -1.0


def test_every_code_is_a_fixed_point_and_every_gap_rounds_to_nearest_even():
    vals = decode_all()
    finite = np.sort(vals[np.isfinite(vals) & (vals >= 0)])
    finite = np.unique(finite)                      # +0 and -0 coincide
    assert len(finite) == 127
    assert np.array_equal(round_to_e4m3(finite), finite.astype(np.float32))
    assert np.array_equal(round_to_e4m3(-finite), (-finite).astype(np.float32))
    codes = {v: c for c, v in enumerate(vals[:127])}
    for lo, hi in zip(finite[:-1], finite[1:]):
        mid = 0.5 * (lo + hi)
        even = lo if codes[lo] % 2 == 0 else hi
        assert round_to_e4m3(mid) == np.float32(even), (lo, hi)
        eps = (hi - lo) * 1e-6
        assert round_to_e4m3(mid - eps) == np.float32(lo) and round_to_e4m3(mid + eps) == np.float32(hi)
        assert round_to_e4m3(-mid) == -np.float32(even)
    assert round_to_e4m3(1e9) == np.float32(E4M3_MAX) and round_to_e4m3(-500.0) == -np.float32(E4M3_MAX)
    assert np.isnan(round_to_e4m3(np.nan))


def test_rounding_of_probabilities_near_one():
    """The neighbours of 1 are 0.9375 and 1.125: everything above 0.96875 becomes exactly 1 (for
    bf16 the threshold is 1 - 2^-9), which is why unit probabilities are so much more frequent."""
    assert round_to_e4m3(0.9688) == 1.0 and round_to_e4m3(0.9687) == np.float32(0.9375)
    assert round_to_e4m3(0.96875) == 1.0          # the tie goes to the even code (1.0 = 0x38)
