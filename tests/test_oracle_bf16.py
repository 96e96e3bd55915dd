"""Pins for oracle.bf16 (CPU only): the paper's worked example, its 2-bit table, the defining
properties of round-to-nearest-even, and an independent library conversion."""
import os

import numpy as np
import torch

from oracle.bf16 import bf16_bits, bits_to_float32, round_to_bf16, is_bf16_valued

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_kv(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = line.split("=", 1)
        out[k.strip()] = v.strip()
    return out


def _bits(s):
    return int(s.replace(" ", ""), 2)


def test_worked_addition_of_the_paper():
    g = _read_kv("bf16_worked_addition.txt")
    a = np.array([_bits(g["operand_a_bits"])], dtype=np.uint32).view(np.float32)
    b = np.array([_bits(g["operand_b_bits"])], dtype=np.uint32).view(np.float32)
    assert float(a[0]) == float(g["operand_a_value"])
    assert float(b[0]) == float(g["operand_b_value"])
    # the first operand is a bf16 value plus a small residual that sets the sticky bit
    a_hi = bits_to_float32(np.array([_bits(g["operand_a_bits"]) >> 16], dtype=np.uint16))
    assert float(a_hi[0]) == float(g["operand_a_bf16_part"])
    assert abs(float(a[0]) - float(a_hi[0]) + 0.00087) < 5e-6
    s = (a + b).astype(np.float32)                      # binary32 addition
    assert int(s.view(np.uint32)[0]) == _bits(g["sum_fp32_bits"])
    assert float(s[0]) == float(g["sum_fp32_value"])
    r = bf16_bits(s)
    assert int(r[0]) == _bits(g["sum_bf16_bits"])
    rv = round_to_bf16(s)
    assert float(rv[0]) == float(g["sum_bf16_value"])
    assert float(rv[0]) - float(s[0]) == float(g["rounding_error"])


def test_two_bit_tail_table_and_tie_frequency():
    """Sec. 3.3.2: adding two same-exponent significands overflows by one bit; the bit shifted
    out is the low bit of the sum of the tails.  It is 1 for 4 of the 10 unordered tail pairs
    (= 8 of 16 ordered pairs).  The same is then checked on real bf16 numbers through the
    rounding helper: the sum needs rounding exactly when that bit is 1, and ties go to even."""
    rows = [l.strip() for l in open(os.path.join(GOLDEN, "two_bit_tail_table.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 10
    ones = 0
    for row in rows:
        lhs, rhs = row.split("=")
        a, b = [int(t.strip(), 2) for t in lhs.split("+")]
        assert a + b == int(rhs.strip(), 2)
        ones += (a + b) & 1
    assert ones == 4
    ordered = sum(((a + b) & 1) for a in range(4) for b in range(4))
    assert ordered == 8
    # on bf16 numbers in [1,2): x = 1 + f/128
    n_inexact = 0
    for fa in range(128):
        for fb in range(128):
            x = np.float32(1 + fa / 128.0); y = np.float32(1 + fb / 128.0)
            s = np.array([x + y], dtype=np.float32)
            r = round_to_bf16(s)
            rounding_bit = (fa + fb) & 1
            if rounding_bit:
                n_inexact += 1
                assert r[0] != s[0]
                # exact tie: result has an even last fraction bit, error is half an ulp (2^-7)
                assert abs(float(r[0]) - float(s[0])) == 2.0 ** -7
                assert (int(bf16_bits(r)[0]) & 1) == 0
            else:
                assert r[0] == s[0]
    assert n_inexact == 128 * 128 // 2


def test_sticky_residual_turns_every_tie_into_round_away():
    """Sec. 3.3.2: a small same-signed residual carried in the binary32 accumulator makes
    every midpoint round away from zero, so the mean error of negative sums is negative."""
    errs = []
    for fa in range(128):
        for fb in range(128):
            a = -np.float32(1 + fa / 128.0); b = -np.float32(1 + fb / 128.0)
            acc = np.float32(a + np.float32(-2.0 ** -12))       # residual from small terms
            s = np.array([acc + b], dtype=np.float32)
            errs.append(float(round_to_bf16(s)[0]) - float(s[0]))
    errs = np.array(errs)
    # midpoints (half of the pairs) go down by 2^-7 - 2^-12, the rest up by 2^-12
    expected = 0.5 * (-(2.0 ** -7 - 2.0 ** -12)) + 0.5 * (2.0 ** -12)
    assert abs(errs.mean() - expected) < 1e-12
    assert errs.mean() < 0


def test_rne_defining_properties_exhaustive_upper_half():
    hi = np.arange(0, 0x7F80, dtype=np.uint32)            # all finite non-negative bf16 patterns
    for low, want in ((0x0000, "exact"), (0x7FFF, "down"), (0x8001, "up"), (0x8000, "tie")):
        x = ((hi << 16) | low).view(np.float32)
        r = bf16_bits(x).astype(np.uint32)
        if want in ("exact", "down"):
            assert np.array_equal(r, hi)
        elif want == "up":
            assert np.array_equal(r, hi + 1)
        else:
            assert np.array_equal(r, hi + (hi & 1))       # to the even neighbour
    # sign symmetry
    x = ((hi << 16) | 0x8000).view(np.float32)
    assert np.array_equal(round_to_bf16(-x), -round_to_bf16(x))


def test_nearest_and_idempotent_random():
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-30, 30, 200000))).astype(np.float32)
    r = round_to_bf16(x)
    assert np.array_equal(round_to_bf16(r), r)
    assert is_bf16_valued(r)
    ulp = 2.0 ** (np.floor(np.log2(np.abs(r.astype(np.float64)))) - 7)
    assert np.all(np.abs(r.astype(np.float64) - x.astype(np.float64)) <= 0.5 * ulp * (1 + 1e-12))
    order = np.argsort(x)
    assert np.all(np.diff(r[order]) >= 0)                  # monotone


def test_against_torch_conversion():
    rng = np.random.default_rng(11)
    u = rng.integers(0, 2 ** 32, size=1_000_000, dtype=np.uint64).astype(np.uint32)
    ties = (np.arange(0, 2 ** 16, dtype=np.uint32) << 16) | 0x8000
    u = np.concatenate([u, ties, ties - 1, ties + 1])
    x = u.view(np.float32)
    keep = ~np.isnan(x)
    x = x[keep]
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bf16_bits(x), want)
