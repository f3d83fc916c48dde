"""Pin of the quantizer's quotient (Sec. 3.2 format; the reading that codes are rint((x - bias) / scale_stored) with a
correctly rounded binary32 subtraction and a correctly rounded binary32 division, ties to even).

The expected scale bits, bias bits and codes are worked out here in exact rational arithmetic
(`fractions.Fraction`): every binary32 operation is the exact result rounded once to 24 significant bits, every
stored parameter the exact value rounded once to binary16 or bfloat16.  Nothing of the oracle's arithmetic is
re-used.  The inputs are groups whose quotients lie on, just below and just above k + 1/2 for scales that are not
powers of two, where a reciprocal multiply, a fused operation or a division by the unrounded scale gives other
codes than the division; the test first shows that the rows do separate those variants.  Runs without a GPU."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests.util import tie_adjacent_rows, tie_adjacent_rows_bf16, unpack_codes

F16 = np.float16


def floor_log2(q):
    """Largest e with 2**e <= q, for a positive Fraction."""
    e = q.numerator.bit_length() - q.denominator.bit_length()
    if Fraction(2) ** e > q:
        e -= 1
    assert Fraction(2) ** e <= q < Fraction(2) ** (e + 1)
    return e


def rint_even(q):
    """Nearest integer to a Fraction, ties to the even one."""
    fl = q.numerator // q.denominator
    rem = q - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return fl


def round_to(q, precision, emin):
    """The exact value q rounded once, to nearest even, to a binary format with `precision` significant bits whose
    smallest normal exponent is emin (subnormals below it).  No overflow handling: the rows stay in range."""
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    e = max(floor_log2(a), emin)
    ulp = Fraction(2) ** (e - (precision - 1))
    return sign * rint_even(a / ulp) * ulp


def fl32(q):
    return round_to(q, 24, -126)


PARAM = {oracle.F16_PARAMS: (11, -14), oracle.BF16_PARAMS: (8, -126)}


def exact_group(xg, fmt):
    """xg: 64 binary16 values -> (scale as Fraction, bias as Fraction, 64 codes), each step of the format rounded once."""
    x = [Fraction(float(v)) for v in xg]
    mn, mx = min(x), max(x)
    scale32 = fl32(fl32(mx - mn) / 15)
    s = round_to(scale32, *PARAM[fmt])
    b = round_to(mn, *PARAM[fmt])
    if fmt == oracle.F16_PARAMS:
        assert b == mn                       # a binary16 minimum is stored as it is
    codes = []
    for v in x:
        if s == 0:
            codes.append(0)
            continue
        quotient = fl32(fl32(v - b) / s)
        codes.append(min(max(rint_even(quotient), 0), 15))
    return s, b, codes


def param_values(bits, fmt):
    bits = np.asarray(bits, np.uint16)
    if fmt == oracle.F16_PARAMS:
        return bits.view(F16).astype(np.float64)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def reciprocal_codes(x, s, b):
    """Codes of the cheaper quotient (x - b) * (1 / s), in numpy binary32: used only to show that the rows tell it
    from the division."""
    x, s, b = (np.asarray(v, np.float32) for v in (x, s, b))
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        t = np.where(s == 0, np.float32(0), (x - b) * (np.float32(1) / s))
    return np.clip(np.rint(t), 0, 15).astype(np.uint8)


@pytest.mark.parametrize("fmt,rows", [(oracle.F16_PARAMS, tie_adjacent_rows), (oracle.BF16_PARAMS, tie_adjacent_rows_bf16)],
                         ids=["binary16_params", "bfloat16_params"])
def test_quotient_is_the_correctly_rounded_binary32_division(fmt, rows):
    rng = np.random.default_rng(11)
    ties = rows()
    assert ties.shape[0] > 700 and ties.shape[1] == 64
    # plus ordinary groups: unit normal, with x8 elements, far from zero (a bfloat16 bias is then not the minimum
    # and both clamps act), tiny
    wide = rng.standard_normal((60, 64))
    wide[:, ::9] *= 8
    x = np.concatenate([ties, rng.standard_normal((60, 64)).astype(F16), wide.astype(F16),
                        (1000 + rng.standard_normal((60, 64))).astype(F16),
                        (-3 + 0.01 * rng.standard_normal((60, 64))).astype(F16),
                        (rng.standard_normal((30, 64)) * 1e-5).astype(F16)])
    codes, scale, bias = oracle.quantize(x, fmt)
    got = unpack_codes(codes)
    want = np.empty(x.shape, np.uint8)
    want_s = np.empty(len(x))
    want_b = np.empty(len(x))
    for r in range(len(x)):
        s, b, c = exact_group(x[r], fmt)
        want[r], want_s[r], want_b[r] = c, float(s), float(b)       # parameters are exactly representable doubles
    assert np.array_equal(param_values(scale[:, 0], fmt), want_s), "stored scale"
    assert np.array_equal(param_values(bias[:, 0], fmt), want_b), "stored bias"
    bad = np.argwhere(got != want)
    assert len(bad) == 0, f"{len(bad)} codes differ from the exact quotient, first at {bad[0]}"
    # the rows are sharp enough: a reciprocal multiply would change some codes (it must not pass this test)
    n = len(ties)
    recip = reciprocal_codes(x[:n], want_s[:n, None], want_b[:n, None])
    assert (recip != want[:n]).sum() >= 20
    # and every code value occurs, so a clamp or an offset cannot hide
    assert set(np.unique(want)) == set(range(16))


def test_exact_model_on_hand_checked_quotients():
    """The rational model itself, on values small enough to check by hand: scale 3/8 (0x3600), bias 0,
    x = 3/8 * (k + 1/2) are exact ties (to even); one binary16 step above or below decides the other way."""
    s = 0.375
    g = np.zeros(64)
    g[1] = 15 * s
    g[2:8] = [0.5 * s, 1.5 * s, 2.5 * s, 3.5 * s, 13.5 * s, 14.5 * s]
    x = g.astype(F16)
    assert np.array_equal(x.astype(np.float64), g)                   # all exactly representable
    st, bt, c = exact_group(x, oracle.F16_PARAMS)
    assert st == Fraction(3, 8) and bt == 0
    assert c[:8] == [0, 15, 0, 2, 2, 4, 14, 14]
    up = (x.view(np.uint16) + np.uint16(1)).view(F16)
    up[:2] = x[:2]
    assert exact_group(up, oracle.F16_PARAMS)[2][2:8] == [1, 2, 3, 4, 14, 15]
    codes, scale, bias = oracle.quantize(np.stack([x, up]))
    assert scale[0, 0] == 0x3600 and bias[0, 0] == 0
    assert unpack_codes(codes)[0, :8].tolist() == c[:8]
    assert unpack_codes(codes)[1, 2:8].tolist() == [1, 2, 3, 4, 14, 15]
