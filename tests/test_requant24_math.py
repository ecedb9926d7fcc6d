"""The 24-bit requantisation used by the Dense epilogues and the attention kernel, checked as arithmetic on the CPU.

The kernels limit the accumulator to per-channel bounds, multiply by b 2^(s-c) with a 24-bit multiply-add whose addend
carries bias and rounding, and read the int8 result from the top of the 32-bit word (s = 24: top byte; residual layers,
s = 23: top nine bits, then the residual term is added and the sum clamped).  This file re-derives the constants from
their definition and compares the outcome with the plain definition (Eq. 7-10 with round-half-up and the symmetric
clamp; and, as the selectable other reading, Eq. 10's bare shift, where the rounding addend is 0) over exhaustive or
dense ranges.  Nothing here touches the GPU or the library: it pins the derivation.
"""
import random

import pytest


def rnd_shift(v, c, rnd=1):
    """rnd = 1: round half up; rnd = 0: the bare shift of Eq. 10 (floor)"""
    return (v + (rnd << (c - 1))) >> c


def clamp8(v):
    return max(-127, min(127, v))


def wrap32(v):
    v &= 0xFFFFFFFF
    return v - (1 << 32) if v >= (1 << 31) else v


def mul24(a, b):
    """low 32 bits of the product of the sign-extended low 24 bits (what v_mad_i32_i24 multiplies)"""
    def sx(x):
        x &= 0xFFFFFF
        return x - (1 << 24) if x >= (1 << 23) else x
    return sx(a) * sx(b)


def constants(b, c, bias, wlim, s, rnd=1):
    half, two_c = rnd << (c - 1), 1 << c                  # the rounding addend h: 2^(c-1), or 0 for the bare shift
    lp = -((-(wlim * two_c - half)) // b)                 # first v with (b v + h) >> c >= wlim (ceiling division)
    ln = -(((wlim - 1) * two_c + 1 + half + b - 1) // b)  # last v with (b v + h) >> c <= -wlim
    lo, hi = ln - bias, lp - bias
    ok = 1 <= c <= s and 1 <= b < (1 << (c - 1)) and -(1 << 23) <= lo and hi < (1 << 23)
    mb = b << (s - c)
    ad = wrap32((bias * b + half) << (s - c))
    return ok, lo, hi, mb, ad


def narrow(v_acc, b, c, bias, wlim, s, rnd=1):
    ok, lo, hi, mb, ad = constants(b, c, bias, wlim, s, rnd)
    assert ok
    m = max(lo, min(hi, v_acc))
    return wrap32(mul24(m, mb) + ad) >> s


@pytest.mark.parametrize("rnd", [1, 0])
@pytest.mark.parametrize("seed", range(40))
def test_top_byte_form_equals_the_definition(seed, rnd):
    rng = random.Random(seed)
    c = rng.choice([1, 2, 5, 11, 16, 20, 23, 24]) if seed % 3 else rng.randint(2, 24)
    if c == 1:
        pytest.skip("b < 2^(c-1) leaves no multiplier at c = 1")
    b = rng.choice([1, (1 << (c - 1)) - 1, rng.randint(1, (1 << (c - 1)) - 1)])
    bias = rng.choice([0, rng.randint(-(1 << 20), 1 << 20)])
    ok, lo, hi, mb, ad = constants(b, c, bias, 127, 24, rnd)
    if not ok:
        pytest.skip("outside the narrow form (bounds beyond 24 bits)")
    # accumulators around both bounds, around zero, and spread over the whole 24-bit-plus range
    vs = set(range(lo - 300, lo + 300)) | set(range(hi - 300, hi + 300)) | set(range(-bias - 300, -bias + 300))
    vs |= {rng.randint(-(1 << 30), 1 << 30) for _ in range(3000)} | {-(1 << 31), (1 << 31) - 1}
    for v in vs:
        assert narrow(v, b, c, bias, 127, 24, rnd) == clamp8(rnd_shift(b * (v + bias), c, rnd)), (v, b, c, bias)


@pytest.mark.parametrize("rnd", [1, 0])
@pytest.mark.parametrize("seed", range(40))
def test_residual_form_equals_the_definition(seed, rnd):
    """First term limited to +-(127 + R2) in bits 23..31, residual term by its own 24-bit multiply-add, sum clamped."""
    rng = random.Random(1000 + seed)
    cr = rng.randint(1, 30)
    br = rng.randint(1, min((1 << 23) - 1, max(1, (1 << cr) + rng.choice([0, 1, -1]) * rng.randint(0, 1 << max(0, cr - 3)))))
    hr = rnd << (cr - 1)
    r2 = max((127 * br + hr) >> cr, -((-128 * br + hr) >> cr))
    if r2 > 128:
        pytest.skip("residual term too large for the narrow form")
    wlim = 127 + r2
    c = rng.randint(2, 23)
    b = rng.choice([1, (1 << (c - 1)) - 1, rng.randint(1, (1 << (c - 1)) - 1)])
    bias = rng.choice([0, rng.randint(-(1 << 19), 1 << 19)])
    ok, lo, hi, mb, ad = constants(b, c, bias, wlim, 23, rnd)
    if not ok:
        pytest.skip("outside the narrow form")
    vs = set(range(lo - 200, lo + 200)) | set(range(hi - 200, hi + 200)) | set(range(-bias - 200, -bias + 200))
    vs |= {rng.randint(-(1 << 30), 1 << 30) for _ in range(1500)} | {-(1 << 31), (1 << 31) - 1}
    for v in vs:
        t1 = narrow(v, b, c, bias, wlim, 23, rnd)
        for res in (-128, -127, -1, 0, 1, 127, rng.randint(-128, 127)):
            t2 = wrap32(mul24(res, br) + hr) >> cr
            assert t2 == rnd_shift(br * res, cr, rnd)
            want = clamp8(rnd_shift(b * (v + bias), c, rnd) + rnd_shift(br * res, cr, rnd))
            assert clamp8(t1 + t2) == want, (v, res, b, c, bias, br, cr)
