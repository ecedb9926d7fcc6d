"""Pins for the CPU oracle: every function is checked against something other than itself.

The oracle is what the GPU library is compared with, so it is pinned here to what the paper and
plain mathematics fix: exact rational rounding (Eq. 8-10), floor(sqrt) (Eq. 20), exp / softmax /
GELU / LayerNorm in floating point within bounds derived from the two approximations of
Eq. 13 and Eq. 15, closed forms, invariants and library integer matmuls.  No GPU is used.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle as orc
from paper_2207_01405_amd import synth


def round_half_up(fr):
    return math.floor(fr + Fraction(1, 2))


# ------------------------------------------------------------------ dyadic requantisation (Eq. 8-10)
def test_rnd_shift_is_exact_rational_round_half_up():
    vs = list(range(-4096, 4097, 13)) + [-4096, -1, 0, 1, 4096, 4095, -4095]
    bs = [2 ** 14, 2 ** 14 + 1, 20011, 23170, 30000, 2 ** 15 - 1]
    for c in range(1, 31):
        for b in bs:
            got = orc.rnd_shift_vec(np.array(vs, np.int64) * b, c)
            want = [round_half_up(Fraction(b * v, 2 ** c)) for v in vs]
            assert got.tolist() == want, (b, c)


def test_requant_random_wide_operands_and_clamp():
    rng = np.random.default_rng(7)
    for _ in range(3000):
        v = int(rng.integers(-2 ** 31 + 1, 2 ** 31))
        b = int(rng.integers(1, 2 ** 31))
        c = int(rng.integers(1, 47))
        exact = round_half_up(Fraction(b * v, 2 ** c))
        assert orc.rnd_shift(b * v, c) == exact
        assert orc.requant(v, b, c) == max(-127, min(127, exact))
    # ties go up, for both signs
    assert orc.rnd_shift(1, 1) == 1 and orc.rnd_shift(-1, 1) == 0 and orc.rnd_shift(-3, 1) == -1
    assert orc.requant(10 ** 6, 2 ** 14, 14) == 127 and orc.requant(-10 ** 6, 2 ** 14, 14) == -127


def test_dyadic_pair_tracks_real_rescale_within_one_lsb():
    """Eq. 9: with b/2^c the nearest dyadic to a real rescale x (b in [2^14, 2^15)), |b/2^c - x| <= 2^-(c+1),
    so the integer pipeline is within one LSB of round(x * v) while |v| <= 2^(c+1)."""
    rng = np.random.default_rng(11)
    for _ in range(300):
        x = Fraction(int(rng.integers(1, 2 ** 40)), 2 ** 50)            # a real rescale in (0, 2^-10)
        c = 0
        while round(x * 2 ** (c + 1)) < 2 ** 15:
            c += 1
        b = round(x * 2 ** c)
        assert 2 ** 14 <= b < 2 ** 15 and abs(Fraction(b, 2 ** c) - x) <= Fraction(1, 2 ** (c + 1))
        for v in rng.integers(-2 ** 22, 2 ** 22, size=20):
            v = int(v)
            assert abs(orc.rnd_shift(b * v, c) - round_half_up(x * v)) <= 1


# ------------------------------------------------------------------ integer square root (Eq. 20)
def _isqrt_np(v):
    s = np.floor(np.sqrt(v.astype(np.float64))).astype(np.int64)
    s = np.where(s * s > v, s - 1, s)
    s = np.where((s + 1) * (s + 1) <= v, s + 1, s)
    return s


def test_isqrt10_exhaustive_against_floor_sqrt():
    """Ten fixed iterations land on floor(sqrt v), except when v + 1 is a perfect square, where the
    iteration oscillates between floor and floor + 1; nothing else may happen."""
    n_plus1 = 0
    for lo in range(0, 2 ** 24, 2 ** 22):
        v = np.arange(lo, lo + 2 ** 22, dtype=np.int64)
        r = orc.isqrt10_vec(v)
        s = _isqrt_np(v)
        sq_next = (s + 1) * (s + 1) == v + 1
        assert np.array_equal(r[~sq_next], s[~sq_next])
        assert np.all((r[sq_next] == s[sq_next]) | (r[sq_next] == s[sq_next] + 1))
        n_plus1 += int((r != s).sum())
    assert n_plus1 > 0          # the oscillation is real: a plain floor(sqrt) is not the same function
    assert orc.isqrt10(0) == 0 and orc.isqrt10(1) == 1 and orc.isqrt10(2) == 1 and orc.isqrt10(4) == 2


def test_isqrt10_large_values():
    rng = np.random.default_rng(5)
    for v in rng.integers(1, 2 ** 52, size=4000):
        v = int(v)
        s = math.isqrt(v)
        r = orc.isqrt10(v)
        assert r == s or (r == s + 1 and (s + 1) ** 2 == v + 1)


def test_isqrt10_is_the_tenth_iterate_not_the_converged_one():
    # For v = k^2 - 1 the iteration never settles (e.g. v = 8 from x0 = 4: 3, 2, 3, 2, ...), so the
    # result is defined by the iteration count; the big-integer loop below is Eq. 20 taken literally.
    assert orc.isqrt10(8) == 2 and orc.isqrt10(15) == 4 and orc.isqrt10(3) == 2

    def by_hand(v):
        x = 1 << (v.bit_length() // 2)
        for _ in range(10):
            x = (x + v // x) >> 1
        return x
    for v in (3, 8, 15, 24, 35, 48, 63, 80, 99, 16128, 16129, 64515):
        assert orc.isqrt10(v) == by_hand(v)


# ------------------------------------------------------------------ ShiftExp (Eq. 13-15, Algorithm 1)
def test_shiftexp_closed_forms_and_worked_example():
    for i0 in (4, 8, 12, 32, 64):
        n = 16 - i0.bit_length()
        assert orc.shiftexp(0, i0, n) == i0 << n                     # e^0 = 1 exactly: S/2^N * (I_0 << N) = 1
    # I_0 = 32, I = -32 (x = -1): I_p = -32 - 16 + 2 = -46, q = 1, r = 14, I_b = -7 + 32 = 25
    assert orc.shiftexp(-32, 32, 10) == (25 << 10) >> 1
    # one more by hand: I_0 = 8, I = -5: I_p = -5 + (-3) - (-1) = -7, q = 0, r = 7, I_b = (-7 >> 1) + 8 = 4
    assert orc.shiftexp(-5, 8, 12) == 4 << 12
    # q beyond N: the value is shifted out to zero instead of a negative shift
    assert orc.shiftexp(-127 * 2, 4, 13) == ((((-(-381 + 95 * 4)) >> 1) + 4) << 13) >> 95


@pytest.mark.parametrize("i0,lo,hi", [(8, -0.10, 0.15), (12, -0.07, 0.13), (16, -0.05, 0.13),
                                      (32, -0.03, 0.11), (64, -0.02, 0.10), (100, -0.01, 0.10)])
def test_shiftexp_tracks_exp_within_the_two_approximations(i0, lo, hi):
    """Error model on e^x > 1e-3: the linear 2^f ~ f/2 + 1 overestimates by at most 6.2 %; (1.0111)_b
    for log2 e adds at most +2.5 %; the floors of the shifts move the exponent by < 2/I_0 either way and
    the final shift loses < 1 part in 16.  The measured envelope must lie inside the bound."""
    n = 16 - i0.bit_length()
    I = np.arange(0, -int(6.9 * i0) - 1, -1)
    e = orc.shiftexp_vec(I, i0, n).astype(np.float64) / (i0 * 2.0 ** n)
    rel = e / np.exp(I / i0) - 1.0
    assert lo <= rel.min() and rel.max() <= hi
    assert np.all(np.diff(e) <= 0)                                   # non-increasing as I decreases
    assert np.all(e > 0) and e[0] == 1.0


# ------------------------------------------------------------------ IntDiv (Eq. 16)
def test_intdiv_is_scaled_quotient():
    rng = np.random.default_rng(3)
    for _ in range(2000):
        s = int(rng.integers(2 ** 15, 2 ** 24))
        a = int(rng.integers(0, min(s, 2 ** 16) + 1))
        got = orc.intdiv(a, s, 8, 31)
        exact = Fraction(a * 128, s)
        # floor(2^M / s) underestimates 2^M / s by < 1, so the result is within one below the exact floor
        assert math.floor(exact) - 1 <= got <= math.floor(exact)
    assert orc.intdiv(2 ** 15, 2 ** 15, 8, 31) == 128               # a/s = 1 -> 2^(k-1)


# ------------------------------------------------------------------ Shiftmax (Algorithm 1)
def _sp(i0):
    return synth.shift_params(i0)


@pytest.mark.parametrize("i0", [8, 32, 64])
def test_shiftmax_against_float_softmax_and_invariants(i0):
    rng = np.random.default_rng(i0)
    p = _sp(i0)
    for d in (2, 3, 5, 8, 16, 49, 65, 197):
        x = np.clip(np.rint(rng.standard_normal((400, d)) * i0 * 1.5), -127, 127).astype(np.int8)
        y = orc.shiftmax(x, p).astype(np.int64)
        z = x.astype(np.float64) / i0
        z -= z.max(1, keepdims=True)
        sm = np.exp(z)
        sm /= sm.sum(1, keepdims=True)
        assert np.abs(y / 128.0 - sm).max() <= 0.05                  # includes the 1/128 output step
        assert y.min() >= 0 and y.max() <= 127
        s = y.sum(1)
        assert np.all(s <= 128) and np.all(s > 128 - d)              # each floor loses less than one LSB
        assert np.all(np.take_along_axis(y, x.argmax(1)[:, None], 1)[:, 0] == y.max(1))   # argmax kept
        # order preserving: a larger input never gets a smaller output
        order = np.argsort(x, axis=1, kind="stable")
        assert np.all(np.diff(np.take_along_axis(y, order, 1), axis=1) >= 0)
        # permutation equivariance and invariance to a common shift of the row
        perm = rng.permutation(d)
        assert np.array_equal(orc.shiftmax(x[:, perm], p), y[:, perm].astype(np.int8))
        room = 127 - x.max(1, keepdims=True).astype(np.int64)
        shifted = (x.astype(np.int64) + np.minimum(room, 5)).astype(np.int8)
        keep = (x.astype(np.int64) + np.minimum(room, 5)).min(1) >= -127
        assert np.array_equal(orc.shiftmax(shifted, p)[keep], y[keep].astype(np.int8))


def test_shiftmax_special_rows():
    p = _sp(32)
    assert orc.shiftmax(np.array([[5]], np.int8), p).tolist() == [[127]]          # 2^(k-1) limited to int8
    assert orc.shiftmax(np.array([[-7, -7]], np.int8), p).tolist() == [[64, 64]]
    assert orc.shiftmax(np.array([[9, 9, 9, 9]], np.int8), p).tolist() == [[32, 32, 32, 32]]
    y = orc.shiftmax(np.array([[127, -127, -127]], np.int8), p)
    assert y.tolist() == [[127, 0, 0]]
    # ld > cols: the tail of each row is ignored
    x = np.array([[1, 2, 3, 99], [3, 2, 1, -99]], np.int8)
    assert np.array_equal(orc.shiftmax(x, p, cols=3), orc.shiftmax(np.ascontiguousarray(x[:, :3]), p))
    assert orc.shiftmax(np.zeros((0, 4), np.int8), p).shape == (0, 4)


def test_shiftmax_bias_rows_follow_head_and_token():
    rng = np.random.default_rng(9)
    H, T, cols, n_img = 3, 5, 7, 2
    p = _sp(32)
    x = rng.integers(-60, 60, size=(n_img * H * T, cols)).astype(np.int8)
    bias = rng.integers(-60, 60, size=(H, T, cols)).astype(np.int8)
    got = orc.shiftmax(x, p, bias=bias, H=H, T=T)
    # same thing with the bias added by hand (values stay inside int8 here)
    full = x.reshape(n_img, H, T, cols).astype(np.int64) + bias[None].astype(np.int64)
    assert np.abs(full).max() <= 127
    want = orc.shiftmax(full.reshape(-1, cols).astype(np.int8), p)
    assert np.array_equal(got, want)
    # and with sums outside int8 the rows still behave like softmax of the wide sum
    xb = np.full((H * T, cols), 100, np.int8); xb[:, 0] = 127
    bb = np.zeros((H, T, cols), np.int8); bb[:, :, 1] = 127
    y = orc.shiftmax(xb, p, bias=bb, H=H, T=T).astype(np.int64)
    assert np.all(y.argmax(1) == 1)


# ------------------------------------------------------------------ ShiftGELU (Algorithm 2)
@pytest.mark.parametrize("i0,tol", [(4, 0.09), (8, 0.06), (16, 0.06), (32, 0.05), (64, 0.05)])
def test_shiftgelu_against_float_gelu(i0, tol):
    p = _sp(i0)
    I = np.arange(-127, 128).astype(np.int8)
    g = orc.shiftgelu_raw(I, p).astype(np.float64)
    x = I.astype(np.float64) / i0
    val = g / (i0 * 128.0)                                            # S_out = S_in / 2^(k-1)
    sig = x / (1.0 + np.exp(-1.702 * x))
    erf = np.array([0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in x])
    # bound: sigmoid error of the two ShiftExp approximations (<= ~4 % of |x|) plus the 1/128 step on |x|
    assert np.abs(val - sig).max() <= tol and np.abs(val - erf).max() <= tol + 0.02
    assert g[127] == 0                                                # GELU(0) = 0
    assert np.all(np.sign(g) * np.sign(I.astype(np.int64)) >= 0)      # never flips sign
    assert np.all(np.abs(g) <= np.abs(I.astype(np.int64)) * 128)


def test_shiftgelu_saturates_like_gelu():
    p = _sp(8)                                                        # x = I/8: +-127 is x ~ +-16
    g = orc.shiftgelu_raw(np.array([127, 100, -100, -127], np.int8), p)
    assert g[0] in (127 * 128, 127 * 127) and g[1] in (100 * 128, 100 * 127)
    assert g[2] == 0 and g[3] == 0
    # the int8 version is the raw value pushed through the pinned requantisation
    x = np.arange(-127, 128).astype(np.int8)
    raw = orc.shiftgelu_raw(x, p)
    y = orc.shiftgelu(x, p, (24171, 21))
    assert np.array_equal(y.astype(np.int64), orc.requant_vec(raw.astype(np.int64), 24171, 21))


def test_shiftgelu_handworked_values():
    # I_0 = 32, N = 10, I = 32 (x = 1): I_p = 32 + 16 + 4 + 2 = 54; e1 = ShiftExp(0) = 32768;
    # e2 = ShiftExp(-54): I_p' = -54 - 27 + 4 = -77, q = 2, r = 13, I_b = -7 + 32 = 25, e2 = 25600 >> 2 = 6400;
    # I_div = (floor(2^31 / 39168) * 32768) >> 24 = (54827 * 32768) >> 24 = 107; g = 32 * 107
    assert orc.shiftgelu_raw(np.array([32], np.int8), _sp(32)).tolist() == [32 * 107]
    # I = -1: I_p = -1 - 1 - 1 - 1 = -4 (arithmetic shifts round toward minus infinity)
    # e1 = ShiftExp(-4): I_p' = -4 - 2 + 1 = -5, q = 0, r = 5, I_b = -3 + 32 = 29 -> 29696; e2 = 32768
    # I_div = (floor(2^31 / 62464) * 29696) >> 24 = (34379 * 29696) >> 24 = 60; g = -60
    assert orc.shiftgelu_raw(np.array([-1], np.int8), _sp(32)).tolist() == [-60]


# ------------------------------------------------------------------ I-LayerNorm (Eq. 19-20)
def test_ilayernorm_constant_row_and_shift_invariance():
    rng = np.random.default_rng(21)
    C = 96
    g = rng.integers(128, 400, size=C).astype(np.int32)
    b = rng.integers(-2 ** 24, 2 ** 24, size=C).astype(np.int32)
    for cval in (-127, -3, 0, 50, 127):
        y = orc.ilayernorm(np.full((2, C), cval, np.int8), g, b, 16, 19)
        want = [max(-127, min(127, round_half_up(Fraction(int(v), 2 ** 19)))) for v in b]
        assert y[0].tolist() == want and y[1].tolist() == want       # zero deviation: only beta survives
    x = synth.make_rows(1, 64, C, "normal", 20.0)
    y0 = orc.ilayernorm(x, g, b, 16, 19)
    for sh in (-20, 7, 20):
        xs = x.astype(np.int64) + sh
        ok = (xs.max(1) <= 127) & (xs.min(1) >= -127)
        assert ok.sum() > 10
        assert np.array_equal(orc.ilayernorm(xs[ok].astype(np.int8), g, b, 16, 19), y0[ok])


@pytest.mark.parametrize("C,dist", [(64, "normal"), (192, "uniform"), (384, "normal"), (768, "student_t")])
def test_ilayernorm_against_float_layernorm(C, dist):
    rng = np.random.default_rng(C)
    gamma = 1.0 + 0.1 * rng.standard_normal(C)
    beta = 0.1 * rng.standard_normal(C)
    s_out, F, c = 1.0 / 32.0, 16, 19
    gq = np.rint(gamma * 2.0 ** (c - F) / s_out).astype(np.int32)
    bq = np.rint(beta * 2.0 ** c / s_out).astype(np.int32)
    x = synth.make_rows(C, 200, C, dist, 30.0)
    y = orc.ilayernorm(x, gq, bq, F, c).astype(np.float64)
    xf = x.astype(np.float64)
    mu = xf.mean(1, keepdims=True)
    sd = np.sqrt(((xf - mu) ** 2).mean(1, keepdims=True))
    keep = sd[:, 0] >= 2.0
    ref = (xf - mu) / np.maximum(sd, 1e-9) * gamma / s_out + beta / s_out
    # error budget per element (in output LSBs): the integer std lies in (sd - 1, sd + 1.03], the mean is
    # off by <= 1/2, gamma_q is rounded to 1/16, 2^-F truncation of the reciprocal, final rounding 1/2
    dev = np.abs(xf - mu) + 0.5
    gs = np.abs(gamma) / s_out
    bound = dev * gs * 1.03 / (sd * (sd - 1.0)) + 0.5 * gs / (sd - 1.0) + dev / (sd - 1.0) / 16.0 \
        + dev * gs * 2.0 ** -F + 0.5 + 1e-6
    unclipped = np.abs(ref) < 126.0
    m = keep[:, None] & unclipped
    assert m.mean() > 0.8
    assert np.all(np.abs(y - ref)[m] <= bound[m])
    assert np.abs(y - ref)[m].max() <= 6.0


def test_ilayernorm_rounds_mean_to_nearest_and_floors_variance():
    # row [1, 2]: sum 3, mean = floor((3 + 1) / 2) = 2; dev = [-1, 0]; var = floor(1 / 2) = 0 -> std forced to 1
    # f = 2^16; y = dev * 2^16 * gamma + beta, shift 19
    y = orc.ilayernorm(np.array([[1, 2]], np.int8), np.array([24, 24], np.int32), np.array([0, 0], np.int32), 16, 19)
    assert y.tolist() == [[round_half_up(Fraction(-(2 ** 16) * 24, 2 ** 19)), 0]]
    # row [-1, -2]: sum -3, mean = floor((-3 + 1) / 2) = -1; dev = [0, -1]
    y = orc.ilayernorm(np.array([[-1, -2]], np.int8), np.array([24, 24], np.int32), np.array([0, 0], np.int32), 16, 19)
    assert y.tolist() == [[0, -3]]
    # row [10, -10, 10, -10]: mean 0, var 100, std 10, f = 6553; y = +-10 * 6553 * 256 >> 19 -> round(31.997) = 32
    y = orc.ilayernorm(np.array([[10, -10, 10, -10]], np.int8), np.full(4, 256, np.int32), np.zeros(4, np.int32), 16, 19)
    assert y.tolist() == [[32, -32, 32, -32]]


# ------------------------------------------------------------------ Dense / MatMul (Eq. 7-10)
def _np_requant(acc, b, c):
    """Per-column dyadic rounding built from the pinned scalar primitive."""
    out = np.empty_like(acc)
    for j in range(acc.shape[1]):
        out[:, j] = orc.rnd_shift_vec(acc[:, j] * int(b[j]), int(c[j]))
    return out


@pytest.mark.parametrize("M,N,K", [(37, 24, 16), (5, 7, 80), (65, 192, 64), (130, 40, 256)])
def test_linear_against_library_integer_matmul(M, N, K):
    x = synth.make_rows(M + N, M, K, "normal", 32.0)
    w, bias, rq_b, rq_c = synth.make_linear(M * N, N, K)
    acc = x.astype(np.int64) @ w.astype(np.int64).T + bias.astype(np.int64)[None]
    want = np.clip(_np_requant(acc, rq_b, rq_c), -127, 127)
    got = orc.linear_requant(x, w, bias, rq_b, rq_c)
    assert np.array_equal(got.astype(np.int64), want)
    assert np.abs(want).mean() > 3 and (np.abs(want) == 127).mean() < 0.2                # not degenerate
    # no bias
    want0 = np.clip(_np_requant(acc - bias[None], rq_b, rq_c), -127, 127)
    assert np.array_equal(orc.linear_requant(x, w, None, rq_b, rq_c).astype(np.int64), want0)
    # residual: requantised separately, added before the clamp
    res = synth.make_rows(99, M, N, "uniform")
    rr = (23456, 15)
    want_r = np.clip(_np_requant(acc, rq_b, rq_c)
                     + orc.rnd_shift_vec(res.astype(np.int64) * rr[0], rr[1]), -127, 127)
    got_r = orc.linear_requant(x, w, bias, rq_b, rq_c, residual=res, res_rq=rr)
    assert np.array_equal(got_r.astype(np.int64), want_r)
    # fused ShiftGELU: the int8 result pushed through the pinned elementwise op
    gp, grq = _sp(32), (24171, 21)
    got_g = orc.linear_requant(x, w, bias, rq_b, rq_c, gelu=gp, gelu_rq=grq)
    assert np.array_equal(got_g, orc.shiftgelu(want.astype(np.int8), gp, grq))


def test_linear_identity_and_one_hot():
    K = 32
    x = synth.make_rows(3, 9, K, "uniform")
    eye = np.eye(K, dtype=np.int8)
    one = np.full(K, 2 ** 14, np.int32)
    y = orc.linear_requant(x, eye, None, one, np.full(K, 14, np.int32))      # b / 2^c = 1
    assert np.array_equal(y, x)
    y = orc.linear_requant(x, (3 * eye).astype(np.int8), None, one, np.full(K, 15, np.int32))   # * 3 / 2, ties up
    assert np.array_equal(y.astype(np.int64), np.clip(np.floor(x.astype(np.int64) * 1.5 + 0.5), -127, 127))
    # one-hot input row k picks column k of w^T, i.e. w[:, k]
    w = synth.make_rows(4, 5, K, "uniform")                                   # [N=5, K]
    oh = np.zeros((K, K), np.int8); np.fill_diagonal(oh, 1)
    y = orc.linear_requant(oh, w, None, np.full(5, 2 ** 14, np.int32), np.full(5, 14, np.int32))
    assert np.array_equal(y, w.T)


# ------------------------------------------------------------------ attention, block, forward
def _attention_by_parts(qkv, dims, qk_rq, sm, pv_rq, rel_bias):
    B, T, C, H = dims["B"], dims["T"], dims["C"], dims["H"]
    d = C // H
    q3 = qkv.reshape(B, T, 3, H, d).astype(np.int64)
    o = np.empty((B, T, H, d), np.int64)
    scores = np.empty((B, H, T, T), np.int64)
    probs = np.empty((B, H, T, T), np.int64)
    for b in range(B):
        for h in range(H):
            Q, K, V = q3[b, :, 0, h], q3[b, :, 1, h], q3[b, :, 2, h]
            A = np.clip(orc.rnd_shift_vec((Q @ K.T) * qk_rq[0], qk_rq[1]), -127, 127)
            scores[b, h] = A
            if rel_bias is None:
                P = orc.shiftmax(A.astype(np.int8), sm)
            else:
                P = orc.shiftmax(A.astype(np.int8), sm, bias=rel_bias[h][None], H=1, T=T)
            probs[b, h] = P
            o[b, :, h] = np.clip(orc.rnd_shift_vec((P.astype(np.int64) @ V) * pv_rq[0], pv_rq[1]), -127, 127)
    return o.reshape(B * T, C), scores, probs


@pytest.mark.parametrize("name,B", [("c0_tiny", 2), ("c4_swin_t", 3)])
def test_attention_against_library_matmuls(name, B):
    cfg = synth.CONFIGS[name]
    dims = synth.dims_of(cfg, B)
    blk = synth.make_block(cfg, 0)
    qkv = synth.make_rows(17, B * cfg["T"], 3 * cfg["C"], "normal", 32.0)
    o, sc, pr = orc.attention(qkv, dims, blk["qk_rq"], blk["softmax"], blk["pv_rq"], blk["rel_bias"], want_taps=True)
    o2, sc2, pr2 = _attention_by_parts(qkv, dims, blk["qk_rq"], blk["softmax"], blk["pv_rq"], blk["rel_bias"])
    assert np.array_equal(sc.astype(np.int64), sc2)
    assert np.array_equal(pr.astype(np.int64), pr2)
    assert np.array_equal(o.astype(np.int64), o2)
    assert np.abs(o2).mean() > 1.0 and pr2.max() > 8


def test_attention_with_constant_values_returns_the_scaled_row_sum():
    cfg = synth.CONFIGS["c0_tiny"]
    dims = synth.dims_of(cfg, 1)
    T, C = cfg["T"], cfg["C"]
    qkv = synth.make_rows(5, T, 3 * C, "normal", 32.0)
    qkv[:, 2 * C:] = np.arange(C, dtype=np.int8)[None] - 30          # V identical for every token
    sm, qk, pv = synth.shift_params(32), (20000, 22), (2 ** 14, 21)  # P V rescaled by 1/128
    o, sc, pr = orc.attention(qkv, dims, qk, sm, pv, None, want_taps=True)
    rs = pr.astype(np.int64).sum(-1)                                  # [1, H, T]
    d = C // cfg["H"]
    for h in range(cfg["H"]):
        v = qkv[0, 2 * C + h * d: 2 * C + (h + 1) * d].astype(np.int64)
        want = np.floor((rs[0, h][:, None] * v[None]) / 128.0 + 0.5)
        assert np.array_equal(o[:, h * d:(h + 1) * d].astype(np.int64), want)


def _block_by_parts(x, p, dims):
    t = {}
    t["u"] = orc.ilayernorm(x, p["ln1_gamma"], p["ln1_beta"], p["ln1_f_bits"], p["ln1_c_shift"])
    t["qkv"] = orc.linear_requant(t["u"], p["w_qkv"], p["bias_qkv"], p["qkv_rq_b"], p["qkv_rq_c"])
    o, sc, pr = _attention_by_parts(t["qkv"], dims, p["qk_rq"], p["softmax"], p["pv_rq"], p["rel_bias"])
    t["o"], t["scores"], t["probs"] = o.astype(np.int8), sc.astype(np.int8), pr.astype(np.int8)
    t["xhat"] = orc.linear_requant(t["o"], p["w_proj"], p["bias_proj"], p["proj_rq_b"], p["proj_rq_c"],
                                   residual=x, res_rq=p["res1_rq"])
    t["v"] = orc.ilayernorm(t["xhat"], p["ln2_gamma"], p["ln2_beta"], p["ln2_f_bits"], p["ln2_c_shift"])
    t["h"] = orc.linear_requant(t["v"], p["w_fc1"], p["bias_fc1"], p["fc1_rq_b"], p["fc1_rq_c"],
                                gelu=p["gelu"], gelu_rq=p["gelu_rq"])
    y = orc.linear_requant(t["h"], p["w_fc2"], p["bias_fc2"], p["fc2_rq_b"], p["fc2_rq_c"],
                           residual=t["xhat"], res_rq=p["res2_rq"])
    return y, t


@pytest.mark.parametrize("name,B", [("c0_tiny", 2), ("c4_swin_t", 2)])
def test_block_is_the_composition_of_eq_1_and_2(name, B):
    cfg = synth.CONFIGS[name]
    dims = synth.dims_of(cfg, B)
    p = synth.make_block(cfg, 0)
    x = synth.make_input(cfg, B)
    y, taps = orc.encoder_block(x, p, dims, want_taps=True)
    y2, t2 = _block_by_parts(x, p, dims)
    for k in orc.TAP_NAMES:
        assert np.array_equal(taps[k], t2[k]), k
    assert np.array_equal(y, y2)
    assert np.array_equal(orc.encoder_block(x, p, dims), y)


def test_forward_stacks_blocks_and_images_are_independent():
    cfg = dict(synth.CONFIGS["c0_tiny"], L=3)
    B = 3
    dims = synth.dims_of(cfg, B)
    blocks = synth.make_model(cfg)
    fin = synth.make_final_ln(cfg)
    x = synth.make_input(cfg, B)
    y = orc.forward(x, blocks, dims, fin)
    a = x
    for p in blocks:
        a = orc.encoder_block(a, p, dims)
    assert np.array_equal(orc.forward(x, blocks, dims), a)
    assert np.array_equal(y, orc.ilayernorm(a, fin["gamma"], fin["beta"], fin["f_bits"], fin["c_shift"]))
    # an image's result does not depend on its neighbours in the batch
    T = cfg["T"]
    one = orc.forward(x[T:2 * T], blocks, synth.dims_of(cfg, 1), fin)
    assert np.array_equal(one, y[T:2 * T])


def test_synthetic_workloads_are_not_degenerate():
    """The generator's closed-form shift counts keep every tensor of a block alive and mostly unsaturated."""
    for name in ("c0_tiny", "c4_swin_t"):
        cfg = synth.CONFIGS[name]
        B = 2
        _, taps = orc.encoder_block(synth.make_input(cfg, B), synth.make_block(cfg, 0), synth.dims_of(cfg, B), True)
        for k in ("u", "qkv", "scores", "o", "xhat", "v", "h"):
            t = taps[k].astype(np.int64)
            assert t.std() > 4.0 and (np.abs(t) == 127).mean() < 0.08, (name, k)
        assert taps["probs"].max() > 8


# ------------------------------------------------------------------ embedding layer and head
def test_embed_tokens_special_cases():
    """With the identity rescale (2^14, 14) and a zero position embedding the tokens are the sources; a zero source
    leaves the rescaled position embedding; sums saturate symmetrically."""
    rng = np.random.default_rng(11)
    B, P, C = 3, 5, 16
    tok = rng.integers(-127, 128, size=(B * P, C)).astype(np.int8)
    cls = rng.integers(-127, 128, size=C).astype(np.int8)
    pos = rng.integers(-127, 128, size=(P + 1, C)).astype(np.int8)
    ident = (2 ** 14, 14)
    out = orc.embed_tokens(tok, cls, np.zeros_like(pos), ident, ident, B).reshape(B, P + 1, C)
    assert np.array_equal(out[:, 0], np.broadcast_to(cls, (B, C))) and np.array_equal(out[:, 1:].reshape(B * P, C), tok)
    half = (2 ** 13, 14)                                  # x 0.5, ties up
    out = orc.embed_tokens(np.zeros_like(tok), np.zeros_like(cls), pos, ident, half, B).reshape(B, P + 1, C)
    want = np.floor(pos.astype(np.float64) / 2 + 0.5).astype(np.int8)
    assert np.array_equal(out[1], want)
    big = orc.embed_tokens(np.full_like(tok, 127), np.full_like(cls, -127), np.sign(pos + 0.5).astype(np.int8) * 127, ident, ident, B)
    assert big.max() == 127 and big.min() == -127
    # brute force with exact rationals on a few entries
    from fractions import Fraction
    import math
    tq, pq = (23457, 15), (9001, 15)
    out = orc.embed_tokens(tok, cls, pos, tq, pq, B).reshape(B, P + 1, C)
    for (b, t, c) in ((0, 0, 0), (1, 3, 7), (2, 5, 15), (2, 0, 9)):
        s = int(cls[c]) if t == 0 else int(tok[b * P + t - 1, c])
        v = math.floor(Fraction(s * tq[0], 2 ** tq[1]) + Fraction(1, 2)) + math.floor(Fraction(int(pos[t, c]) * pq[0], 2 ** pq[1]) + Fraction(1, 2))
        assert out[b, t, c] == max(-127, min(127, v))


def test_classifier_head_is_dense_on_class_rows():
    rng = np.random.default_rng(12)
    B, T, C, N = 4, 7, 32, 10
    x = rng.integers(-127, 128, size=(B * T, C)).astype(np.int8)
    w = rng.integers(-127, 128, size=(N, C)).astype(np.int8)
    bias = rng.integers(-1000, 1000, size=N).astype(np.int32)
    rq_b = rng.integers(2 ** 14, 2 ** 15, size=N).astype(np.int32); rq_c = np.full(N, 22, np.int32)
    got = orc.classifier_head(x, T, w, bias, rq_b, rq_c)
    acc = x[::T].astype(np.int64) @ w.astype(np.int64).T + bias
    want = np.clip((acc * rq_b + (1 << 21)) >> 22, -127, 127).astype(np.int8)
    assert np.array_equal(got, want)


def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The oracle's no-overflow and shift-range claims, checked by running it (saturated operands, K = 3072, 31-bit
    multipliers, shifts up to 46, one-hot rows) in a build where signed overflow, bad shifts and bad accesses abort."""
    import os
    import subprocess
    src = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "sanitize_check.c")
    exe = str(tmp_path / "orc_check")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", src, "-o", exe],
                   check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "sanitize_check: ok" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]


# ------------------------------------------------------------------ shifted-window attention mask
def test_masked_attention_drops_masked_keys_and_equals_shiftmax_on_the_rest():
    cfg = synth.CONFIGS["c4_swin_t"]
    B = 64
    d = synth.dims_of(cfg, B)
    blk = synth.make_block(cfg, 0)
    qkv = synth.make_rows(5, B * cfg["T"], 3 * cfg["C"], "normal", 32.0)
    mask = synth.make_shift_mask()
    assert mask.shape == (64, 49, 49) and mask[0].sum() == 0 and mask[63].sum() > 0 and np.array_equal(mask[7], mask[7].T)
    o0 = orc.attention(qkv, d, blk["qk_rq"], blk["softmax"], blk["pv_rq"], blk["rel_bias"])
    o1, sc, pr = orc.attention(qkv, d, blk["qk_rq"], blk["softmax"], blk["pv_rq"], blk["rel_bias"], want_taps=True, mask=mask)
    T, C = cfg["T"], cfg["C"]
    plain = [w for w in range(64) if mask[w].sum() == 0]
    assert np.array_equal(o0.reshape(B, T, C)[plain], o1.reshape(B, T, C)[plain])          # unmasked windows untouched
    assert pr[np.broadcast_to(mask[:, None].astype(bool), pr.shape)].max() == 0           # exp(-100) is 0 in ShiftExp
    # a masked row is the Shiftmax of its unmasked keys alone
    w, h, i = 63, 1, 10
    keep = mask[w, i] == 0
    row = sc[w, h, i].astype(np.int64) + blk["rel_bias"][h, i].astype(np.int64)
    sub = np.clip(row[keep], -127, 127).astype(np.int8)[None]                              # in range here: check
    assert np.array_equal(sub[0].astype(np.int64), row[keep])
    assert np.array_equal(pr[w, h, i][keep], orc.shiftmax(sub, blk["softmax"])[0])


def test_shiftexp_is_zero_beyond_a_1024_entry_table_wherever_a_masked_key_can_land():
    """What the GPU kernel relies on: a masked key sits at least 100 I_0 - 508 below the row maximum (scores and bias
    are int8), and every such distance that is >= 1024 has ShiftExp exactly 0, for every I_0 the ABI allows."""
    for i0 in list(range(1, 400)) + [511, 512, 1000, 4095, 4096, 30000, 65535]:
        n = 16 - int(i0).bit_length()
        lo = max(1024, 100 * i0 - 508)
        hi = 100 * i0 + 508
        if hi < lo:
            continue
        pts = np.unique(np.concatenate([np.arange(lo, min(hi, lo + 3000) + 1), np.linspace(lo, hi, 200).astype(np.int64), [hi]]))
        assert orc.shiftexp_vec(-pts, i0, n).max() == 0, i0


# ------------------------------------------------------------------ windowed models: window / stage structure
def test_window_partition_and_reverse_by_explicit_loops():
    rng = np.random.default_rng(21)
    B, g, w, C = 2, 8, 4, 3
    x = rng.integers(-127, 128, size=(B, g, g, C)).astype(np.int8)
    xw = orc.window_partition(x, w)
    n = g // w
    assert xw.shape == (B * n * n, w * w, C)
    for b in range(B):
        for wy in range(n):
            for wx in range(n):
                for iy in range(w):
                    for ix in range(w):
                        assert np.array_equal(xw[(b * n + wy) * n + wx, iy * w + ix], x[b, wy * w + iy, wx * w + ix])
    assert np.array_equal(orc.window_reverse(xw, w, g), x)


@pytest.mark.parametrize("g,w,s", [(8, 4, 2), (14, 7, 3), (56, 7, 3)])
def test_shift_mask_separates_exactly_the_tokens_the_cyclic_shift_wrapped(g, w, s):
    """A token at position y of the shifted image came from (y + s) mod g: it wrapped iff y + s >= g.  Two tokens of a
    window may attend to each other iff neither or both wrapped, per axis."""
    m = orc.shift_mask(g, w, s)
    n = g // w
    assert m.shape == (n * n, w * w, w * w)
    for wy in range(n):
        for wx in range(n):
            ys = np.repeat(np.arange(w) + wy * w, w)
            xs = np.tile(np.arange(w) + wx * w, w)
            wrapped = np.stack([ys + s >= g, xs + s >= g], 1)
            want = (wrapped[:, None, :] != wrapped[None, :, :]).any(-1).astype(np.int8)
            assert np.array_equal(m[wy * n + wx], want), (wy, wx)
    if (g, w, s) == (56, 7, 3):
        assert np.array_equal(m, synth.make_shift_mask(7, 3, 8))      # the generator's table, written another way


def _tiny_swin_block(seed=5, C=32, H=1, T=16):
    return synth.make_block(dict(T=T, C=C, H=H, F=4 * C, seed=seed, i0="fixed", rel_bias=True), 0)


def test_swin_block_with_one_window_is_the_plain_encoder_block():
    p = _tiny_swin_block()
    rng = np.random.default_rng(22)
    B, g = 3, 4
    x = synth.quantize_act(rng.standard_normal((B, g, g, 32)))
    y = orc.swin_block(x, p, g, window=4, shift=0, H=1)
    want = orc.encoder_block(x.reshape(B * 16, 32), p, dict(B=B, T=16, C=32, H=1, F=128))
    assert np.array_equal(y.reshape(B * 16, 32), want)


@pytest.mark.parametrize("shift", [0, 2])
def test_swin_block_equals_the_encoder_block_on_explicitly_gathered_windows(shift):
    """Everything but attention acts on single tokens, so the block equals: gather tokens window by window (index
    table built by loops from the definition of the cyclic shift), run the plain block with the mask, scatter back."""
    p = _tiny_swin_block(seed=6)
    rng = np.random.default_rng(23)
    B, g, w, C = 2, 8, 4, 32
    n = g // w
    x = synth.quantize_act(rng.standard_normal((B, g, g, C)))
    idx = np.empty((B, n * n, w * w), np.int64)
    for b in range(B):
        for wy in range(n):
            for wx in range(n):
                for iy in range(w):
                    for ix in range(w):
                        sy, sx = (wy * w + iy + shift) % g, (wx * w + ix + shift) % g    # where the shifted image took it from
                        idx[b, wy * n + wx, iy * w + ix] = (b * g + sy) * g + sx
    flat = x.reshape(-1, C)
    q = dict(p)
    if shift:
        q["attn_mask"] = orc.shift_mask(g, w, shift)
    yw = orc.encoder_block(flat[idx.reshape(-1)], q, dict(B=B * n * n, T=w * w, C=C, H=1, F=4 * C))
    want = np.empty_like(flat)
    want[idx.reshape(-1)] = yw
    got = orc.swin_block(x, p, g, w, shift, H=1).reshape(-1, C)
    assert np.array_equal(got, want)
    if shift:       # and the mask matters: without it the result differs
        q.pop("attn_mask")
        assert not np.array_equal(orc.encoder_block(flat[idx.reshape(-1)], q, dict(B=B * n * n, T=w * w, C=C, H=1, F=4 * C)), yw)


def test_patch_merge_concatenation_order_by_loops():
    rng = np.random.default_rng(24)
    B, g, C = 2, 4, 8
    x = rng.integers(-127, 128, size=(B, g, g, C)).astype(np.int8)
    (w, _b, rq_b, rq_c) = synth.make_linear(31, 2 * C, 4 * C)
    gq = rng.integers(200, 300, size=4 * C).astype(np.int32)
    bq = rng.integers(-2 ** 17, 2 ** 17, size=4 * C).astype(np.int32)
    m = dict(ln_gamma=gq, ln_beta=bq, f_bits=16, c_shift=19, w=w, rq_b=rq_b, rq_c=rq_c)
    y = orc.patch_merge(x, m)
    assert y.shape == (B, g // 2, g // 2, 2 * C)
    for b in range(B):
        for yy in range(g // 2):
            for xx in range(g // 2):
                row = np.concatenate([x[b, 2 * yy, 2 * xx], x[b, 2 * yy + 1, 2 * xx], x[b, 2 * yy, 2 * xx + 1],
                                      x[b, 2 * yy + 1, 2 * xx + 1]])[None]
                u = orc.ilayernorm(row, gq, bq, 16, 19)
                assert np.array_equal(y[b, yy, xx], orc.linear_requant(u, w, None, rq_b, rq_c)[0])


def test_mean_pool_is_the_rounded_scaled_token_sum():
    rng = np.random.default_rng(25)
    B, T, C = 3, 49, 16
    x = rng.integers(-127, 128, size=(B, T, C)).astype(np.int8)
    c = 20
    b = round(2 ** c / T)
    got = orc.mean_pool(x, (b, c))
    s = x.astype(np.int64).sum(1)
    want = [[max(-127, min(127, round_half_up(Fraction(int(v) * b, 2 ** c)))) for v in row] for row in s]
    assert got.tolist() == want
    assert np.abs(got - x.astype(np.float64).mean(1)).max() <= 0.5 + 127 * T * abs(b / 2 ** c - 1 / T) + 1e-9
    const = np.full((1, T, C), 77, np.int8)
    assert (orc.mean_pool(const, (b, c)) == 77).all()
    assert (orc.mean_pool(const, (2 * b, c)) == 127).all()          # clamps


def test_swin_forward_chains_the_stages_and_images_are_independent():
    cfg = synth.SWIN["swin_tiny_test"]
    m = synth.make_swin_model(cfg)
    x = synth.make_swin_patches(cfg)
    logits, outs, pooled = orc.swin_forward(x, m, want_stages=True)
    g0 = cfg["grid"]
    assert [o.shape for o in outs] == [(2 * 256, 32), (2 * 64, 64), (2 * 16, 128)]
    assert [[p["shift"] for p in st["blocks"]] for st in m["stages"]] == [[0, 2], [0, 2], [0, 0]]
    one = orc.swin_forward(x[g0 * g0:], m)
    assert np.array_equal(one, logits[1:])
    # the last steps by hand from the last stage's output
    f = m["final_ln"]
    z = orc.ilayernorm(outs[-1], f["gamma"], f["beta"], f["f_bits"], f["c_shift"]).reshape(2, 16, 128)
    assert np.array_equal(pooled, orc.mean_pool(z, m["pool_rq"]))
    hd = m["head"]
    assert np.array_equal(logits, orc.linear_requant(pooled, hd["w"], hd["bias"], hd["rq_b"], hd["rq_c"]))
    for o in outs:
        assert 4.0 < o.std() < 90.0 and (np.abs(o) == 127).mean() < 0.2


# ------------------------------------------------------------------ alternative readings kept as variants
# The row-maximum form needs a wide ShiftExp (values up to 2^29 here) and, with sums that large, a reciprocal
# 2^M / sum with M well above 31, or IntDiv keeps only three bits of the quotient.
WIDE = dict(i0=32, n_shift=24, m_bits=46, k_out=8)


def test_shiftgelu_rowmax_equals_the_elementwise_form_where_the_two_maxima_coincide():
    """Rows without a positive entry have m = 0 for every element in both readings; a constant row has m = I_p."""
    rq = (24171, 21)
    neg = -np.abs(synth.make_rows(61, 40, 96, "normal", 40.0))
    assert np.array_equal(orc.shiftgelu_rowmax(neg, WIDE, rq), orc.shiftgelu(neg, WIDE, rq))
    const = np.repeat(np.arange(-127, 128, dtype=np.int8)[:, None], 7, axis=1)
    assert np.array_equal(orc.shiftgelu_rowmax(const, WIDE, rq), orc.shiftgelu(const, WIDE, rq))
    one = np.arange(-127, 128, dtype=np.int8)[:, None]
    assert np.array_equal(orc.shiftgelu_rowmax(one, WIDE, rq), orc.shiftgelu(one, WIDE, rq))


@pytest.mark.parametrize("i0,tol", [(32, 0.06), (16, 0.09)])
def test_shiftgelu_rowmax_against_float_gelu(i0, tol):
    """x sigmoid(1.702 x) in floating point; Eq. 18 is an identity for any maximum, so the row form has the same
    target.  Tolerance: the two approximations of ShiftExp plus one output LSB, relative to the output scale."""
    p = dict(WIDE, i0=i0, n_shift=29 - i0.bit_length())
    S = 1.0 / i0
    x = synth.make_rows(62, 64, 384, "normal", 1.2 * i0)          # real values about N(0, 1.2^2), a few beyond 4
    s_out = 4.0 / 127.0
    b, c = orc.dyadic_from_float(S / 128.0 / s_out, 15)
    got = orc.shiftgelu_rowmax(x, p, (b, c)).astype(np.float64) * s_out
    xr = x.astype(np.float64) * S
    want = xr / (1.0 + np.exp(-1.702 * xr))
    assert np.abs(got - np.clip(want, -4, 4)).max() <= tol * max(1.0, np.abs(want).max())


def test_shiftgelu_rowmax_loses_small_values_next_to_a_large_maximum_with_a_16_bit_shiftexp():
    """Why the elementwise reading is the default: with the 16-bit ShiftExp range of the other operators, a row whose
    maximum is large shifts BOTH exponent images of a moderate element out to zero; the quotient is then undefined
    (taken as 0) although the true GELU value is not small.  A wide ShiftExp pushes this far out."""
    narrow = dict(i0=8, n_shift=12, m_bits=31, k_out=8)
    wide = dict(i0=8, n_shift=26, m_bits=46, k_out=8)
    row = np.array([[64, 16, 8, 0, -8]], np.int8)                # real 8, 2, 1, 0, -1
    rq = (2 ** 14, 21)                                           # x * 128 -> x
    elem = orc.shiftgelu(row, narrow, rq)[0]
    assert elem[1] >= 15 and elem[2] >= 6                        # GELU(2) = 1.94 -> 15 or 16, GELU(1) = 0.85 -> 6 or 7
    lost = orc.shiftgelu_rowmax(row, narrow, rq)[0]
    assert lost[0] == elem[0] and lost[2] == 0 and lost[4] == 0 != elem[4]    # both exponent images vanished
    kept = orc.shiftgelu_rowmax(row, wide, rq)[0]
    assert np.abs(kept.astype(int) - elem.astype(int)).max() <= 1
    far = np.array([[127, 16, 8, 0, -8]], np.int8)               # a maximum of 15.9: beyond even the widest 32-bit ShiftExp
    assert orc.shiftgelu_rowmax(far, wide, rq)[0][1] == 0


def test_floor_requantisation_differs_from_the_rounded_one_by_at_most_one_step():
    """Eq. 10 printed as a bare shift (floor) against Eq. 8's rounding, the reading used everywhere here: the floor is
    never above, at most one below, and they differ for about half of all values, which is why the rounded form
    (exactly floor(b v / 2^c + 1/2)) is the one built."""
    rng = np.random.default_rng(63)
    v = rng.integers(-2 ** 22, 2 ** 22, size=20000)
    for b, c in ((23170, 22), (2 ** 14, 20), (32767, 24)):
        rounded = orc.rnd_shift_vec(v * b, c)
        floored = (v * b) >> c
        d = rounded - floored
        assert d.min() == 0 and d.max() == 1 and 0.4 < d.mean() < 0.6
        frac = [Fraction(int(x) * b, 2 ** c) for x in v[:200]]
        assert floored[:200].tolist() == [math.floor(f) for f in frac]


def test_floor_mode_of_the_dense_layer_and_of_attention_against_exact_fractions():
    """The selectable other reading of Eq. 10 (a bare shift): every requantisation of the layer is floor(b v / 2^c),
    checked element by element with exact rationals; with all products exact multiples of 2^c both modes coincide."""
    rng = np.random.default_rng(91)
    M, N, K = 5, 7, 16
    x = rng.integers(-128, 128, (M, K)).astype(np.int8)
    w = rng.integers(-128, 128, (N, K)).astype(np.int8)
    bias = rng.integers(-3000, 3000, N).astype(np.int32)
    b = rng.integers(200, 16000, N).astype(np.int32)
    c = rng.integers(15, 22, N).astype(np.int32)
    res = rng.integers(-128, 128, (M, N)).astype(np.int8)
    acc = x.astype(np.int64) @ w.astype(np.int64).T + bias
    fl = lambda v, bb, cc: math.floor(Fraction(int(v) * int(bb), 2 ** int(cc)))
    clamp = lambda v: max(-127, min(127, v))
    got = orc.linear_requant(x, w, bias, b, c, floor_shift=True)
    assert got.tolist() == [[clamp(fl(acc[m, j], b[j], c[j])) for j in range(N)] for m in range(M)]
    rq = (23456, 15)
    got = orc.linear_requant(x, w, bias, b, c, residual=res, res_rq=rq, floor_shift=True)
    assert got.tolist() == [[clamp(fl(acc[m, j], b[j], c[j]) + fl(res[m, j], *rq)) for j in range(N)] for m in range(M)]
    assert not np.array_equal(got, orc.linear_requant(x, w, bias, b, c, residual=res, res_rq=rq))
    # ShiftGELU between the layers: only its output requantisation changes with the mode
    p, grq = synth.shift_params(32), (24171, 21)
    plain = orc.linear_requant(x, w, bias, b, c, floor_shift=True)
    raw = orc.shiftgelu_raw(plain, p).astype(np.int64)
    got = orc.linear_requant(x, w, bias, b, c, gelu=p, gelu_rq=grq, floor_shift=True)
    assert got.tolist() == [[clamp(fl(raw[m, j], *grq)) for j in range(N)] for m in range(M)]
    # b v a multiple of 2^c everywhere: nothing to round, the modes agree
    same = orc.linear_requant(x, w, None, np.full(N, 1 << 10, np.int32), np.full(N, 10, np.int32), floor_shift=True)
    assert np.array_equal(same, orc.linear_requant(x, w, None, np.full(N, 1 << 10, np.int32), np.full(N, 10, np.int32)))

    # attention: scores and output requantised by floor, Shiftmax untouched
    d = dict(B=1, T=5, C=8, H=2, F=16)
    qkv = rng.integers(-128, 128, (5, 24)).astype(np.int8)
    qk, pv, sm = (1234, 14), (300, 15), synth.shift_params(32)
    o, sc, pr = orc.attention(qkv, d, qk, sm, pv, want_taps=True, floor_shift=True)
    for h in range(2):
        q = qkv[:, 4 * h:4 * h + 4].astype(np.int64); k = qkv[:, 8 + 4 * h:12 + 4 * h].astype(np.int64)
        v = qkv[:, 16 + 4 * h:20 + 4 * h].astype(np.int64)
        s_want = [[clamp(fl(t, *qk)) for t in row] for row in (q @ k.T)]
        assert sc[0, h].tolist() == s_want
        assert np.array_equal(pr[0, h], orc.shiftmax(np.array(s_want, np.int8), sm))
        o_want = [[clamp(fl(t, *pv)) for t in row] for row in (pr[0, h].astype(np.int64) @ v)]
        assert o[:, 4 * h:4 * h + 4].tolist() == o_want
    assert not np.array_equal(sc, orc.attention(qkv, d, qk, sm, pv, want_taps=True)[1])
