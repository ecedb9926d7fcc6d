"""GPU parity: every C-ABI entry point of libivit.so against the CPU oracle, bit for bit.

All tensors are integers, so the bar is exact equality on every element (and on every intermediate tensor
of a block, through the debug taps).  Inputs are the seeded synthetic workloads of
paper_2207_01405_amd.synth.  Sizes span several tiles and ragged tails; the full-size configurations run on
the GPU in the shape the benchmark times and are checked on sampled images, which the oracle computes one by
one (images are independent through the encoder).
"""
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import oracle as orc
from paper_2207_01405_amd import synth

pytestmark = pytest.mark.gpu


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()


def empty(shape, dtype=None):
    import torch
    return torch.empty(shape, dtype=dtype or torch.int8, device="cuda")


def assert_same(got, want, what):
    got = np.asarray(got); want = np.asarray(want)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        first = tuple(bad[0])
        raise AssertionError("%s: %d of %d elements differ; first at %s: gpu %d, oracle %d" %
                             (what, len(bad), got.size, first, got[first], want[first]))


# ------------------------------------------------------------------ I-LayerNorm
@pytest.mark.parametrize("rows,C,dist", [
    (0, 64, "normal"), (1, 64, "normal"), (65, 64, "normal"), (1001, 96, "normal"), (777, 192, "uniform"),
    (2049, 384, "normal"), (300, 768, "student_t"), (33, 1024, "normal"), (50, 100, "normal"), (7, 4, "uniform"),
    (64, 384, "const"), (131, 1536, "normal"), (20, 2048, "student_t"), (9, 1040, "uniform")])
def test_ilayernorm(ivit, rows, C, dist):
    rng = np.random.default_rng(rows + C)
    x = synth.make_rows(rows + C, rows, C, dist, 30.0)
    if rows > 0:
        x[0, :3] = -128; x[-1, -1] = -128           # the ABI takes any int8, -128 included
    g = np.rint((1.0 + 0.1 * rng.standard_normal(C)) * 256).astype(np.int32)
    b = np.rint(0.1 * rng.standard_normal(C) * 2 ** 24).astype(np.int32)
    y = empty((rows, C))
    ivit.ivit_ilayernorm(dev(x), dev(g), dev(b), y, 16, 19)
    assert_same(host(y), orc.ilayernorm(x, g, b, 16, 19), "ilayernorm")


@pytest.mark.parametrize("rows,C", [(170003, 384), (400007, 96)])
def test_ilayernorm_many_rows_every_row(ivit, rows, C):
    """Row counts that reach the kernel instantiations the bandwidth figures are quoted on (8 rows per thread at
    C = 384, 4 at C = 96).  The input is a 4096-row tile repeated, so the oracle runs on the tile and every row of the
    output is compared (rows are independent)."""
    rng = np.random.default_rng(C)
    tile = synth.make_rows(rows + C, 4096, C, "normal", 30.0)
    tile[5, :9] = -128; tile[6] = 127; tile[7] = -128; tile[8, ::2] = -128
    x = np.tile(tile, ((rows + 4095) // 4096, 1))[:rows]
    g = np.rint((1.0 + 0.1 * rng.standard_normal(C)) * 256).astype(np.int32)
    b = np.rint(0.1 * rng.standard_normal(C) * 2 ** 24).astype(np.int32)
    y = empty((rows, C))
    ivit.ivit_ilayernorm(dev(x), dev(g), dev(b), y, 16, 19)
    want = np.tile(orc.ilayernorm(tile, g, b, 16, 19), ((rows + 4095) // 4096, 1))[:rows]
    assert_same(host(y), want, "ilayernorm on %d rows of %d" % (rows, C))


def test_ilayernorm_other_shift_counts_and_spike_rows(ivit):
    C = 768
    x = np.zeros((16, C), np.int8)
    x[np.arange(16), np.arange(16) * 40] = 127           # one-hot spikes: the largest normalised values
    x[8:] = -x[8:]
    b = np.full(C, -12345, np.int32)
    for f_bits, c_shift, gam in ((16, 19, 511), (12, 14, 511), (20, 23, 15), (8, 12, 32767)):
        g = np.full(C, gam, np.int32)              # |dev * f * gamma| stays below 2^31, as the ABI requires
        y = empty((16, C))
        ivit.ivit_ilayernorm(dev(x), dev(g), dev(b), y, f_bits, c_shift)
        assert_same(host(y), orc.ilayernorm(x, g, b, f_bits, c_shift), "ilayernorm f=%d c=%d" % (f_bits, c_shift))


def test_ilayernorm_rows_whose_variance_is_one_below_a_square(ivit):
    """Variances m^2 - 1 are where the ten-step square root of Eq. 20 never settles (it alternates between m - 1 and m);
    m^2 and m^2 - 2 sit on either side.  Rows built to have exactly these variances: k entries at +a, k at -a, one probe
    entry of 1 in a channel of the row's own, the rest 0 (mean 0, variance floor((2 k a^2 + 1) / C)).  The probe
    channel's gamma and beta are set so that its output is 64 for the right standard deviation and moves by several
    steps for a neighbouring one, so a wrong choice between m - 1 and m cannot hide in the int8 rounding."""
    C, F, c = 384, 16, 10
    reach = {}
    for k in range(1, 41):
        for a in range(1, 128):
            reach.setdefault((2 * k * a * a + 1) // C, (k, a))
    rows, stds = [], []
    for m in range(2, 128):
        for v in (m * m - 1, m * m, m * m - 2):
            if v in reach and len(rows) < 300:
                k, a = reach[v]
                r = np.zeros(C, np.int8); r[:k] = a; r[k:2 * k] = -a; r[80 + len(rows)] = 1
                rows.append(r); stds.append(orc.isqrt10(v))
    assert len(rows) > 100
    x = np.stack(rows)
    g = np.ones(C, np.int32); b = np.zeros(C, np.int32)
    G = 2048
    for i, sd in enumerate(stds):
        f = (1 << F) // sd
        g[80 + i] = G; b[80 + i] = 64 * (1 << c) - G * f
        for other in (sd - 1, sd + 1):                       # what a neighbouring standard deviation would print there
            if other >= 1:
                assert abs(((G * ((1 << F) // other) + b[80 + i] + (1 << (c - 1))) >> c) - 64) >= 2
    y = empty(x.shape)
    ivit.ivit_ilayernorm(dev(x), dev(g), dev(b), y, F, c)
    want = orc.ilayernorm(x, g, b, F, c)
    assert [int(want[i, 80 + i]) for i in range(len(rows))] == [64] * len(rows)
    assert_same(host(y), want, "ilayernorm on rows with variance m^2 - 1")


@pytest.mark.parametrize("C,f_bits,c_shift", [(64, 16, 19), (96, 12, 14), (384, 16, 19), (768, 8, 12), (768, 16, 22), (2048, 10, 30)])
def test_ilayernorm_at_the_largest_admissible_parameters(ivit, C, f_bits, c_shift):
    """gamma_q and beta_q of magnitude ivit_ilayernorm_limits allows, on the rows that drive |x - mean| f to its
    bound (constant rows with a few spikes, the variance-3 rows among them) and on ordinary rows: the 32-bit
    arithmetic of the kernel must still equal the 64-bit arithmetic of the oracle."""
    gmax, bmax = ivit.ivit_ilayernorm_limits(C, f_bits, c_shift)
    assert gmax > 0
    rng = np.random.default_rng(C + f_bits)
    rows = []
    for k in (1, 2, 3, 4):
        for h in range(1, 256, 2):
            for base in (0, -128, 127):
                r = np.full(C, base, np.int64)
                r[rng.choice(C, k, replace=False)] = base + h if base <= 0 else base - h
                rows.append(np.clip(r, -128, 127))
    x = np.concatenate([np.stack(rows).astype(np.int8), synth.make_rows(C, 300, C, "normal", 30.0)])
    for sign in (1, -1):
        g = np.where(rng.random(C) < 0.5, gmax, -gmax).astype(np.int32)
        b = np.full(C, sign * bmax, np.int32)
        g[::7] = rng.integers(-gmax, gmax + 1, len(g[::7]))
        y = empty(x.shape)
        ivit.ivit_ilayernorm(dev(x), dev(g), dev(b), y, f_bits, c_shift)
        assert_same(host(y), orc.ilayernorm(x, g, b, f_bits, c_shift), "ilayernorm at the limits C=%d" % C)


# ------------------------------------------------------------------ Shiftmax
@pytest.mark.parametrize("rows,cols,ld,i0", [
    (0, 49, 49, 32), (1, 1, 1, 32), (5, 49, 49, 32), (1000, 65, 65, 32), (4099, 197, 197, 32), (333, 197, 208, 12),
    (100, 256, 256, 64), (17, 1000, 1024, 8), (64, 64, 64, 4), (300, 130, 131, 100),
    # 16 <= cols <= 256: lanes own 16 bytes each, the last one overlapping its neighbour; ragged row counts
    (1, 16, 16, 32), (7, 17, 17, 32), (129, 31, 31, 32), (2000, 32, 40, 16), (1031, 48, 48, 32), (555, 63, 63, 8),
    (4097, 65, 65, 32), (513, 128, 128, 32), (77, 129, 135, 32), (1001, 255, 255, 32), (9000, 49, 49, 32),
    (20000, 197, 197, 20), (3, 15, 15, 32)])
def test_shiftmax(ivit, rows, cols, ld, i0):
    x = synth.make_rows(rows + cols, rows, ld, "normal", 1.5 * min(i0, 40))
    p = synth.shift_params(i0)
    y = empty((rows, cols))
    ivit.ivit_shiftmax(dev(x), y, p, cols=cols)
    assert_same(host(y), orc.shiftmax(x, p, cols=cols), "shiftmax")


def test_shiftmax_extreme_rows(ivit):
    p = synth.shift_params(32)
    x = np.full((6, 197), -128, np.int8)
    x[0, 5] = 127                      # one dominant element
    x[1] = 7                           # all equal
    x[2] = np.arange(197) % 256 - 128  # a ramp
    x[3, :] = 127
    x[4, ::2] = 127
    x[5, 196] = -127
    y = empty((6, 197))
    ivit.ivit_shiftmax(dev(x), y, p)
    assert_same(host(y), orc.shiftmax(x, p), "shiftmax extremes")


def test_shiftmax_general_intdiv_parameters(ivit):
    # I_0 << N not above 2^(k_out - 1), small M, narrow outputs: the reciprocal cannot be pre-shifted
    x = synth.make_rows(9, 700, 197, "normal", 30.0)
    for prm in (dict(i0=3, n_shift=2, m_bits=31, k_out=8), dict(i0=32, n_shift=10, m_bits=20, k_out=8),
                dict(i0=32, n_shift=10, m_bits=31, k_out=4), dict(i0=100, n_shift=0, m_bits=7, k_out=8)):
        y = empty(x.shape)
        ivit.ivit_shiftmax(dev(x), y, prm)
        assert_same(host(y), orc.shiftmax(x, prm), "shiftmax %r" % (prm,))


@pytest.mark.parametrize("n_img,H,T", [(3, 3, 49), (2, 2, 65)])
def test_shiftmax_with_relative_position_bias(ivit, n_img, H, T):
    rng = np.random.default_rng(T)
    x = synth.make_rows(T, n_img * H * T, T, "normal", 40.0)
    bias = np.clip(np.rint(rng.standard_normal((H, T, T)) * 50), -128, 127).astype(np.int8)
    p = synth.shift_params(32)
    y = empty(x.shape)
    ivit.ivit_shiftmax(dev(x), y, p, bias=dev(bias), H=H, T=T)
    assert_same(host(y), orc.shiftmax(x, p, bias=bias, H=H, T=T), "shiftmax+bias")


# ------------------------------------------------------------------ ShiftGELU
@pytest.mark.parametrize("n,i0", [(0, 32), (1, 32), (255, 8), (100003, 32), (65536, 12), (4099, 64)])
def test_shiftgelu(ivit, n, i0):
    import torch
    x = np.random.default_rng(n).integers(-128, 128, size=n).astype(np.int8)
    p = synth.shift_params(i0)
    rq = (24171, 21)
    y = empty((n,))
    ivit.ivit_shiftgelu(dev(x), y, p, rq)
    assert_same(host(y), orc.shiftgelu(x, p, rq), "shiftgelu")
    y16 = empty((n,), torch.int16)
    ivit.ivit_shiftgelu_raw(dev(x), y16, p)
    assert_same(host(y16).astype(np.int32), orc.shiftgelu_raw(x, p), "shiftgelu_raw")
    if n > 16:                          # unaligned views take the byte path
        xd = dev(np.concatenate([np.zeros(1, np.int8), x]))[1:]
        yb = empty((n + 1,))[1:]
        ivit.ivit_shiftgelu(xd, yb, p, rq)
        assert_same(host(yb), orc.shiftgelu(x, p, rq), "shiftgelu unaligned")


@pytest.mark.parametrize("rows,cols,i0,wide,dist", [
    (0, 64, 32, True, "normal"), (1, 4, 32, True, "uniform"), (37, 100, 32, True, "normal"), (513, 384, 16, True, "normal"),
    (300, 1536, 32, True, "student_t"), (65, 3072, 8, True, "normal"), (9, 4096, 32, True, "uniform"), (200, 768, 32, False, "normal"),
    (64, 1536, 8, False, "student_t"), (40, 256, 4, True, "const")])
def test_shiftgelu_rowmax(ivit, rows, cols, i0, wide, dist):
    """The row-maximum reading of Algorithm 2, wide (ShiftExp up to 2^29, 46-bit reciprocal) and 16-bit parameters."""
    x = synth.make_rows(rows + cols, rows, cols, dist, 1.5 * i0)
    if rows > 3:
        x[1] = -np.abs(x[1]); x[2, 0] = 127; x[3] = 127
    p = dict(i0=i0, n_shift=29 - i0.bit_length(), m_bits=46, k_out=8) if wide else synth.shift_params(i0)
    rq = (24171, 21)
    y = empty((rows, cols))
    ivit.ivit_shiftgelu_rowmax(dev(x), y, p, rq)
    assert_same(host(y), orc.shiftgelu_rowmax(x, p, rq) if rows else x, "shiftgelu with the row maximum")
    if rows:
        z = dev(x)
        ivit.ivit_shiftgelu_rowmax(z, z, p, rq)                     # in place
        assert_same(host(z), orc.shiftgelu_rowmax(x, p, rq), "shiftgelu with the row maximum, in place")


# ------------------------------------------------------------------ Dense / MatMul + requant
LIN_SHAPES = [(0, 64, 64), (1, 1, 16), (5, 7, 80), (65, 192, 64), (130, 40, 256), (129, 100, 48), (1000, 384, 384),
              (197, 1536, 384), (300, 384, 1536), (257, 130, 3072), (64, 256, 16),
              # weight-stationary kernel: partial channel slabs, one-chunk K, even / odd unit counts, many groups per wavefront
              (333, 208, 96), (40, 16, 32), (515, 2304, 768), (30011, 128, 384), (2100, 768, 1152), (77, 1168, 640),
              # the largest K the entry point takes, and many short rows
              (3, 16, 65536), (70001, 16, 16)]


@pytest.fixture(params=[None, "many_rows"])
def dense_path(request):
    """Shapes with few rows take a kernel of their own; "many_rows" (an option of ivit_linear_requant_ex) keeps them on
    the kernels for many rows, so that the small test shapes exercise both.  None calls ivit_linear_requant itself."""
    return request.param


@pytest.mark.parametrize("M,N,K", LIN_SHAPES)
@pytest.mark.parametrize("epi", ["plain", "residual", "gelu"])
def test_linear_requant(ivit, dense_path, M, N, K, epi):
    x = synth.make_rows(M + N + K, M, K, "normal", 32.0)
    w, bias, rq_b, rq_c = synth.make_linear(M * 7 + N, N, K)
    if M > 0:
        x[0, :5] = -128; x[-1, -3:] = -128; w[0, :4] = -128; w[-1, -1] = -128        # the ABI takes any int8
    kw_o, kw_g = {}, {}
    if epi == "residual":
        res = synth.make_rows(N + 1, M, N, "uniform")
        kw_o = dict(residual=res, res_rq=(23456, 15)); kw_g = dict(residual=dev(res), res_rq=(23456, 15))
    elif epi == "gelu":
        kw_o = dict(gelu=synth.shift_params(32), gelu_rq=(24171, 21)); kw_g = dict(kw_o)
    y = empty((M, N))
    ivit.ivit_linear_requant(dev(x), dev(w), dev(bias), dev(rq_b), dev(rq_c), y, kernel=dense_path, **kw_g)
    assert_same(host(y), orc.linear_requant(x, w, bias, rq_b, rq_c, **kw_o), "linear %s" % epi)


@pytest.fixture(params=[None, "floor"])
def rounding(request):
    """None: the entry point's own rounding (to nearest); "floor": the bare shift of Eq. 10, an option of the _ex entry
    points, compared with the oracle's floor mode."""
    return request.param


def test_linear_requant_general_dyadic_pairs_and_no_bias(ivit, dense_path, rounding):
    """Multipliers and shifts outside the 15-bit fast range take the 64-bit path, channel by channel."""
    fs = rounding == "floor"
    rng = np.random.default_rng(42)
    M, N, K = 200, 96, 128
    x = synth.make_rows(1, M, K, "uniform")
    w = synth.make_rows(2, N, K, "uniform")
    rq_c = rng.integers(1, 47, size=N).astype(np.int32)
    # keep the product scale around 2^-11 so that outputs stay informative: b ~ 2^(c - 11)
    rq_b = np.array([int(rng.integers(2 ** max(0, min(29, c - 12)), 2 ** max(1, min(31, c - 10)))) for c in rq_c],
                    np.int32)
    rq_b[:8] = 2 ** 31 - 1; rq_c[:8] = 46
    res = synth.make_rows(3, M, N, "uniform")
    gl = dict(gelu=synth.shift_params(20), gelu_rq=(2 ** 31 - 1, 38))
    for kw_o, kw_g in (({}, {}), (dict(residual=res, res_rq=(2 ** 31 - 1, 31)), dict(residual=dev(res), res_rq=(2 ** 31 - 1, 31))),
                       (dict(residual=res, res_rq=(3, 1)), dict(residual=dev(res), res_rq=(3, 1))), (gl, gl)):
        y = empty((M, N))
        ivit.ivit_linear_requant(dev(x), dev(w), None, dev(rq_b), dev(rq_c), y, kernel=dense_path, rounding=rounding, **kw_g)
        want = orc.linear_requant(x, w, None, rq_b, rq_c, floor_shift=fs, **kw_o)
        assert_same(host(y), want, "linear general")
        assert np.abs(want.astype(np.int32)).mean() > 2


def test_linear_requant_largest_accumulators(ivit, dense_path):
    """K = 65536 with every operand at +-127: the dot products reach +-65536 * 127^2 = +-1.057e9, the largest an int32
    accumulator of this entry point ever holds; shifts chosen so that results spread over the int8 range."""
    M, N, K = 8, 32, 65536
    x = np.full((M, K), 127, np.int8); x[1] = -127; x[2, ::2] = -127; x[3, : K // 4] = -127; x[4:] = synth.make_rows(1, 4, K, "uniform")
    w = np.full((N, K), 127, np.int8); w[1::2] = -127; w[2, ::3] = 0; w[5] = synth.make_rows(2, 1, K, "uniform")[0]
    bias = np.linspace(-2 ** 20, 2 ** 20, N).astype(np.int32)
    rq_c = np.full(N, 24, np.int32); rq_c[8:16] = 31; rq_c[16:24] = 40
    rq_b = np.full(N, 3, np.int32); rq_b[8:16] = 200; rq_b[16:24] = 2 ** 17 + 1; rq_b[24:] = 1
    for kw_o, kw_g in (({}, {}), (dict(gelu=synth.shift_params(32), gelu_rq=(24171, 21)),) * 2):
        y = empty((M, N))
        ivit.ivit_linear_requant(dev(x), dev(w), dev(bias), dev(rq_b), dev(rq_c), y, kernel=dense_path, **kw_g)
        want = orc.linear_requant(x, w, bias, rq_b, rq_c, **kw_o)
        assert_same(host(y), want, "linear with the largest accumulators")
    plain = orc.linear_requant(x, w, bias, rq_b, rq_c)
    assert (np.abs(plain) == 127).any() and (np.abs(plain) < 127).mean() > 0.3


@pytest.mark.parametrize("K", [128, 1536, 384, 768])
def test_linear_requant_narrow_multiplier_path_at_its_limits(ivit, dense_path, K, rounding):
    """Per-channel parameters at and around the limits of the 24-bit requantisation (shift 1..24, multiplier just
    below and at 2^(c-1), biases that push the clamp bounds to and past 24 bits), on operands that drive the
    accumulators to both saturated ends (K * 127^2 exceeds 2^23 for the larger K) and through the whole range.
    Slabs of 64 channels share one regime each, so both the narrow path and its fallbacks run.  K = 384, 768 and 1536
    are run on the kernels that keep the weights in registers as well (their workgroups span 256 or 128 channels)."""
    if K in (384, 768, 1536) and dense_path == "many_rows":
        dense_path = "reg_stationary"
    fs = rounding == "floor"
    rng = np.random.default_rng(K)
    M, N = 333, 64 * 10
    x = synth.make_rows(K, M, K, "uniform")
    x[0:8] = 127; x[8:16] = -127; x[16:24] = 0; x[24:32, ::2] = 127; x[24:32, 1::2] = -127
    w = synth.make_rows(K + 1, N, K, "uniform")
    w[0::64] = 127; w[1::64] = -127; w[2::64] = 0
    w[3::64] = (np.arange(K) % 2 * 2 - 1) * 127
    b = np.empty(N, np.int64); c = np.empty(N, np.int64); bias = np.zeros(N, np.int64)
    sig = math.sqrt(K) * 73.0 * 73.0                                   # accumulator spread of uniform operands
    for slab in range(10):
        sl = slice(64 * slab, 64 * slab + 64)
        if slab < 6:        # narrow path: c from the top of the range down, b ~ 30 2^c / sigma, capped below 2^(c-1)
            cc = (24, 23, 20, 17, 14, 11)[slab]
            top = 2 ** (cc - 1) - 1
            c[sl] = cc
            b[sl] = np.clip(rng.integers(int(20 * 2 ** cc / sig) + 1, int(40 * 2 ** cc / sig) + 2, size=64), 1, top)
            b[64 * slab] = top; b[64 * slab + 1] = 1
            bias[sl] = rng.integers(-int(3 * sig), int(3 * sig), size=64)
            bias[64 * slab + 5] = 2 ** 20; bias[64 * slab + 6] = -2 ** 20
        elif slab == 6:     # b = 2^(c-1) exactly: just outside
            c[sl] = 16; b[sl] = 2 ** 15
        elif slab == 7:     # biases near +-2^23: bounds leave the 24-bit range for some channels
            c[sl] = 22; b[sl] = rng.integers(2 ** 14, 2 ** 15, size=64); bias[sl] = rng.choice([-1, 1], 64) * (2 ** 23 - rng.integers(0, 2 ** 17, size=64))
        elif slab == 8:     # c = 25: outside
            c[sl] = 25; b[sl] = rng.integers(2 ** 15, 2 ** 16, size=64)
        else:               # mixed shifts inside one slab, all narrow
            c[sl] = rng.integers(18, 25, size=64); b[sl] = [int(rng.integers(2 ** (cc - 10), 2 ** (cc - 8))) for cc in c[sl]]
            bias[sl] = rng.integers(-2 ** 18, 2 ** 18, size=64)
    b = b.astype(np.int32); c = c.astype(np.int32); bias = bias.astype(np.int32)
    gl = dict(gelu=synth.shift_params(32), gelu_rq=(24171, 21))
    for kw in ({}, gl):
        y = empty((M, N))
        ivit.ivit_linear_requant(dev(x), dev(w), dev(bias), dev(b), dev(c), y, kernel=dense_path, rounding=rounding, **kw)
        want = orc.linear_requant(x, w, bias, b, c, floor_shift=fs, **kw)
        assert_same(host(y), want, "linear at the limits of the narrow path" + (" + gelu" if kw else ""))
    plain = orc.linear_requant(x, w, bias, b, c)
    assert (plain == 127).mean() > 0.02 and (plain == -127).mean() > 0.02 and (np.abs(plain) < 127).mean() > 0.3
    # the residual layers' 24-bit form (shift <= 23, residual multiplier below 2^23, residual term at most 128 in
    # magnitude) at and past its limits; the residual holds -128 as well, and saturated rows on both sides
    res = synth.make_rows(K + 2, M, N, "uniform")
    res[0:4] = 127; res[4:8] = -128; res[8:12] = -127; res[12:16] = 127; res[16:20] = -128
    for rq in ((2 ** 15, 15), (2 ** 15 - 1, 15), (2 ** 15 + 1, 15), (33000, 15), (2 ** 23 - 1, 23), (2 ** 23, 23),
               (2 ** 23 - 1, 30), (5, 31), (1, 1), (3, 2), (23456, 15)):
        y = empty((M, N))
        ivit.ivit_linear_requant(dev(x), dev(w), dev(bias), dev(b), dev(c), y, residual=dev(res), res_rq=rq, kernel=dense_path,
                                 rounding=rounding)
        want = orc.linear_requant(x, w, bias, b, c, residual=res, res_rq=rq, floor_shift=fs)
        assert_same(host(y), want, "linear + residual at the limits of the narrow path, residual pair %s" % (rq,))


# Eq. 10 as a bare shift: every epilogue of every Dense kernel (few rows, tiled, weights in LDS, weights in registers)
FLOOR_SHAPES = [(65, 192, 64, None), (5, 7, 80, None), (1000, 384, 384, "many_rows"), (300, 384, 1536, "many_rows"),
                (257, 130, 3072, "many_rows"), (333, 208, 96, "many_rows"), (30011, 128, 384, None),
                (1000, 1152, 384, "reg_stationary"), (4100, 384, 384, "reg_stationary"), (515, 256, 768, "reg_stationary"),
                (700, 384, 1536, "reg_stationary"), (700, 256, 512, "big_tiles")]


@pytest.mark.parametrize("M,N,K,kernel", FLOOR_SHAPES)
@pytest.mark.parametrize("epi", ["plain", "residual", "gelu"])
def test_linear_requant_floor_mode(ivit, M, N, K, kernel, epi):
    x = synth.make_rows(M + N + K, M, K, "normal", 32.0)
    w, bias, rq_b, rq_c = synth.make_linear(M * 7 + N, N, K)
    x[0, :5] = -128; w[-1, -1] = -128
    kw_o, kw_g = {}, {}
    if epi == "residual":
        res = synth.make_rows(N + 1, M, N, "uniform")
        kw_o = dict(residual=res, res_rq=(23456, 15)); kw_g = dict(residual=dev(res), res_rq=(23456, 15))
    elif epi == "gelu":
        kw_o = dict(gelu=synth.shift_params(32), gelu_rq=(24171, 21)); kw_g = dict(kw_o)
    y = empty((M, N))
    ivit.ivit_linear_requant(dev(x), dev(w), dev(bias), dev(rq_b), dev(rq_c), y, kernel=kernel, rounding="floor", **kw_g)
    want = orc.linear_requant(x, w, bias, rq_b, rq_c, floor_shift=True, **kw_o)
    assert_same(host(y), want, "linear %s, floor" % epi)
    assert (want != orc.linear_requant(x, w, bias, rq_b, rq_c, **kw_o)).mean() > 0.05      # the modes really differ
    y2 = empty((M, N))                                                                      # and "nearest" through the option
    ivit.ivit_linear_requant(dev(x), dev(w), dev(bias), dev(rq_b), dev(rq_c), y2, kernel=kernel, rounding="nearest", **kw_g)
    assert_same(host(y2), orc.linear_requant(x, w, bias, rq_b, rq_c, **kw_o), "linear %s, nearest through the option" % epi)


# the kernel that keeps the weights in registers (K = 384 / 768): row counts around the 32-token tiles and around the
# number of workgroups, channel counts that fill, underfill and overfill the workgroups' slabs (384 channels at
# K = 384, 256 at K = 768), every epilogue; forced through the option so that small row counts reach it too
RS_SHAPES = [(1, 32, 384), (31, 384, 384), (32, 96, 384), (33, 1152, 384), (197, 384, 384), (1000, 1536, 384), (2500, 416, 384),
             (8203, 384, 384), (9000, 1152, 384), (64, 768, 768), (333, 256, 768), (1577, 2304, 768), (300, 3072, 768),
             (8300, 768, 768), (95, 160, 768),
             # K = 1536: the kernel that splits K over pairs of wavefronts (128 channels per workgroup): one tile, an even and an
             # odd number of tiles per workgroup, partial slabs, more workgroups than tiles
             (1, 32, 1536), (32, 128, 1536), (33, 384, 1536), (197, 96, 1536), (1000, 384, 1536), (2500, 416, 1536),
             (8203, 384, 1536), (16400, 128, 1536), (300, 1536, 1536),
             # K = 192 (no residual layers): six k-steps a tile
             (1, 32, 192), (33, 576, 192), (197, 768, 192), (1000, 96, 192), (8203, 576, 192), (20000, 768, 192)]


# the kernel with 256 x 128 tiles and both operands streamed: one tile, ragged last tiles, several tiles per workgroup
# (more than 256 tiles), the shortest K it takes, long K; with 18 stages or more (K >= 2304) and a second tile in the
# workgroup the epilogue of a tile runs inside the next tile's k-loop: 18 stages exactly, 20 (the last tile's last
# stages request nothing more), 24
TL_SHAPES = [(1, 128, 384), (255, 128, 640), (256, 256, 3072), (257, 128, 1024), (700, 384, 768), (5000, 768, 3072),
             (40000, 256, 384), (33000, 384, 512), (17000, 512, 2304), (9001, 1024, 2560), (33000, 384, 3072),
             (16500, 512, 2048)]


@pytest.mark.parametrize("M,N,K", TL_SHAPES)
@pytest.mark.parametrize("epi", ["plain", "residual", "gelu"])
def test_linear_requant_big_tiles(ivit, M, N, K, epi):
    x = synth.make_rows(M + N + K, M, K, "normal", 32.0)
    x[0, :7] = -128; x[-1, -3:] = -128
    w, bias, rq_b, rq_c = synth.make_linear(M * 7 + N, N, K)
    w[0, :5] = -128
    kw_o, kw_g = {}, {}
    if epi == "residual":
        res = synth.make_rows(N + 1, M, N, "uniform")
        res[-1, ::3] = -128
        kw_o = dict(residual=res, res_rq=(23456, 15)); kw_g = dict(residual=dev(res), res_rq=(23456, 15))
    elif epi == "gelu":
        kw_o = dict(gelu=synth.shift_params(32), gelu_rq=(24171, 21)); kw_g = dict(kw_o)
    y = empty((M, N))
    ivit.ivit_linear_requant(dev(x), dev(w), dev(bias), dev(rq_b), dev(rq_c), y, kernel="big_tiles", **kw_g)
    if M * N * K <= 6e9:
        assert_same(host(y), orc.linear_requant(x, w, bias, rq_b, rq_c, **kw_o), "linear (big tiles) %s" % epi)
    else:       # the oracle on a sample of rows (first and last tiles, and rows spread over the rest); every row against the other kernel
        rows = np.unique(np.concatenate([np.arange(0, 300), np.arange(M - 300, M), np.arange(0, M, 97)]))
        assert_same(host(y)[rows], orc.linear_requant(x[rows], w, bias, rq_b, rq_c, **({} if epi != "residual" else dict(residual=res[rows], res_rq=(23456, 15))) if epi != "gelu" else kw_o), "linear (big tiles) %s, sampled rows" % epi)
        y2 = empty((M, N))
        ivit.ivit_linear_requant(dev(x), dev(w), dev(bias), dev(rq_b), dev(rq_c), y2, kernel="many_rows", **kw_g)
        assert bool((y == y2).all())


@pytest.mark.parametrize("rounding", ["nearest", "floor"])
@pytest.mark.parametrize("epi", ["plain", "residual", "gelu"])
def test_linear_requant_big_tiles_mixed_epilogue_forms(ivit, rounding, epi):
    """Long rows and more tiles than workgroups, so that epilogues run inside the next tile's k-loop; eight channels
    with a pair outside the 24-bit form make the wavefronts that own them take the 64-bit epilogue between two tiles
    while the others carry on; both rounding modes.  Every row against the tiled kernel, a sample against the oracle."""
    M, N, K = 17000, 512, 2304
    x = synth.make_rows(11, M, K, "normal", 32.0)
    w, bias, rq_b, rq_c = synth.make_linear(12, N, K)
    rq_b[64:72] = 2 ** 31 - 1; rq_c[64:72] = 44
    x[-1, -5:] = -128; w[3, :9] = -128
    kw_o, kw_g = {}, {}
    if epi == "residual":
        res = synth.make_rows(13, M, N, "uniform")
        kw_o = dict(residual=res, res_rq=(23456, 15)); kw_g = dict(residual=dev(res), res_rq=(23456, 15))
    elif epi == "gelu":
        kw_o = dict(gelu=synth.shift_params(32), gelu_rq=(24171, 21)); kw_g = dict(kw_o)
    ys = {}
    for kernel in ("big_tiles", "many_rows"):
        ys[kernel] = empty((M, N))
        ivit.ivit_linear_requant(dev(x), dev(w), dev(bias), dev(rq_b), dev(rq_c), ys[kernel], kernel=kernel, rounding=rounding, **kw_g)
    assert bool((ys["big_tiles"] == ys["many_rows"]).all())
    rows = np.unique(np.concatenate([np.arange(0, 260), np.arange(M - 260, M), np.arange(0, M, 211)]))
    kw_s = dict(kw_o)
    if epi == "residual":
        kw_s["residual"] = res[rows]
    want = orc.linear_requant(x[rows], w, bias, rq_b, rq_c, floor_shift=(rounding == "floor"), **kw_s)
    assert_same(host(ys["big_tiles"])[rows], want, "linear (big tiles, mixed forms) %s %s" % (epi, rounding))
    assert np.abs(want[:, 64:72].astype(np.int32)).max() > 0 and np.abs(want[:, :64].astype(np.int32)).mean() > 2


@pytest.mark.parametrize("M,N,K", RS_SHAPES)
@pytest.mark.parametrize("epi", ["plain", "residual", "gelu"])
def test_linear_requant_weights_in_registers(ivit, M, N, K, epi):
    if K == 192 and epi == "residual":
        with pytest.raises(ivit.IvitError) as err:
            ivit.ivit_linear_requant(empty((M, K)), empty((N, K)), None, dev(np.ones(N, np.int32)), dev(np.ones(N, np.int32)), empty((M, N)),
                                     residual=empty((M, N)), res_rq=(3, 1), kernel="reg_stationary")
        assert err.value.status == ivit.IVIT_ERR_SHAPE
        return
    x = synth.make_rows(M + N + K, M, K, "normal", 32.0)
    x[0, :7] = -128                                    # the ABI takes any int8
    w, bias, rq_b, rq_c = synth.make_linear(M * 7 + N, N, K)
    w[0, :5] = -128
    kw_o, kw_g = {}, {}
    if epi == "residual":
        res = synth.make_rows(N + 1, M, N, "uniform")
        res[-1, ::3] = -128
        kw_o = dict(residual=res, res_rq=(23456, 15)); kw_g = dict(residual=dev(res), res_rq=(23456, 15))
    elif epi == "gelu":
        kw_o = dict(gelu=synth.shift_params(32), gelu_rq=(24171, 21)); kw_g = dict(kw_o)
    y = empty((M, N))
    ivit.ivit_linear_requant(dev(x), dev(w), dev(bias), dev(rq_b), dev(rq_c), y, kernel="reg_stationary", **kw_g)
    assert_same(host(y), orc.linear_requant(x, w, bias, rq_b, rq_c, **kw_o), "linear (weights in registers) %s" % epi)


def test_linear_requant_weights_in_registers_general_pairs_and_refusals(ivit):
    """Pairs outside the 24-bit form (shifts up to 46, 31-bit multipliers, no bias) on the kernel that keeps the weights
    in registers: a workgroup with such a channel takes the 64-bit form for all of its channels.  Shapes the kernel
    does not take are refused."""
    rng = np.random.default_rng(7)
    M, N, K = 700, 448, 384
    x = synth.make_rows(1, M, K, "uniform")
    w = synth.make_rows(2, N, K, "uniform")
    rq_c = rng.integers(1, 47, size=N).astype(np.int32)
    rq_b = np.array([int(rng.integers(2 ** max(0, min(29, c - 13)), 2 ** max(1, min(31, c - 11)))) for c in rq_c], np.int32)
    rq_b[:8] = 2 ** 31 - 1; rq_c[:8] = 46
    res = synth.make_rows(3, M, N, "uniform")
    gl = dict(gelu=synth.shift_params(20), gelu_rq=(2 ** 31 - 1, 38))
    for kw_o, kw_g in (({}, {}), (dict(residual=res, res_rq=(2 ** 31 - 1, 31)), dict(residual=dev(res), res_rq=(2 ** 31 - 1, 31))),
                       (dict(residual=res, res_rq=(3, 1)), dict(residual=dev(res), res_rq=(3, 1))), (gl, gl)):
        y = empty((M, N))
        ivit.ivit_linear_requant(dev(x), dev(w), None, dev(rq_b), dev(rq_c), y, kernel="reg_stationary", **kw_g)
        want = orc.linear_requant(x, w, None, rq_b, rq_c, **kw_o)
        assert_same(host(y), want, "linear general (weights in registers)")
        assert np.abs(want.astype(np.int32)).mean() > 2
    for Mb, Nb, Kb in ((64, 64, 128), (64, 48, 384), (64, 1000, 768), (64, 48, 1536), (64, 64, 3072)):
        with pytest.raises(ivit.IvitError) as err:
            ivit.ivit_linear_requant(empty((Mb, Kb)), empty((Nb, Kb)), None, dev(rq_b[:1].repeat(Nb)), dev(rq_c[:1].repeat(Nb)),
                                     empty((Mb, Nb)), kernel="reg_stationary")
        assert err.value.status == ivit.IVIT_ERR_SHAPE


# ------------------------------------------------------------------ fused attention
ATT_CASES = [("c0_tiny", 2, None), ("c4_swin_t", 5, None), ("c2_deit_s", 2, None), ("c1_deit_t", 1, None),
             ("c0_tiny", 1, dict(T=1)), ("c2_deit_s", 1, dict(T=256)), ("c4_swin_t", 2, dict(T=16)),
             ("c2_deit_s", 1, dict(T=130))]


@pytest.mark.parametrize("name,B,over", ATT_CASES)
def test_attention(ivit, name, B, over):
    cfg = dict(synth.CONFIGS[name], **(over or {}))
    d = synth.dims_of(cfg, B)
    blk = synth.make_block(cfg, 0)
    qkv = synth.make_rows(B + cfg["T"], B * cfg["T"], 3 * cfg["C"], "normal", 32.0)
    qkv[0, :6] = -128; qkv[0, cfg["C"]:cfg["C"] + 6] = -128; qkv[-1, -6:] = -128; qkv[::7, 2 * cfg["C"] + 1] = -128   # -128 in Q, K and V
    o = empty((B * cfg["T"], cfg["C"]))
    sc = empty((B, cfg["H"], cfg["T"], cfg["T"])); pr = empty((B, cfg["H"], cfg["T"], cfg["T"]))
    rb = None if blk["rel_bias"] is None else dev(blk["rel_bias"])
    ivit.ivit_attention(dev(qkv), o, d, blk["qk_rq"], blk["softmax"], blk["pv_rq"], rel_bias=rb, tap_scores=sc, tap_probs=pr)
    o_ref, sc_ref, pr_ref = orc.attention(qkv, d, blk["qk_rq"], blk["softmax"], blk["pv_rq"], blk["rel_bias"], want_taps=True)
    assert_same(host(sc), sc_ref, "scores")
    assert_same(host(pr), pr_ref, "probs")
    assert_same(host(o), o_ref, "attention out")
    o2 = empty(o.shape)                     # without taps: same result
    ivit.ivit_attention(dev(qkv), o2, d, blk["qk_rq"], blk["softmax"], blk["pv_rq"], rel_bias=rb)
    assert_same(host(o2), o_ref, "attention out (no taps)")


@pytest.mark.parametrize("qk,pv", [
    ((1200000007, 38), (40000, 15)),            # beyond 32 bits: the general 64-bit requantisation
    ((4700011, 30), (9000001, 31)),             # c above 24: the 32-bit form
    ((2 ** 14 - 1, 15), (20011, 22)),           # b just below 2^(c-1) / an ordinary pair: the 24-bit form
    ((2 ** 14, 15), (20011, 22)),               # b = 2^(c-1): just outside the 24-bit form
    ((3, 24), (24001, 21)),                     # bounds of the 24-bit form beyond 24 bits (tiny multiplier)
    ((37, 10), (5, 4)),                         # small shifts
])
def test_attention_dyadic_pair_regimes(ivit, qk, pv, rounding):
    fs = rounding == "floor"
    cfg = synth.CONFIGS["c0_tiny"]
    d = synth.dims_of(cfg, 2)
    qkv = synth.make_rows(3, 2 * cfg["T"], 3 * cfg["C"], "normal", 50.0)
    qkv[:4] = 127; qkv[4:8] = -127              # saturating dot products on both sides
    sm = synth.shift_params(12)
    want, _, pr_ref = orc.attention(qkv, d, qk, sm, pv, want_taps=True, floor_shift=fs)
    o = empty((2 * cfg["T"], cfg["C"]))
    att = (lambda *a, **kw: ivit.ivit_window_attention(*a, None, None, rounding="floor", **kw)) if fs else ivit.ivit_attention
    att(dev(qkv), o, d, qk, sm, pv)
    assert_same(host(o), want, "attention, pair regime")
    pr = empty(pr_ref.shape)
    att(dev(qkv), o, d, qk, sm, pv, tap_probs=pr)
    assert_same(host(pr), pr_ref, "attention probabilities, pair regime")
    assert_same(host(o), want, "attention with taps, pair regime")


@pytest.mark.parametrize("name,B", [("c0_tiny", 2), ("c2_deit_s", 2), ("c4_swin_t", 5), ("c3_vit_b", 1)])
def test_attention_floor_mode(ivit, name, B):
    """Eq. 10 as a bare shift in both requantisations of the attention layer (scores, output), with and without taps."""
    cfg = synth.CONFIGS[name]
    d = synth.dims_of(cfg, B)
    blk = synth.make_block(cfg, 0)
    qkv = synth.make_rows(B + cfg["T"], B * cfg["T"], 3 * cfg["C"], "normal", 32.0)
    qkv[0, :6] = -128; qkv[-1, -6:] = -128
    rb = None if blk["rel_bias"] is None else dev(blk["rel_bias"])
    o_ref, sc_ref, pr_ref = orc.attention(qkv, d, blk["qk_rq"], blk["softmax"], blk["pv_rq"], blk["rel_bias"], want_taps=True,
                                          floor_shift=True)
    o = empty((B * cfg["T"], cfg["C"]))
    ivit.ivit_window_attention(dev(qkv), o, d, blk["qk_rq"], blk["softmax"], blk["pv_rq"], rb, None, rounding="floor")
    assert_same(host(o), o_ref, "attention out, floor")
    sc = empty(sc_ref.shape); pr = empty(pr_ref.shape); o2 = empty(o.shape)
    ivit.ivit_window_attention(dev(qkv), o2, d, blk["qk_rq"], blk["softmax"], blk["pv_rq"], rb, None, tap_scores=sc, tap_probs=pr,
                               rounding="floor")
    assert_same(host(sc), sc_ref, "scores, floor")
    assert_same(host(pr), pr_ref, "probs, floor")
    assert_same(host(o2), o_ref, "attention out with taps, floor")
    assert (o_ref != orc.attention(qkv, d, blk["qk_rq"], blk["softmax"], blk["pv_rq"], blk["rel_bias"])).mean() > 0.02
    o3 = empty(o.shape)
    ivit.ivit_window_attention(dev(qkv), o3, d, blk["qk_rq"], blk["softmax"], blk["pv_rq"], rb, None, rounding="nearest")
    assert_same(host(o3), orc.attention(qkv, d, blk["qk_rq"], blk["softmax"], blk["pv_rq"], blk["rel_bias"]), "nearest through the option")


# ------------------------------------------------------------------ encoder block with every intermediate tensor
def _gpu_block(ivit, x, p, d, want_taps):
    import torch
    R = d["B"] * d["T"]
    ws = torch.empty(ivit.ivit_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    y = empty((R, d["C"]))
    taps = None
    if want_taps:
        taps = {"u": empty((R, d["C"])), "qkv": empty((R, 3 * d["C"])),
                "scores": empty((d["B"], d["H"], d["T"], d["T"])), "probs": empty((d["B"], d["H"], d["T"], d["T"])),
                "o": empty((R, d["C"])), "xhat": empty((R, d["C"])), "v": empty((R, d["C"])), "h": empty((R, d["F"]))}
    pd = ivit.to_device(p)
    ivit.ivit_encoder_block(dev(x), y, pd, d, ws, taps=taps)
    return host(y), (None if taps is None else {k: host(v) for k, v in taps.items()})


@pytest.mark.parametrize("name,B,layer", [("c0_tiny", 1, 0), ("c0_tiny", 3, 0), ("c4_swin_t", 8, 0), ("c1_deit_t", 2, 0),
                                          ("c2_deit_s", 2, 0), ("c2_deit_s", 1, 5), ("c3_vit_b", 1, 0)])
def test_encoder_block_all_tensors(ivit, name, B, layer):
    cfg = synth.CONFIGS[name]
    d = synth.dims_of(cfg, B)
    p = synth.make_block(cfg, layer)
    x = synth.make_input(cfg, B)
    y, taps = _gpu_block(ivit, x, p, d, True)
    y_ref, t_ref = orc.encoder_block(x, p, d, want_taps=True)
    for k in orc.TAP_NAMES:
        assert_same(taps[k], t_ref[k], "%s tap %s" % (name, k))
    assert_same(y, y_ref, "%s block output" % name)
    y2, _ = _gpu_block(ivit, x, p, d, False)
    assert_same(y2, y_ref, "%s block output (no taps)" % name)


def test_encoder_block_empty_batch(ivit):
    import torch
    cfg = synth.CONFIGS["c0_tiny"]
    d = synth.dims_of(cfg, 0)
    ws = torch.empty(ivit.ivit_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    x = empty((16,)); y = empty((16,))
    ivit.ivit_encoder_block(x, y, ivit.to_device(synth.make_block(cfg, 0)), d, ws)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ forward
def _oracle_forward_images(cfg, x, blocks, images, final_ln=None):
    """Oracle forward of the chosen images, one image per call, images in parallel threads."""
    T = cfg["T"]
    d1 = synth.dims_of(cfg, 1)

    def one(i):
        return orc.forward(x[i * T:(i + 1) * T], blocks, d1, final_ln)
    with ThreadPoolExecutor(max_workers=8) as ex:
        return list(ex.map(one, images))


def _gpu_forward(ivit, cfg, x, blocks, B, final_ln=None):
    import torch
    d = synth.dims_of(cfg, B)
    ws = torch.empty(ivit.ivit_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    y = empty(x.shape)
    bl = [ivit.to_device(p) for p in blocks]
    fl = None if final_ln is None else ivit.to_device(final_ln)
    ivit.ivit_forward(dev(x), y, bl, d, ws, final_ln=fl)
    out = host(y)
    y2 = empty(x.shape)                     # integer kernels must be run-to-run identical
    ivit.ivit_forward(dev(x), y2, bl, d, ws, final_ln=fl)
    assert np.array_equal(out, host(y2)), "forward is not deterministic"
    return out


def test_forward_small_stack_with_final_layernorm(ivit):
    cfg = dict(synth.CONFIGS["c0_tiny"], L=3)
    B = 5
    blocks, fin = synth.make_model(cfg), synth.make_final_ln(cfg)
    x = synth.make_input(cfg, B)
    got = _gpu_forward(ivit, cfg, x, blocks, B, fin)
    assert_same(got, orc.forward(x, blocks, synth.dims_of(cfg, B), fin), "forward c0 x3 + LN")
    got0 = _gpu_forward(ivit, cfg, x, [], B, None)
    assert_same(got0, x, "forward with no blocks")


FULL = [("c1_deit_t", (0, 21, 63)), ("c2_deit_s", (0, 37, 90, 127)), ("c3_vit_b", (5, 255)),
        ("c4_swin_t", (0, 1, 63, 64, 4095, 8191))]


@pytest.mark.parametrize("name,images", FULL)
def test_forward_full_size_sampled_images(ivit, name, images):
    """The configuration at its full batch, as the benchmark runs it; sampled images against the oracle."""
    cfg = synth.CONFIGS[name]
    blocks = synth.make_model(cfg)
    x = synth.make_input(cfg)
    got = _gpu_forward(ivit, cfg, x, blocks, cfg["B"])
    want = _oracle_forward_images(cfg, x, blocks, images)
    T = cfg["T"]
    for i, w in zip(images, want):
        assert_same(got[i * T:(i + 1) * T], w, "%s image %d" % (name, i))
    assert np.abs(got.astype(np.int32)).mean() > 3


@pytest.mark.parametrize("name", ["c1_deit_t", "c2_deit_s", "c3_vit_b", "c4_swin_t"])
def test_forward_full_size_every_image_against_stored_oracle_digests(ivit, name):
    """Every image of the full batch: digests of the oracle's outputs, written by tests/golden/make_checksums.py
    (which calls only the oracle and the seeded generators), against digests of the library's output."""
    import hashlib
    import json
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "forward_checksums.json")
    ref = json.load(open(path))[name]
    cfg = synth.CONFIGS[name]
    assert (ref["images"], ref["tokens"], ref["dim"], ref["blocks"]) == (cfg["B"], cfg["T"], cfg["C"], cfg["L"])
    got = np.ascontiguousarray(_gpu_forward(ivit, cfg, synth.make_input(cfg), synth.make_model(cfg), cfg["B"]))
    step = cfg["T"] * ref["images_per_digest"]
    dig = [hashlib.sha256(got[i:i + step].tobytes()).hexdigest()[:16] for i in range(0, got.shape[0], step)]
    bad = [i for i, (a, b) in enumerate(zip(dig, ref["sha256_64"])) if a != b]
    assert len(dig) == len(ref["sha256_64"]) and not bad, "%s: %d of %d digests differ, first %s" % (name, len(bad), len(dig), bad[:5])


# ------------------------------------------------------------------ embedding layer, head, patches -> logits
@pytest.mark.parametrize("B,P,C,tq,pq", [(0, 4, 64, (2 ** 14, 14), (2 ** 13, 14)), (3, 0, 16, (23457, 15), (9001, 15)),
                                         (5, 196, 384, (23457, 15), (9001, 15)), (2, 64, 64, (2 ** 31 - 1, 33), (7, 1)),
                                         (129, 48, 96, (30000, 15), (3, 2))])
def test_embed_tokens(ivit, B, P, C, tq, pq):
    rng = np.random.default_rng(B + P + C)
    tok = rng.integers(-127, 128, size=(B * P, C)).astype(np.int8)
    cls = rng.integers(-127, 128, size=C).astype(np.int8)
    pos = rng.integers(-127, 128, size=(P + 1, C)).astype(np.int8)
    out = empty((B * (P + 1), C))
    ivit.ivit_embed_tokens(dev(tok), dev(cls), dev(pos), tq, pq, out, B, P)
    assert_same(host(out), orc.embed_tokens(tok, cls, pos, tq, pq, B), "embed_tokens")


@pytest.mark.parametrize("B,T,C,N", [(1, 1, 16, 1), (7, 65, 64, 10), (128, 197, 384, 1000), (33, 197, 768, 1000), (256, 5, 192, 21)])
def test_classifier_head(ivit, B, T, C, N):
    x = synth.make_rows(B + N, B * T, C, "normal", 32.0)
    w, bias, rq_b, rq_c = synth.make_linear(N + 3, N, C)
    out = empty((B, N))
    ivit.ivit_classifier_head(dev(x), T, dev(w), dev(bias), dev(rq_b), dev(rq_c), out)
    assert_same(host(out), orc.classifier_head(x, T, w, bias, rq_b, rq_c), "classifier head")


@pytest.mark.parametrize("name,B,L", [("c0_tiny", 1, 1), ("c0_tiny", 5, 1), ("c1_deit_t", 3, 2), ("c2_deit_s", 2, 12)])
def test_forward_image_patches_to_logits(ivit, name, B, L):
    import torch
    cfg = synth.CONFIGS[name]
    d = synth.dims_of(cfg, B)
    blocks = synth.make_model(cfg, L)
    image = synth.make_image_params(cfg)
    fl = synth.make_final_ln(cfg)
    patches = synth.make_patches(cfg, B)
    want = orc.forward_image(patches, image, blocks, d, fl)
    ws = torch.empty(ivit.ivit_image_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    logits = empty(want.shape)
    img_d = ivit.to_device(image); fl_d = ivit.to_device(fl); blk_d = [ivit.to_device(p) for p in blocks]
    ivit.ivit_forward_image(dev(patches), logits, img_d, blk_d, d, ws, fl_d)
    assert_same(host(logits), want, "logits %s" % name)
    assert np.abs(want.astype(np.int32)).mean() > 2 and len(np.unique(want.argmax(axis=1))) >= min(B, 2) - 1


def test_forward_under_hip_graph_capture_replays_identically(ivit):
    """ivit_forward allocates nothing and records no memset, so it can be captured; every replay, with eager work
    and synchronisations in between, must reproduce the eager (oracle-checked) result."""
    import torch
    cfg = synth.CONFIGS["c1_deit_t"]
    B = 4
    d = synth.dims_of(cfg, B)
    blocks = synth.make_model(cfg, 3)
    x = synth.make_input(cfg)[: B * cfg["T"]]
    want = orc.forward(x, blocks, d)
    blk_d = [ivit.to_device(p) for p in blocks]
    structs = [ivit.block_params(p) for p in blk_d]
    xd = dev(x); y_eager = empty(x.shape); y_graph = empty(x.shape)
    ws = torch.empty(ivit.ivit_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        ivit.ivit_forward(xd, y_eager, structs, d, ws, stream=s.cuda_stream)
    torch.cuda.synchronize()
    assert_same(host(y_eager), want, "eager forward")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        ivit.ivit_forward(xd, y_graph, structs, d, ws, stream=torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        y_graph.zero_()
        ws.random_(0, 255)                           # eager work between replays; the workspace holds no state
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert_same(host(y_graph), want, "graph replay %d" % rep)


# ------------------------------------------------------------------ shifted-window attention mask
@pytest.mark.parametrize("name,B,i0,with_bias", [("c4_swin_t", 64, 32, True), ("c4_swin_t", 130, 32, False), ("c4_swin_t", 64, 2, True),
                                                 ("c4_swin_t", 64, 5, True), ("c4_swin_t", 64, 6, False), ("c4_swin_t", 64, 11, True),
                                                 ("c4_swin_t", 64, 1000, True), ("c2_deit_s", 5, 32, False), ("c0_tiny", 3, 12, False)])
def test_attention_with_shift_mask(ivit, name, B, i0, with_bias):
    cfg = synth.CONFIGS[name]
    T = cfg["T"]
    d = synth.dims_of(cfg, B)
    blk = synth.make_block(cfg, 0)
    sm = synth.shift_params(i0)
    rng = np.random.default_rng(B + i0)
    if T == 49:
        mask = synth.make_shift_mask()
    else:                                            # any pattern is legal: three mask types, random, diagonal kept
        mask = (rng.random((3, T, T)) < 0.4).astype(np.int8)
        mask[:, np.arange(T), np.arange(T)] = 0
        mask[1, 7, :] = 1                            # a row with every key masked
    rb = blk["rel_bias"] if with_bias and blk["rel_bias"] is not None else None
    if with_bias and rb is None:
        rb = np.clip(np.rint(rng.standard_normal((cfg["H"], T, T)) * 40), -127, 127).astype(np.int8)
    qkv = synth.make_rows(B + T, B * T, 3 * cfg["C"], "normal", 32.0)
    want, sc_ref, pr_ref = orc.attention(qkv, d, blk["qk_rq"], sm, blk["pv_rq"], rb, want_taps=True, mask=mask)
    o = empty((B * T, cfg["C"])); pr = empty((B, cfg["H"], T, T))
    ivit.ivit_attention(dev(qkv), o, d, blk["qk_rq"], sm, blk["pv_rq"], rel_bias=None if rb is None else dev(rb), mask=dev(mask), tap_probs=pr)
    assert_same(host(pr), pr_ref, "masked probs")
    assert_same(host(o), want, "masked attention")
    o2 = empty(o.shape)
    ivit.ivit_attention(dev(qkv), o2, d, blk["qk_rq"], sm, blk["pv_rq"], rel_bias=None if rb is None else dev(rb), mask=dev(mask))
    assert_same(host(o2), want, "masked attention (no taps)")


def test_encoder_block_with_shift_mask(ivit):
    cfg = synth.CONFIGS["c4_swin_t"]
    B = 128
    d = synth.dims_of(cfg, B)
    p = dict(synth.make_block(cfg, 0), attn_mask=synth.make_shift_mask())
    x = synth.make_input(cfg)[: B * cfg["T"]]
    y_ref, t_ref = orc.encoder_block(x, p, d, want_taps=True)
    y, taps = _gpu_block(ivit, x, p, d, True)
    for k in orc.TAP_NAMES:
        assert_same(taps[k], t_ref[k], "masked block tensor " + k)
    assert_same(y, y_ref, "masked block output")
    y_plain, _ = orc.encoder_block(x, synth.make_block(cfg, 0), d, want_taps=True)
    assert not np.array_equal(y_plain, y_ref)


# ------------------------------------------------------------------ windowed models: gathered windows, merging, pooling, forward
def _oracle_window_attention(qkv, B, g, w, s, C, H, blk, sm, rel_bias):
    """The definition: roll the image-order tensor, cut it into windows, attend, put the windows back, roll back."""
    q = qkv.reshape(B, g, g, 3 * C)
    if s:
        q = np.roll(q, (-s, -s), axis=(1, 2))
    qw = orc.window_partition(q, w)
    d = dict(B=qw.shape[0], T=w * w, C=C, H=H, F=4 * C)
    o, sc, pr = orc.attention(qw.reshape(-1, 3 * C), d, blk["qk_rq"], sm, blk["pv_rq"], rel_bias, want_taps=True,
                              mask=orc.shift_mask(g, w, s) if s else None)
    oi = orc.window_reverse(o.reshape(-1, w * w, C), w, g)
    if s:
        oi = np.roll(oi, (s, s), axis=(1, 2))
    return oi.reshape(-1, C), pr, d


@pytest.mark.parametrize("B,g,w,s,C,H", [(3, 56, 7, 3, 96, 3), (2, 56, 7, 0, 96, 3), (5, 28, 7, 3, 192, 6), (9, 14, 7, 3, 384, 12),
                                         (2, 16, 4, 2, 64, 1), (1, 12, 3, 1, 64, 2), (4, 7, 7, 0, 768, 24)])
def test_window_attention_on_image_order_tokens(ivit, B, g, w, s, C, H):
    T = w * w
    blk = synth.make_block(dict(T=T, C=C, H=H, F=4 * C, seed=40 + g, i0="fixed", rel_bias=True), 0)
    sm = synth.shift_params(32)
    qkv = synth.make_rows(B * g + s, B * g * g, 3 * C, "normal", 32.0)
    want, pr_ref, d = _oracle_window_attention(qkv, B, g, w, s, C, H, blk, sm, blk["rel_bias"])
    idx = dev(ivit.ivit_swin_window_index(g, w, s))
    mask = dev(ivit.ivit_swin_shift_mask(g, w, s)) if s else None
    o = empty((B * g * g, C)); pr = empty((d["B"], H, T, T))
    ivit.ivit_window_attention(dev(qkv), o, d, blk["qk_rq"], sm, blk["pv_rq"], dev(blk["rel_bias"]), idx, mask=mask, tap_probs=pr)
    assert_same(host(pr), pr_ref, "window attention probabilities")
    assert_same(host(o), want, "window attention output (image order)")
    o2 = empty(o.shape)
    ivit.ivit_window_attention(dev(qkv), o2, d, blk["qk_rq"], sm, blk["pv_rq"], dev(blk["rel_bias"]), idx, mask=mask)
    assert_same(host(o2), want, "window attention output (no taps)")


def test_window_attention_clamps_table_entries_outside_the_image(ivit):
    """An entry beyond the image reads (and writes) the image's last row instead of faulting."""
    B, g, w, C, H = 2, 8, 4, 64, 2
    T, n_win = w * w, 4
    blk = synth.make_block(dict(T=T, C=C, H=H, F=4 * C, seed=77, i0="fixed", rel_bias=True), 0)
    sm = synth.shift_params(32)
    qkv = synth.make_rows(5, B * g * g, 3 * C, "normal", 32.0)
    idx = ivit.ivit_swin_window_index(g, w, 0)
    orphan = int(idx[0, 5])
    bad = idx.copy(); bad[0, 5] = 10 ** 9
    clamped = idx.copy(); clamped[0, 5] = g * g - 1
    rows = (np.arange(B)[:, None, None] * g * g + clamped[None]).reshape(-1)
    d = dict(B=B * n_win, T=T, C=C, H=H, F=4 * C)
    ow = orc.attention(qkv[rows], d, blk["qk_rq"], sm, blk["pv_rq"], blk["rel_bias"])
    o = empty((B * g * g, C)); o.fill_(-128)
    ivit.ivit_window_attention(dev(qkv), o, d, blk["qk_rq"], sm, blk["pv_rq"], dev(blk["rel_bias"]), dev(bad))
    got = host(o)
    for b in range(B):
        assert (got[b * g * g + orphan] == -128).all()          # no window owns this row any more
    check = np.ones(B * n_win * T, bool)
    for b in range(B):                                          # the last row of each image has two writers
        check[(rows == b * g * g + g * g - 1)] = False
    assert_same(got[rows[check]], ow[check], "rows with one writer")


@pytest.mark.parametrize("B,g,w,s,C,H,layer", [(2, 56, 7, 3, 96, 3, 1), (2, 28, 7, 0, 192, 6, 0), (3, 14, 7, 3, 384, 12, 1), (2, 8, 4, 2, 32, 1, 1)])
def test_swin_block_all_tensors(ivit, B, g, w, s, C, H, layer):
    """The block on image-order tokens with the library's index table and mask, every tensor: row-wise tensors against
    the oracle's block, scores and probabilities (window-major) against the oracle's attention on explicit windows."""
    T, n_win = w * w, (g // w) ** 2
    p = synth.make_block(dict(T=T, C=C, H=H, F=4 * C, seed=50 + g, i0="fixed", rel_bias=True), layer)
    x = synth.quantize_act(np.random.default_rng(g + s).standard_normal((B * g * g, C)))
    y_ref = orc.swin_block(x.reshape(B, g, g, C), p, g, w, s, H).reshape(-1, C)
    q = dict(p, tok_index=ivit.ivit_swin_window_index(g, w, s))
    if s:
        q["attn_mask"] = ivit.ivit_swin_shift_mask(g, w, s)
    d = dict(B=B * n_win, T=T, C=C, H=H, F=4 * C)
    y, taps = _gpu_block(ivit, x, q, d, True)
    assert_same(y, y_ref, "swin block output")
    u = orc.ilayernorm(x, p["ln1_gamma"], p["ln1_beta"], p["ln1_f_bits"], p["ln1_c_shift"])
    assert_same(taps["u"], u, "u")
    qkv = orc.linear_requant(u, p["w_qkv"], p["bias_qkv"], p["qkv_rq_b"], p["qkv_rq_c"])
    assert_same(taps["qkv"], qkv, "qkv (image order)")
    o_ref, pr_ref, _ = _oracle_window_attention(qkv, B, g, w, s, C, H, p, p["softmax"], p["rel_bias"])
    assert_same(taps["probs"], pr_ref, "probs (window major)")
    assert_same(taps["o"], o_ref, "o (image order)")
    y2, _ = _gpu_block(ivit, x, q, d, False)
    assert_same(y2, y_ref, "swin block output (no taps)")


@pytest.mark.parametrize("B,g,C", [(0, 8, 32), (1, 2, 16), (3, 56, 96), (2, 28, 192), (5, 14, 384), (2, 6, 48)])
def test_patch_merge_gather(ivit, B, g, C):
    x = synth.make_rows(B + g, B * g * g, C, "uniform").reshape(B, g, g, C)
    want = np.concatenate([x[:, 0::2, 0::2], x[:, 1::2, 0::2], x[:, 0::2, 1::2], x[:, 1::2, 1::2]], axis=-1)
    y = empty((B, g // 2, g // 2, 4 * C))
    ivit.ivit_patch_merge_gather(dev(x), y, B, g, C)
    assert_same(host(y), want, "patch merging concatenation")


@pytest.mark.parametrize("B,T,C,rq", [(0, 49, 64, (21400, 20)), (1, 1, 4, (2 ** 14, 14)), (128, 49, 768, (21400, 20)),
                                      (7, 16, 128, (2 ** 16, 20)), (3, 197, 384, (2 ** 30 + 12345, 37)), (5, 49, 96, (2 ** 20, 20))])
def test_mean_pool(ivit, B, T, C, rq):
    x = synth.make_rows(B + T, B * T, C, "normal", 50.0).reshape(B, T, C)
    y = empty((B, C))
    ivit.ivit_mean_pool(dev(x), y, B, T, C, rq)
    assert_same(host(y), orc.mean_pool(x, rq) if B else np.empty((0, C), np.int8), "mean pool")


def _gpu_swin(ivit, cfg, model, patches, B):
    import torch
    m = ivit.swin_to_device(model)
    sp, keep = ivit.swin_params(m)
    ws = torch.empty(ivit.ivit_swin_workspace_bytes(sp, B), dtype=torch.uint8, device="cuda")
    logits = empty((B, cfg["n_classes"]))
    ivit.ivit_forward_swin(dev(patches), logits, sp, B, ws)
    return host(logits)


@pytest.mark.parametrize("name,B", [("swin_tiny_test", 2), ("swin_tiny_test", 7), ("swin_t", 2), ("swin_s", 1)])
def test_forward_swin_patches_to_logits(ivit, name, B):
    cfg = synth.SWIN[name]
    model = synth.make_swin_model(cfg)
    patches = synth.make_swin_patches(cfg, B)
    want = orc.swin_forward(patches, model)
    assert want.std() > 5
    assert_same(_gpu_swin(ivit, cfg, model, patches, B), want, "%s logits" % name)


def test_forward_swin_full_size_every_image_against_stored_oracle_digests(ivit):
    """Swin-T shape, 128 images (the shape the benchmark times): digests of the oracle's logits per image, written by
    tests/golden/make_checksums.py, against digests of the library's logits."""
    import hashlib
    import json
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "forward_checksums.json")
    ref = json.load(open(path))["swin_t"]
    cfg = synth.SWIN["swin_t"]
    assert (ref["images"], ref["n_classes"]) == (cfg["B"], cfg["n_classes"])
    got = np.ascontiguousarray(_gpu_swin(ivit, cfg, synth.make_swin_model(cfg), synth.make_swin_patches(cfg), cfg["B"]))
    dig = [hashlib.sha256(got[i].tobytes()).hexdigest()[:16] for i in range(cfg["B"])]
    bad = [i for i, (a, b) in enumerate(zip(dig, ref["sha256_64"])) if a != b]
    assert len(dig) == len(ref["sha256_64"]) and not bad, "swin_t: %d of %d digests differ, first %s" % (len(bad), len(dig), bad[:5])
