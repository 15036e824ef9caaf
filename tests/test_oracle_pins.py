"""Pins of the CPU oracle against things other than itself: closed forms, library
routines, brute force on tiny inputs, invariants and worked examples.  CPU only."""
import math
import os

import numpy as np
import pytest
import scipy.integrate
import scipy.special

import synth_inputs as si
from oracle import qp_oracle as orc

BITS = (2, 3, 4, 6, 8, 16)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- statistics

def test_stats_constant_tensor():
    rc, st = orc.stats(np.full(1000, 1.25, np.float32))
    assert rc == 0
    assert st.mean == 1.25 and st.mad == 0.0 and st.var == 0.0
    assert st.min == 1.25 and st.max == 1.25 and st.abs_mean == 1.25
    assert st.b_r == 0.0 and st.peak_count == 1000


@pytest.mark.parametrize("n", [2, 10, 4096, 100000])
def test_stats_ramp_closed_form(n):
    # x_i = i, i = 0..n-1, n even: mean (n-1)/2, population variance (n^2-1)/12, MAD n/4.
    rc, st = orc.stats(np.arange(n, dtype=np.float32))
    assert rc == 0
    assert st.mean == pytest.approx((n - 1) / 2, rel=1e-14)
    assert st.var == pytest.approx((n * n - 1) / 12, rel=1e-13)
    assert st.mad == pytest.approx(n / 4, rel=1e-14)
    assert st.min == 0.0 and st.max == n - 1
    assert st.abs_mean == pytest.approx((n - 1) / 2, rel=1e-14)


def test_stats_two_point():
    rc, st = orc.stats(np.tile(np.array([-3.0, 3.0], np.float32), 500))
    assert rc == 0
    assert st.mean == 0.0 and st.mad == 3.0 and st.var == 9.0 and st.abs_mean == 3.0


def test_stats_shifted_two_point_mad_about_mean():
    # MAD is about the mean, abs_mean is not: values {1, 5} -> mean 3, MAD 2, abs_mean 3.
    rc, st = orc.stats(np.tile(np.array([1.0, 5.0], np.float32), 100))
    assert (st.mean, st.mad, st.abs_mean, st.var) == (3.0, 2.0, 3.0, 4.0)


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_stats_against_numpy_float64(name):
    x = si.make_config(name, n=200_000)
    rc, st = orc.stats(x)
    assert rc == 0
    x64 = x.astype(np.float64)
    mu = x64.mean()
    assert st.mean == pytest.approx(mu, rel=1e-12, abs=1e-15)
    assert st.mad == pytest.approx(np.abs(x64 - mu).mean(), rel=1e-12)
    assert st.abs_mean == pytest.approx(np.abs(x64).mean(), rel=1e-12)
    assert st.var == pytest.approx(x64.var(), rel=1e-12)
    assert st.min == float(x.min()) and st.max == float(x.max())
    assert st.n == x.size and st.n_nonfinite == 0


def test_stats_statistical_laplace_and_gauss():
    rng = np.random.default_rng(11)
    n = 1_000_000
    b = 0.7
    rc, st = orc.stats(rng.laplace(0.3, b, n).astype(np.float32))
    assert st.mad == pytest.approx(b, rel=5e-3)            # E|x-mu| = b
    assert st.var == pytest.approx(2 * b * b, rel=1e-2)    # Var = 2 b^2
    assert st.b_r == pytest.approx(b, rel=0.1)             # pdf peak 1/(2b)
    sigma = 1.3
    rc, st = orc.stats(rng.normal(-0.2, sigma, n).astype(np.float32))
    assert st.mad == pytest.approx(sigma * math.sqrt(2 / math.pi), rel=5e-3)
    assert st.var == pytest.approx(sigma * sigma, rel=5e-3)


def test_stats_nonfinite_is_reported():
    x = np.ones(100, np.float32)
    x[7] = np.nan
    x[9] = np.inf
    rc, st = orc.stats(x)
    assert rc == 1 and st.n_nonfinite == 2


def test_stats_bf16_widening_is_exact():
    h = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x8000, 0x7F7F], np.uint16)
    w = orc.widen_bf16(h)
    assert w[0] == 1.0 and w[1] == -1.0 and w[2] == np.float32(3.140625) and w[3] == 0.0
    assert np.array_equal(w, si.bf16_bits_to_f32(h))
    # rounding a float32 to bf16 and widening again never moves it by more than 2^-8 relative
    x = si.laplace_outliers(5000, 3)
    back = orc.widen_bf16(si.f32_to_bf16_bits(x))
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)


# ----------------------------------------------------------------------------- histogram / b_R

@pytest.mark.parametrize("nbins", [16, 256, 2048])
def test_histogram_matches_numpy_on_dyadic_grid(nbins):
    # values k/8 in [0, 256]: (x - min) * nbins/(max-min) is exact in fp32 and in fp64,
    # so fp32 binning cannot differ from numpy's fp64 binning.
    rng = np.random.default_rng(5)
    x = (rng.integers(0, 2049, size=50_000) / 8.0).astype(np.float32)
    x[0], x[1] = 0.0, 256.0
    rc, st, hist = orc.stats(x, nbins=nbins, want_hist=True)
    ref, _ = np.histogram(x.astype(np.float64), bins=nbins, range=(0.0, 256.0))
    assert np.array_equal(hist[:nbins], ref.astype(np.uint32))
    assert st.peak_count == ref.max()
    binw = 256.0 / nbins
    assert st.peak_density == pytest.approx(ref.max() / (x.size * binw), rel=1e-14)
    assert st.b_r == pytest.approx(1.0 / (2.0 * st.peak_density), rel=1e-15)
    assert int(hist.sum()) == x.size


def test_histogram_counts_everything_and_max_lands_in_last_bin():
    x = si.make_config("C2", n=100_000)
    rc, st, hist = orc.stats(x, want_hist=True)
    assert int(hist.sum()) == x.size
    assert hist[2047] >= 1 and hist[0] >= 1
    ref, _ = np.histogram(x.astype(np.float64), bins=2048, range=(float(x.min()), float(x.max())))
    # fp32 vs fp64 bin edges can move a handful of elements by one bin, never more
    assert np.abs(hist.astype(np.int64) - ref).sum() <= 2 * 50


# ----------------------------------------------------------------------------- ACIQ constants

def _golden_laplace():
    rows = []
    with open(os.path.join(GOLDEN, "aciq_laplace_constants.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                b, v = line.split()
                rows.append((int(b), float(v)))
    return rows


def test_laplace_constants_match_values_printed_in_cited_aciq_paper():
    for bits, printed in _golden_laplace():
        # printed with two decimals (3.8972 appears as 3.89): agree to within one unit of the last digit
        assert abs(orc.laplace_F(bits) - printed) < 0.0075


@pytest.mark.parametrize("bits", BITS)
def test_laplace_constant_is_lambert_w(bits):
    ref = scipy.special.lambertw(3.0 * 4.0 ** bits).real
    assert orc.laplace_F(bits) == pytest.approx(ref, rel=1e-14)
    w = orc.laplace_F(bits)
    assert w * math.exp(w) == pytest.approx(3.0 * 4.0 ** bits, rel=1e-12)


@pytest.mark.parametrize("z", [1e-6, 0.1, 1.0, math.e, 48.0, 1e5, 1e12])
def test_lambert_w_general(z):
    assert orc.lambert_w0(z) == pytest.approx(scipy.special.lambertw(z).real, rel=1e-13)


@pytest.mark.parametrize("bits", [2, 3, 4, 6, 8])
def test_laplace_constant_minimises_numerically_integrated_noise(bits):
    # clipping noise by quadrature of the unit Laplace density (not the closed form),
    # rounding noise of a uniform grid with 2^q cells over [-a, a]: (2a/2^q)^2 / 12.
    def noise(a):
        clip = 2.0 * scipy.integrate.quad(lambda x: (x - a) ** 2 * 0.5 * math.exp(-x), a, np.inf)[0]
        return clip + (2.0 * a / 2 ** bits) ** 2 / 12.0
    grid = np.arange(0.5, 14.0, 1e-3)
    a_best = grid[np.argmin([noise(a) for a in grid])]
    assert orc.laplace_F(bits) == pytest.approx(a_best, abs=2e-3)


@pytest.mark.parametrize("bits", [2, 3, 4, 6, 8])
def test_gauss_constant_minimises_numerically_integrated_noise(bits):
    phi = lambda x: math.exp(-0.5 * x * x) / math.sqrt(2 * math.pi)
    def noise(a):
        clip = 2.0 * scipy.integrate.quad(lambda x: (x - a) ** 2 * phi(x), a, np.inf)[0]
        return clip + (2.0 * a / 2 ** bits) ** 2 / 12.0
    grid = np.arange(0.5, 6.0, 1e-3)
    a_best = grid[np.argmin([noise(a) for a in grid])]
    assert orc.gauss_G(bits) == pytest.approx(a_best, abs=2e-3)


def test_gauss_constant_satisfies_stationarity_at_16_bits():
    a = orc.gauss_G(16)
    q = 0.5 * scipy.special.erfc(a / math.sqrt(2))
    phi = math.exp(-0.5 * a * a) / math.sqrt(2 * math.pi)
    assert phi - a * q == pytest.approx(a / (6 * 4.0 ** 16), rel=1e-9)


def test_aciq_alpha_is_constant_times_scale():
    x = si.make_config("C1")
    rc, st = orc.stats(x)
    for bits in BITS:
        assert orc.aciq_alpha(st, bits) == pytest.approx(scipy.special.lambertw(3 * 4.0 ** bits).real * st.mad, rel=1e-13)
        assert orc.aciq_alpha(st, bits, orc.GAUSS) == pytest.approx(orc.gauss_G(bits) * math.sqrt(st.var), rel=1e-15)
    with pytest.raises(ValueError):
        orc.aciq_alpha(st, 5)


# ----------------------------------------------------------------------------- quantization grid

@pytest.mark.parametrize("bits", BITS)
def test_qparams_grid(bits):
    q = orc.make_qparams(0.25, 3.0, bits, 10)
    L = 2 ** bits - 1
    assert q.levels == L and q.lo == np.float32(-2.75) and q.hi == np.float32(3.25)
    assert q.scale == np.float32(6.0 / L) and q.inv_scale == np.float32(L / 6.0)
    q0 = orc.make_qparams(1.0, 0.0, bits, 10)
    assert q0.lo == q0.hi == 1.0 and q0.scale == 0.0 and q0.inv_scale == 0.0


def test_quantize_8bit_identity_and_round_half_even():
    q = orc.make_qparams(127.5, 127.5, 8, 256)
    assert (q.lo, q.hi, q.scale, q.inv_scale) == (0.0, 255.0, 1.0, 1.0)
    x = np.arange(256, dtype=np.float32)
    assert np.array_equal(orc.quantize(x, q), np.arange(256, dtype=np.uint32))
    assert np.array_equal(orc.dequantize(np.arange(256), q), x)
    halves = np.array([0.5, 1.5, 2.5, 3.5, 254.5, 0.49999997, 0.50000006], np.float32)
    assert list(orc.quantize(halves, q)) == [0, 2, 2, 4, 254, 0, 1]


@pytest.mark.parametrize("bits", BITS)
def test_quantize_invariants(bits):
    x = si.make_config("C2", n=60_000)
    rc, st = orc.stats(x)
    q = orc.make_qparams(st.mean, orc.aciq_alpha(st, bits), bits, x.size)
    codes = orc.quantize(x, q)
    L = 2 ** bits - 1
    assert codes.max() <= L and codes.min() >= 0
    assert np.all(codes[x <= q.lo] == 0) and np.all(codes[x >= q.hi] == L)
    assert (x <= q.lo).any() and (x >= q.hi).any() or bits == 16
    # monotone
    order = np.argsort(x, kind="stable")
    assert np.all(np.diff(codes[order].astype(np.int64)) >= 0)
    # in-range error at most half a step (plus rounding slack of the fp32 products)
    y = orc.dequantize(codes, q)
    inside = (x >= q.lo) & (x <= q.hi)
    err = np.abs(x[inside].astype(np.float64) - y[inside].astype(np.float64))
    slack = (2.0 ** -22) * max(abs(q.lo), abs(q.hi)) + q.scale * 2.0 ** -7
    assert err.max() <= q.scale / 2 + slack
    # outside the range the value is clamped to an end point
    assert np.all(y[x <= q.lo] == np.float32(q.lo))
    assert np.all(np.abs(y[x >= q.hi].astype(np.float64) - q.hi) <= 4 * np.spacing(np.float32(abs(q.hi))))


def test_quantize_nan_and_inf():
    q = orc.make_qparams(0.0, 1.0, 4, 3)
    codes = orc.quantize(np.array([np.nan, np.inf, -np.inf], np.float32), q)
    assert list(codes) == [0, 15, 0]


def test_quantize_degenerate_range_gives_zero_codes():
    q = orc.make_qparams(1.25, 0.0, 4, 5)
    x = np.array([1.25, 0.0, 9.0, -3.0, 1.25], np.float32)
    assert np.all(orc.quantize(x, q) == 0)
    assert np.all(orc.dequantize(np.zeros(5, np.uint32), q) == np.float32(1.25))


@pytest.mark.parametrize("bits", BITS)
def test_quantize_matches_independent_numpy_statement(bits):
    x = si.make_config("C3", n=50_000)
    rc, st = orc.stats(x)
    q = orc.make_qparams(st.mean, orc.aciq_alpha(st, bits), bits, x.size)
    lo, hi, inv = np.float32(q.lo), np.float32(q.hi), np.float32(q.inv_scale)
    t = (np.minimum(np.maximum(x, lo), hi) - lo) * inv
    assert t.dtype == np.float32
    ref = np.clip(np.rint(t), 0, 2 ** bits - 1).astype(np.uint32)
    assert np.array_equal(orc.quantize(x, q), ref)


# ----------------------------------------------------------------------------- dequantize

@pytest.mark.parametrize("bits", BITS)
def test_dequant_is_fp64_definition_rounded_once(bits):
    q = orc.make_qparams(0.137, 2.9, bits, 1)
    L = 2 ** bits - 1
    codes = np.unique(np.concatenate([np.arange(0, min(L, 4096) + 1), np.linspace(0, L, 999).astype(np.int64)]))
    y = orc.dequantize(codes.astype(np.uint32), q)
    exact = np.float64(q.lo) + codes.astype(np.float64) * np.float64(q.scale)   # exact in fp64 here
    ref = exact.astype(np.float32)
    ulp = np.spacing(np.abs(ref))
    assert np.all(np.abs(y.astype(np.float64) - ref.astype(np.float64)) <= ulp)
    # the product c*scale has at most 40 significant bits and exponents are close, so the
    # fp64 sum is exact and a single rounding must reproduce fmaf bit for bit
    assert np.array_equal(y, ref)
    assert y[0] == np.float32(q.lo)


# ----------------------------------------------------------------------------- wire format

def _numpy_pack(codes, bits):
    bitsarr = ((codes[:, None].astype(np.uint64) >> np.arange(bits, dtype=np.uint64)) & 1).astype(np.uint8).reshape(-1)
    by = np.packbits(bitsarr, bitorder="little")
    total = 4 * ((codes.size * bits + 31) // 32)
    return np.concatenate([by, np.zeros(total - by.size, np.uint8)])


def test_pack_hand_worked_example():
    with open(os.path.join(GOLDEN, "pack_example_k3.txt")) as f:
        line = [l for l in f if l.strip() and not l.startswith("#")][0]
    bits, codes, hexbytes = [s.strip() for s in line.split("|")]
    out = orc.pack(np.array([int(c) for c in codes.split()], np.uint32), int(bits))
    assert list(out) == [int(h, 16) for h in hexbytes.split()]


@pytest.mark.parametrize("bits", BITS)
def test_pack_matches_numpy_packbits_and_round_trips(bits):
    rng = np.random.default_rng(bits)
    for n in list(range(0, 70)) + [255, 256, 257, 1000, 4099]:
        codes = rng.integers(0, 2 ** bits, size=n, dtype=np.uint32)
        out = orc.pack(codes, bits)
        assert out.size == 4 * ((n * bits + 31) // 32) == orc.packed_bytes(n, bits)
        assert np.array_equal(out, _numpy_pack(codes, bits))
        assert np.array_equal(orc.unpack(out, n, bits), codes)


def test_pack_special_cases_are_plain_arrays():
    rng = np.random.default_rng(0)
    c8 = rng.integers(0, 256, size=64, dtype=np.uint32)
    assert np.array_equal(orc.pack(c8, 8), c8.astype(np.uint8))
    c16 = rng.integers(0, 65536, size=64, dtype=np.uint32)
    assert np.array_equal(orc.pack(c16, 16).view("<u2"), c16.astype(np.uint16))
    c4 = rng.integers(0, 16, size=64, dtype=np.uint32)
    assert np.array_equal(orc.pack(c4, 4), (c4[0::2] | (c4[1::2] << 4)).astype(np.uint8))
    c2 = rng.integers(0, 4, size=64, dtype=np.uint32)
    assert np.array_equal(orc.pack(c2, 2), (c2[0::4] | (c2[1::4] << 2) | (c2[2::4] << 4) | (c2[3::4] << 6)).astype(np.uint8))


def test_packed_size_is_n_q_over_8_so_8bit_is_4x():
    # Sec. 3: 8-bit quantization compresses fp32 activations four times.
    n = si.numel("C2")
    assert orc.packed_bytes(n, 8) * 4 == n * 4
    for bits in BITS:
        assert orc.packed_bytes(n, bits) == n * bits // 8
    assert orc.packed_bytes(10, 5) == 0


# ----------------------------------------------------------------------------- directed search

def _numpy_scores(x, mean, b_e, b_r, bits, t):
    """Independent sweep: every candidate scored with numpy float32/float64 operations."""
    F = scipy.special.lambertw(3.0 * 4.0 ** bits).real
    L = 2 ** bits - 1
    scores = []
    alphas = []
    for j in range(t + 1):
        b = b_e + j * ((b_r - b_e) / t)
        a32 = np.float32(F * b)
        c32 = np.float32(mean)
        lo = np.float32(np.float64(c32) - np.float64(a32))
        hi = np.float32(np.float64(c32) + np.float64(a32))
        rng_ = np.float64(hi) - np.float64(lo)
        scale = np.float32(rng_ / L)
        inv = np.float32(L / rng_)
        tq = (np.minimum(np.maximum(x, lo), hi) - lo) * inv
        r = np.clip(np.rint(tq), 0, L)
        xh = (np.float64(lo) + r.astype(np.float64) * np.float64(scale)).astype(np.float32)
        e = (x - xh).astype(np.float64)
        scores.append(float(np.sum(e * e)))
        alphas.append(F * b)
    return np.array(scores), np.array(alphas)


@pytest.mark.parametrize("name,bits", [("C1", 2), ("C1", 4), ("C2", 3), ("C3", 2), ("C3", 4), ("C3", 8), ("C2", 16)])
def test_search_matches_brute_force_numpy_sweep(name, bits):
    x = si.make_config(name, n=4096)
    rc, st = orc.stats(x)
    res, q, scores = orc.dsaciq_search(x, st, bits, 100)
    ref, alphas = _numpy_scores(x, st.mean, st.mad, st.b_r, bits, 100)
    assert np.allclose(scores, ref, rtol=1e-6, atol=0)
    j_ref = int(np.argmin(ref))
    if res.j_star != j_ref:     # only a numerical near-tie may differ
        assert abs(ref[res.j_star] - ref[j_ref]) <= 1e-6 * ref[j_ref]
    assert res.alpha_star == pytest.approx(alphas[res.j_star], rel=1e-13)
    assert res.mse_star == pytest.approx(scores[res.j_star] / x.size, rel=1e-15)
    assert res.mse_aciq == pytest.approx(scores[0] / x.size, rel=1e-15)
    assert res.j_star == int(np.argmin(scores))          # first minimum
    assert res.mse_star <= res.mse_aciq
    lo_b, hi_b = sorted((st.mad, st.b_r))
    assert lo_b <= res.b_star <= hi_b
    assert (q.lo, q.hi) == (orc.make_qparams(st.mean, res.alpha_star, bits, x.size).lo,
                            orc.make_qparams(st.mean, res.alpha_star, bits, x.size).hi)


def test_search_scores_equal_sq_error_of_each_candidate():
    x = si.make_config("C3", n=3000)
    rc, st = orc.stats(x)
    res, q, scores = orc.dsaciq_search(x, st, 4, 20)
    F = orc.laplace_F(4)
    for j in (0, 7, 20):
        b = st.mad + j * ((st.b_r - st.mad) / 20)
        qj = orc.make_qparams(st.mean, F * b, 4, x.size)
        codes = orc.quantize(x, qj)
        y = orc.dequantize(orc.unpack(orc.pack(codes, 4), x.size, 4), qj)   # through the wire format
        e = (x - y).astype(np.float64)
        assert scores[j] == pytest.approx(float(np.sum(e * e)), rel=1e-13)


def test_search_degenerate_inputs_keep_b_e():
    x = np.full(500, 2.0, np.float32)
    rc, st = orc.stats(x)
    res, q, scores = orc.dsaciq_search(x, st, 4, 100)
    assert res.j_star == 0 and res.b_star == 0.0 and np.all(scores == scores[0])
    x = si.laplace_outliers(2000, 1)
    rc, st = orc.stats(x)
    st.b_r = float("inf")
    res, q, scores = orc.dsaciq_search(x, st, 4, 100)
    assert res.j_star == 0 and res.b_star == st.mad and np.all(scores == scores[0])
    st.b_r = st.mad
    res, q, scores = orc.dsaciq_search(x, st, 2, 100)
    assert res.j_star == 0


def test_search_helps_on_skewed_data_and_not_on_true_laplace():
    # Sec. 3: the search pays off when the Laplace estimate is far from the real
    # distribution (one-sided post-GELU data) and keeps b_E or a near neighbour otherwise.
    x = si.make_config("C3", n=100_000)
    rc, st = orc.stats(x)
    res, _, _ = orc.dsaciq_search(x, st, 4, 100)
    assert res.j_star > 0 and res.mse_star < 0.9 * res.mse_aciq
    x = np.random.default_rng(3).laplace(0, 0.5, 100_000).astype(np.float32)
    rc, st = orc.stats(x)
    res, _, _ = orc.dsaciq_search(x, st, 4, 100)
    assert res.mse_star >= 0.9 * res.mse_aciq


def test_naive_range_loses_to_aciq_at_low_bitwidth_with_outliers():
    # Sec. 3 (naive PTQ vs ACIQ): with outliers the min/max range has a far larger MSE.
    x = si.make_config("C1")
    rc, st = orc.stats(x)
    for bits in (2, 4):
        naive = orc.make_qparams((st.min + st.max) / 2, (st.max - st.min) / 2, bits, x.size)
        aciq = orc.make_qparams(st.mean, orc.aciq_alpha(st, bits), bits, x.size)
        assert orc.sq_error(x, naive) > 3 * orc.sq_error(x, aciq)
    # with 16 bits the full range is at least as good as the clipped one
    naive = orc.make_qparams((st.min + st.max) / 2, (st.max - st.min) / 2, 16, x.size)
    aciq = orc.make_qparams(st.mean, orc.aciq_alpha(st, 16), 16, x.size)
    assert orc.sq_error(x, naive) <= orc.sq_error(x, aciq)


# ----------------------------------------------------------------------------- adaptive bitwidth rule (Eq. 2)

def _golden_adaptive():
    rows = []
    with open(os.path.join(GOLDEN, "adaptive_bitwidth_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                bw, q = line.split()
                rows.append((float(bw), int(q)))
    return rows


def test_eq2_reproduces_the_papers_adaptivity_run():
    n = 64 * 197 * 768
    for bw_mbps, q_expected in _golden_adaptive():
        for q_cur in (32, 16, 8, 6, 4, 2):          # the rule does not depend on where it starts from
            v_bits = n * q_cur
            assert orc.next_bits(v_bits, q_cur, 64, 100.0, bw_mbps * 1e6) == q_expected, (bw_mbps, q_cur)


def test_eq2_picks_the_highest_power_of_two_that_fits():
    rng = np.random.default_rng(2)
    for _ in range(2000):
        n = int(rng.integers(10_000, 50_000_000))
        s_img, rate = float(rng.integers(1, 129)), float(rng.uniform(5, 500))
        bw = float(10 ** rng.uniform(5.5, 10.5))
        q = orc.next_bits(n * 8, 8, s_img, rate, bw)
        budget = s_img / rate * bw
        fitting = [k for k in (32, 16, 8, 4, 2) if n * k <= budget]
        assert q == (max(fitting) if fitting else 2)


# ----------------------------------------------------------------------------- histogram-fit reading of Eq. 1

def _laplace_cdf(x, mu, b):
    z = (x - mu) / b
    return np.where(z < 0, 0.5 * np.exp(z), 1.0 - 0.5 * np.exp(-z))


def _exact_laplace_histogram(mu, b, lo, hi, nbins, n):
    edges = np.linspace(lo, hi, nbins + 1)
    mass = np.diff(_laplace_cdf(edges, mu, b))
    return np.round(mass / mass.sum() * n).astype(np.uint32)


def test_hist_search_recovers_the_scale_of_an_exact_laplace_histogram():
    # counts taken from the Laplace cdf itself: the pdf that fits them best has the true scale,
    # wherever the interval [b_E, b_R] starts and ends, and in both directions
    mu, b, n, nbins = 0.3, 0.7, 50_000_000, 2048
    for lo_b, hi_b in ((0.35, 1.4), (1.4, 0.35), (0.6, 0.8)):
        st = orc.Stats()
        st.n, st.nbins, st.mean, st.min, st.max = n, nbins, mu, mu - 12 * b, mu + 12 * b
        st.mad, st.b_r = lo_b, hi_b
        hist = _exact_laplace_histogram(mu, b, st.min, st.max, nbins, n)
        st.n = int(hist.sum())
        res, q, scores = orc.hist_search(st, hist, 4, 100)
        grid_step = abs(hi_b - lo_b) / 100
        assert abs(res.b_star - b) <= grid_step, (lo_b, hi_b, res.b_star)
        assert res.mse_star <= res.mse_aciq and res.j_star == int(np.argmin(scores))
        assert res.alpha_star == pytest.approx(orc.laplace_F(4) * res.b_star, rel=1e-15)


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_hist_search_matches_independent_numpy_statement(name):
    x = si.make_config(name, n=300_000)
    rc, st, hist = orc.stats(x, want_hist=True)
    res, q, scores = orc.hist_search(st, hist, 2, 100)
    binw = (st.max - st.min) / st.nbins
    c = st.min + (np.arange(st.nbins) + 0.5) * binw
    d_r = hist[:st.nbins].astype(np.float64) / (st.n * binw)
    ref = []
    for j in range(101):
        bj = st.mad + j * ((st.b_r - st.mad) / 100)
        d_e = np.exp(-np.abs(c - st.mean) / bj) / (2 * bj)
        ref.append(float(np.sum((d_r - d_e) ** 2)))
    ref = np.array(ref)
    assert np.allclose(scores, ref, rtol=1e-12, atol=0)
    assert res.j_star == int(np.argmin(ref)) or abs(ref[res.j_star] - ref.min()) <= 1e-12 * ref.min()
    assert res.mse_aciq == pytest.approx(ref[0] / st.nbins, rel=1e-12)
    lo_b, hi_b = sorted((st.mad, st.b_r))
    assert lo_b <= res.b_star <= hi_b
    oq = orc.make_qparams(st.mean, res.alpha_star, 2, x.size)
    assert (q.lo, q.hi, q.scale) == (oq.lo, oq.hi, oq.scale)


def test_hist_search_degenerate_keeps_b_e():
    x = np.full(100, 3.0, np.float32)
    rc, st, hist = orc.stats(x, want_hist=True)
    st.mad = 0.5          # pretend a scale; the bound is 0, so the grid collapses
    res, q, scores = orc.hist_search(st, hist, 4, 50)
    assert res.j_star == 0 and res.b_star == 0.5


# ----------------------------------------------------------------------------- variants of the search
# (Gaussian model, range intersected with the data's, coarse-to-fine sweep: not the paper's method)

def test_variant_with_defaults_is_the_papers_search():
    for name, bits in (("C1", 2), ("C3", 4), ("C2", 8)):
        x = si.make_config(name, n=6000)
        rc, st = orc.stats(x)
        r0, q0, s0 = orc.dsaciq_search(x, st, bits, 50)
        r1, q1, s1 = orc.dsaciq_search_variant(x, st, bits, 50)
        assert bytes(r0) == bytes(r1) and bytes(q0) == bytes(q1) and np.array_equal(s0, s1)


def test_clipped_grid_hand_worked_and_special_cases():
    # centre 1, alpha 2 -> [-1, 3]; data in [0, 10] -> [0, 3]; 2 bits: 3 intervals of width 1
    q = orc.make_qparams_clipped(1.0, 2.0, 0.0, 10.0, 2, 7)
    assert (q.lo, q.hi, q.scale, q.inv_scale, q.levels, q.n) == (0.0, 3.0, 1.0, 1.0, 3, 7)
    # data on both sides inside the range: both ends move
    q = orc.make_qparams_clipped(0.0, 8.0, -1.5, 6.0, 4, 1)
    assert (q.lo, q.hi) == (-1.5, 6.0) and q.scale == np.float32(7.5 / 15)
    # data range wider than the clipping range: nothing changes
    for bits in (2, 8):
        a = orc.make_qparams(0.3, 1.7, bits, 5)
        b = orc.make_qparams_clipped(0.3, 1.7, -100.0, 100.0, bits, 5)
        assert bytes(a) == bytes(b)
    # one distinct value: empty range, all codes 0
    q = orc.make_qparams_clipped(2.0, 1.0, 2.0, 2.0, 4, 3)
    assert (q.lo, q.hi, q.scale, q.inv_scale) == (2.0, 2.0, 0.0, 0.0)


def _numpy_scores_variant(x, mean, s_e, s_r, const, bits, t, lo_clip, hi_clip):
    """Independent sweep with numpy float32/float64 operations; the range is intersected with [lo_clip, hi_clip]."""
    L = 2 ** bits - 1
    scores = []
    for j in range(t + 1):
        s = s_e + j * ((s_r - s_e) / t)
        a32, c32 = np.float32(const * s), np.float32(mean)
        lo = max(np.float32(np.float64(c32) - np.float64(a32)), np.float32(lo_clip))
        hi = min(np.float32(np.float64(c32) + np.float64(a32)), np.float32(hi_clip))
        rng_ = np.float64(hi) - np.float64(lo)
        scale, inv = np.float32(rng_ / L), np.float32(L / rng_)
        r = np.clip(np.rint((np.minimum(np.maximum(x, lo), hi) - lo) * inv), 0, L)
        xh = (np.float64(lo) + r.astype(np.float64) * np.float64(scale)).astype(np.float32)
        e = (x - xh).astype(np.float64)
        scores.append(float(np.sum(e * e)))
    return np.array(scores)


@pytest.mark.parametrize("name,bits,dist,clip", [("C3", 2, 0, True), ("C3", 4, 0, True), ("C2", 3, 1, False),
                                                 ("C1", 4, 1, False), ("C3", 8, 1, True), ("C2", 2, 0, True)])
def test_variant_matches_brute_force_numpy_sweep(name, bits, dist, clip):
    x = si.make_config(name, n=4096)
    rc, st = orc.stats(x)
    res, q, scores = orc.dsaciq_search_variant(x, st, bits, 60, dist=dist, clip_to_data=clip)
    if dist == orc.GAUSS:
        # Gaussian model: sigma from the variance; bound = sigma of the normal density with the histogram's peak
        const = orc.gauss_G(bits)
        s_e, s_r = np.sqrt(st.var), 1.0 / (np.sqrt(2 * np.pi) * st.peak_density)
    else:
        const = scipy.special.lambertw(3.0 * 4.0 ** bits).real
        s_e, s_r = st.mad, st.b_r
    assert (res.b_e, res.b_r) == (pytest.approx(s_e, rel=1e-15), pytest.approx(s_r, rel=1e-15))
    lo_clip, hi_clip = (st.min, st.max) if clip else (-np.inf, np.inf)
    ref = _numpy_scores_variant(x, st.mean, s_e, s_r, const, bits, 60, lo_clip, hi_clip)
    assert np.allclose(scores, ref, rtol=1e-6, atol=0)
    assert res.j_star == int(np.argmin(scores))
    assert res.alpha_star == pytest.approx(const * (s_e + res.j_star * ((s_r - s_e) / 60)), rel=1e-13)
    if clip:
        assert q.lo >= np.float32(st.min) and q.hi <= np.float32(st.max)
        assert bytes(q) == bytes(orc.make_qparams_clipped(st.mean, res.alpha_star, st.min, st.max, bits, x.size))
    else:
        assert bytes(q) == bytes(orc.make_qparams(st.mean, res.alpha_star, bits, x.size))


def test_gauss_bound_recovers_sigma_of_an_exact_normal_histogram():
    # histogram built from the normal cdf: its peak density is 1/(sigma sqrt(2 pi)) up to the bin width
    sigma, n, nbins = 0.8, 10_000_000, 2048
    edges = np.linspace(-6 * sigma, 6 * sigma, nbins + 1)
    cdf = scipy.special.ndtr(edges / sigma)
    peak = float(np.max(np.diff(cdf))) / (edges[1] - edges[0])
    assert 1.0 / (np.sqrt(2 * np.pi) * peak) == pytest.approx(sigma, rel=1e-4)
    # and on a real sample the oracle's bound lands near sigma (peak of a noisy histogram is biased upwards)
    x = (np.random.default_rng(5).standard_normal(400_000) * sigma).astype(np.float32)
    rc, st = orc.stats(x, nbins=128)
    res, q, scores = orc.dsaciq_search_variant(x, st, 4, 10, dist=orc.GAUSS)
    assert res.b_e == pytest.approx(sigma, rel=5e-3)
    assert res.b_r == pytest.approx(sigma, rel=5e-2) and res.b_r < sigma * 1.001


def test_intersecting_with_the_data_range_helps_one_sided_data_and_is_neutral_otherwise():
    x = si.make_config("C3", n=60_000)          # after a GELU: min about -0.17, long right tail
    rc, st = orc.stats(x)
    for bits in (2, 4):
        r0, _, s0 = orc.dsaciq_search(x, st, bits, 40)
        r1, _, s1 = orc.dsaciq_search_variant(x, st, bits, 40, clip_to_data=True)
        assert r1.mse_star < 0.85 * r0.mse_star
    x = si.make_config("C1", n=60_000)          # symmetric with outliers: every candidate range lies inside the data's
    rc, st = orc.stats(x)
    r0, q0, s0 = orc.dsaciq_search(x, st, 4, 40)
    r1, q1, s1 = orc.dsaciq_search_variant(x, st, 4, 40, clip_to_data=True)
    assert np.array_equal(s0, s1) and bytes(q0) == bytes(q1)


@pytest.mark.parametrize("t,stride", [(100, 10), (100, 7), (100, 1), (37, 5), (10, 10), (10, 30), (1, 3), (255, 16)])
def test_coarse_to_fine_pick_finds_the_minimum_of_a_unimodal_curve(t, stride):
    rng = np.random.default_rng(t * 31 + stride)
    for trial in range(200):
        m = int(rng.integers(0, t + 1))
        down = np.sort(rng.random(m))[::-1] + 1.0          # strictly falling to the minimum ...
        up = np.sort(rng.random(t - m)) + 1.0              # ... and rising after it
        scores = np.concatenate([down, [0.5], up])
        j, ev = orc.c2f_pick(scores, stride)
        assert j == m == int(np.argmin(scores))
        assert ev.sum() <= -(-t // stride) + 1 + 2 * stride - 1


def test_coarse_to_fine_pick_on_arbitrary_curves_is_the_first_minimum_of_what_it_evaluates():
    rng = np.random.default_rng(11)
    for trial in range(300):
        t = int(rng.integers(1, 120))
        stride = int(rng.integers(1, 25))
        scores = rng.integers(0, 6, size=t + 1).astype(np.float64)      # many ties
        j, ev = orc.c2f_pick(scores, stride)
        coarse = sorted(set(min(i * stride, t) for i in range(t // stride + 2)))
        assert all(ev[c] for c in coarse)
        j1 = min(coarse, key=lambda c: (scores[c], c))
        window = range(max(0, j1 - stride + 1), min(t, j1 + stride - 1) + 1)
        assert all(ev[c] for c in window) and ev.sum() == len(set(coarse) | set(window))
        assert j == min(window, key=lambda c: (scores[c], c))
        assert scores[j] == scores[ev].min()                             # nothing evaluated is better


def test_coarse_to_fine_search_equals_pick_on_the_full_sweep():
    for name, bits, clip in (("C1", 2, False), ("C3", 4, True), ("C2", 8, False), ("C3", 2, False)):
        x = si.make_config(name, n=20_000)
        rc, st = orc.stats(x)
        full_r, full_q, full = orc.dsaciq_search_variant(x, st, bits, 100, clip_to_data=clip)
        for stride in (10, 4):
            r, q, sc = orc.dsaciq_search_variant(x, st, bits, 100, clip_to_data=clip, stride=stride)
            j, ev = orc.c2f_pick(full, stride)
            assert r.j_star == j
            assert np.array_equal(sc[ev], full[ev]) and np.isnan(sc[~ev]).all()
            assert r.mse_aciq == full_r.mse_aciq and r.mse_star == full[j] / x.size
            if j == full_r.j_star:       # the usual case: the error curve has one valley
                assert bytes(q) == bytes(full_q) and r.alpha_star == full_r.alpha_star
        # on these inputs the sweep with stride 10 does find the full sweep's winner
        assert orc.c2f_pick(full, 10)[0] == full_r.j_star


# ----------------------------------------------------------------------------- adaptive PDA controller (Sec. 3, Sec. 4.2)

def _replay_link(update, bandwidths_mbps, per_phase, n_elems, latency_s=0.0):
    """Send microbatches over a link whose bandwidth changes per phase (the controller is not told); the
    time a microbatch takes is its payload divided by the bandwidth in force.  Returns the bitwidth used
    for every microbatch."""
    used = []
    q = 32
    for bw in bandwidths_mbps:
        for _ in range(per_phase):
            used.append(q)
            bits = n_elems * q
            seconds = bits / (bw * 1e6) + latency_s if np.isfinite(bw) else 1e-6
            q = update(bits, seconds)
    return used


def test_controller_reproduces_the_papers_five_phases():
    """Sec. 4.2: window 50, microbatch 64, about 100 images/s; bandwidth unlimited -> 400 -> 50 -> 200 -> unlimited
    Mbps at 200-microbatch intervals; the bitwidth settles at 32 -> 16 -> 2 -> 8 -> 32, each one window period after
    the change."""
    n = 64 * 197 * 768
    c = orc.controller(50, 64, 100.0)
    used = _replay_link(lambda b, s: orc.controller_update(c, b, s), [np.inf, 400, 50, 200, np.inf], 200, n)
    settled = [used[200 * p + 199] for p in range(5)]
    assert settled == [32] + [q for _, q in _golden_adaptive()]
    for p in range(1, 5):
        phase = used[200 * p:200 * (p + 1)]
        assert phase[:50] == [settled[p - 1]] * 50           # nothing changes before the window expires
        assert phase[50:] == [settled[p]] * 150              # one decision, then stable
    assert c.decisions == 20


def test_controller_change_inside_a_window_gives_one_transient_decision():
    """When the bandwidth changes in the middle of a window the window average is a mixture, so one intermediate
    bitwidth may be chosen before the next window settles (the paper's run shows such a transient in phase 3)."""
    n = 64 * 197 * 768
    c = orc.controller(50, 64, 100.0, q_start=2)
    used = []
    q = 2
    for m in range(400):
        bw = 50e6 if m < 125 else 200e6          # change half-way through the third window
        used.append(q)
        q = orc.controller_update(c, n * q, n * q / bw)
    assert used[:150] == [2] * 150
    assert set(used[150:200]) == {4}              # the mixed window: 2 bit payloads at 50 and 200 Mbps average 80 Mbps
    assert used[200:] == [8] * 200


def test_controller_decides_exactly_what_eq2_decides_on_the_window_averages():
    rng = np.random.default_rng(8)
    for trial in range(50):
        window = int(rng.integers(1, 20))
        s_img, rate = float(rng.integers(1, 65)), float(rng.uniform(10, 300))
        c = orc.controller(window, s_img, rate, q_start=int(rng.choice([32, 16, 8, 4, 2])))
        n = int(rng.integers(100_000, 20_000_000))
        q = c.q_cur
        bits_w, secs_w = [], []
        for m in range(window * 6):
            bits = n * q
            secs = bits / float(10 ** rng.uniform(6.5, 9.5))
            bits_w.append(bits)
            secs_w.append(secs)
            q_new = orc.controller_update(c, bits, secs)
            if (m + 1) % window == 0:
                expect = orc.next_bits(sum(bits_w) / window, q, s_img, rate, sum(bits_w) / sum(secs_w))
                assert q_new == expect
                bits_w, secs_w = [], []
            else:
                assert q_new == q
            q = q_new


def test_threaded_search_harness_is_the_sequential_search():
    """dsaciq_search_threads only changes who calls orc_sq_error when: scores, winner and grid are those of
    orc_dsaciq_search bit for bit, and orc_search_candidate / orc_search_pick are the loop's two halves."""
    for name, n in (("C2", 50_003), ("C3", 20_001), ("C1", 7_777)):
        x = si.make_config(name, n=n)
        rc, st = orc.stats(x)
        for bits, t in ((2, 100), (8, 100), (4, 7)):
            r1, q1, s1 = orc.dsaciq_search(x, st, bits, t)
            r2, q2, s2 = orc.dsaciq_search_threads(x, st, bits, t, threads=5)
            assert bytes(r1) == bytes(r2) and bytes(q1) == bytes(q2) and np.array_equal(s1, s2)
            F = orc.laplace_F(bits)
            for j in (0, 1, t // 2, t):   # the candidate's grid is F(q) (b_E + j (b_R - b_E)/t) about the mean
                a = orc.make_qparams(st.mean, F * (st.mad + j * ((st.b_r - st.mad) / t)), bits, x.size)
                assert bytes(orc.search_candidate(st, bits, t, x.size, j)) == bytes(a)
    # the decision alone: first minimum, ties to the smaller index
    rc, st = orc.stats(si.make_config("C1", n=1000))
    res, q = orc.search_pick(st, 4, 4, 1000, [5.0, 3.0, 3.0, 4.0, 3.0])
    assert res.j_star == 1 and res.mse_aciq == 5.0 / 1000 and res.mse_star == 3.0 / 1000
    res, q = orc.search_pick(st, 4, 2, 1000, [1.0, 1.0, 1.0])
    assert res.j_star == 0


# ----------------------------------------------------------------------------- which model fits: Laplace or Gaussian

def _exact_normal_histogram(mu, sigma, lo, hi, nbins, n):
    edges = np.linspace(lo, hi, nbins + 1)
    mass = np.diff(scipy.special.ndtr((edges - mu) / sigma))
    return np.round(mass / mass.sum() * n).astype(np.uint32)


def _stats_of_histogram(hist, lo, hi, mu, mad, var):
    st = orc.Stats()
    st.n, st.nbins, st.min, st.max = int(hist.sum()), hist.size, lo, hi
    st.mean, st.mad, st.var = mu, mad, var
    return st


def test_model_fit_picks_the_model_a_histogram_was_drawn_from():
    """A histogram taken from the Laplace cdf, with the Laplace moments (MAD = b, var = 2 b^2), must fit the Laplace
    pdf better than the normal pdf of the same variance, and the other way round for one taken from the normal
    cdf (MAD = sigma sqrt(2/pi), var = sigma^2): in each case the own model's misfit is only the binning error."""
    n, nbins = 40_000_000, 2048
    for mu, s in ((0.0, 1.0), (0.3, 0.7), (-2.0, 0.05)):
        h = _exact_laplace_histogram(mu, s, mu - 12 * s, mu + 12 * s, nbins, n)
        d, fl, fg = orc.model_fit(_stats_of_histogram(h, mu - 12 * s, mu + 12 * s, mu, s, 2 * s * s), h)
        assert d == orc.LAPLACE and fl < 1e-3 * fg
        h = _exact_normal_histogram(mu, s, mu - 8 * s, mu + 8 * s, nbins, n)
        d, fl, fg = orc.model_fit(_stats_of_histogram(h, mu - 8 * s, mu + 8 * s, mu, s * math.sqrt(2 / math.pi), s * s), h)
        assert d == orc.GAUSS and fg < 1e-3 * fl


@pytest.mark.parametrize("name,expect", [("C1", 0), ("C3", None), ("gauss", 1), ("laplace", 0), ("C5", None)])
def test_model_fit_matches_independent_numpy_statement(name, expect):
    if name == "gauss":
        x = (np.random.default_rng(11).standard_normal(300_000) * 0.6 + 0.2).astype(np.float32)
    elif name == "laplace":
        x = np.random.default_rng(12).laplace(-0.1, 0.4, size=300_000).astype(np.float32)
    elif name == "C5":
        x = orc.widen_bf16(si.make_config("C5", n=300_000))
    else:
        x = si.make_config(name, n=300_000)
    for nbins in (2048, 64):
        rc, st, hist = orc.stats(x, nbins=nbins, want_hist=True)
        d, fl, fg = orc.model_fit(st, hist)
        binw = (st.max - st.min) / nbins
        c = st.min + (np.arange(nbins) + 0.5) * binw
        d_r = hist[:nbins].astype(np.float64) / (st.n * binw)
        sg = math.sqrt(st.var)
        ref_l = float(np.sum((d_r - np.exp(-np.abs(c - st.mean) / st.mad) / (2 * st.mad)) ** 2))
        ref_g = float(np.sum((d_r - np.exp(-((c - st.mean) ** 2) / (2 * sg * sg)) / (sg * math.sqrt(2 * math.pi))) ** 2))
        assert fl == pytest.approx(ref_l, rel=1e-12) and fg == pytest.approx(ref_g, rel=1e-12)
        assert d == (orc.GAUSS if ref_g < ref_l else orc.LAPLACE)
        if expect is not None and nbins == 2048:
            assert d == expect
    # the Laplace fit is the histogram-fit search's score of its first candidate (same D_R, same pdf at b_E)
    rc, st, hist = orc.stats(x, want_hist=True)
    res, q, scores = orc.hist_search(st, hist, 4, 10)
    assert orc.model_fit(st, hist)[1] == pytest.approx(scores[0], rel=1e-13)


def test_model_fit_degenerate_inputs_keep_the_papers_model():
    for x in (np.full(500, 2.5, np.float32), np.zeros(10, np.float32), np.array([1.0], np.float32)):
        rc, st, hist = orc.stats(x, want_hist=True)
        d, fl, fg = orc.model_fit(st, hist)
        assert d == orc.LAPLACE and not (fg < fl)
    # an exact tie keeps Laplace: only a strictly better Gaussian fit switches the model
    st = orc.Stats()
    st.n, st.nbins, st.min, st.max, st.mean, st.mad, st.var = 0, 16, 0.0, 1.0, 0.5, 0.2, 0.1
    assert orc.model_fit(st, np.zeros(16, np.uint32))[0] == orc.LAPLACE
