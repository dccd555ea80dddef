"""Pins for the oracle's innovation quantizer (Sec. 2.1, eqs. 5-6).

Nothing here calls the HIP path.  Each test checks the C oracle against
something the paper or arithmetic fixes independently of it: exact rational
brute force, the error bound, grid membership, invariances, closed forms.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(20190907)


def _case(p, scale_g=1.0, scale_h=1.0, rng=RNG):
    g = (rng.standard_normal(p) * scale_g).astype(np.float32)
    h = (rng.standard_normal(p) * scale_h).astype(np.float32)
    return g, h


def _fr(x):
    return Fraction(float(x))


@pytest.mark.parametrize("b", [1, 2, 3, 4, 5, 8, 11, 16])
def test_codes_equal_exact_rational_floor_formula(b):
    """eq. 5 evaluated in exact rational arithmetic on the fp32 inputs."""
    L = 2 ** b - 1
    g, h = _case(300)
    out = oracle.quantize(g, h, b)
    assert out["status"] == oracle.OK
    R = max(abs(_fr(a) - _fr(c)) for a, c in zip(g, h))
    # R itself: the oracle's radius is the fp32-rounded max |g-h|
    assert abs(Fraction(float(out["R"])) - R) <= R * Fraction(1, 2 ** 23)
    tol = max(Fraction(1, 2 ** 12), Fraction(L, 2 ** 20))
    n_tie = 0
    for i in range(g.size):
        t = (_fr(g[i]) - _fr(h[i]) + R) / (2 * R / L) + Fraction(1, 2)
        q_exact = min(max(t.numerator // t.denominator, 0), L)
        frac = t - (t.numerator // t.denominator)
        near_tie = min(frac, 1 - frac) < tol
        if near_tie:
            n_tie += 1
            assert abs(int(out["q"][i]) - q_exact) <= 1
        else:
            assert int(out["q"][i]) == q_exact, (i, b)
    assert n_tie < g.size // 4 + 8


@pytest.mark.parametrize("b", [1, 2, 3, 4])
def test_codes_are_nearest_grid_point_brute_force(b):
    """'adding 1/2 guarantees rounding to the closest point': argmin over all
    2^b grid points -R + 2 tau R j, ties to the larger j."""
    L = 2 ** b - 1
    g, h = _case(200)
    out = oracle.quantize(g, h, b)
    R = _fr(out["R"])
    for i in range(g.size):
        d = _fr(np.float32(g[i]) - np.float32(h[i]))
        dist = [abs(d - (-R + 2 * R * j / L)) for j in range(L + 1)]
        best = min(dist)
        cands = [j for j in range(L + 1) if dist[j] == best]
        q = int(out["q"][i])
        second = sorted(dist)[1] if L >= 1 else None
        if second is not None and (second - best) < R * Fraction(1, 2 ** 18):
            assert abs(q - cands[-1]) <= 1      # numerically tied
        else:
            assert q == cands[-1]


@pytest.mark.parametrize("b", [1, 2, 3, 4, 8, 16])
def test_code_range_and_end_point(b):
    L = 2 ** b - 1
    g, h = _case(1000, 3.0, 0.5)
    out = oracle.quantize(g, h, b)
    q = out["q"]
    assert q.min() >= 0 and q.max() <= L
    # the element that attains the radius maps to an end point of the grid
    i = int(np.argmax(np.abs(g - h)))
    assert q[i] in (0, L)
    assert (q[i] == L) == (g[i] - h[i] > 0)


@pytest.mark.parametrize("b", [1, 2, 3, 4, 8])
def test_error_bound_tau_R(b):
    """||eps||_inf <= tau R (Sec. 2.1), up to the fp32 rounding of h + deltaQ."""
    L = 2 ** b - 1
    for sg, sh in [(1.0, 1.0), (1e-3, 1.0), (1.0, 1e-4), (1e-6, 1e-6)]:
        g, h = _case(4000, sg, sh)
        out = oracle.quantize(g, h, b)
        R = float(out["R"])
        eps = g.astype(np.float64) - out["h_new"].astype(np.float64)
        ulp = np.spacing(np.abs(out["h_new"]).astype(np.float32)).astype(np.float64)
        bound = (R / L) * (1 + 2.0 ** -10) + 0.5 * ulp + 2.0 ** -22 * R
        assert np.all(np.abs(eps) <= bound)
        # unconditional fp32 bound used to size the integer error sum
        assert np.all(np.abs(eps) <= 2 * (R / L) * (1 + L * 2.0 ** -21))


def test_error_bound_holds_when_grid_is_finer_than_fp32():
    """h of order 1, innovation of a few ulps: eps may exceed tau R but never 2 tau R."""
    rng = np.random.default_rng(5)
    h = (1.0 + rng.random(5000)).astype(np.float32)
    k = rng.integers(-3, 4, 5000)
    g = h.copy()
    for _ in range(3):
        g = np.where(k > 0, np.nextafter(g, np.float32(4)), np.where(k < 0, np.nextafter(g, np.float32(0)), g))
        k = k - np.sign(k)
    for b in (3, 8):
        L = 2 ** b - 1
        out = oracle.quantize(g, h, b)
        R = float(out["R"])
        assert R > 0
        eps = g.astype(np.float64) - out["h_new"].astype(np.float64)
        assert np.all(np.abs(eps) <= 2 * (R / L) * (1 + L * 2.0 ** -21))
        naive = float(np.sum(eps ** 2))
        assert out["E2"] == pytest.approx(naive, rel=1e-4, abs=1e-300)


@pytest.mark.parametrize("b", [2, 3, 4, 8])
def test_delta_lies_on_the_grid_and_h_new_is_h_plus_delta(b):
    L = 2 ** b - 1
    g, h = _case(2000)
    out = oracle.quantize(g, h, b)
    R = float(out["R"])
    exact = -R + 2.0 * (R / L) * out["q"].astype(np.float64)
    assert np.all(np.abs(out["delta"].astype(np.float64) - exact) <= 4 * 2.0 ** -24 * R)
    assert np.array_equal(out["h_new"], (h + out["delta"]).astype(np.float32))
    assert np.array_equal(oracle.dequantize(out["q"], b, out["R"]), out["delta"])


@pytest.mark.parametrize("b", [2, 3, 4, 8])
@pytest.mark.parametrize("j", [-20, -3, 5, 17])
def test_power_of_two_scale_invariance(b, j):
    g, h = _case(1500)
    o1 = oracle.quantize(g, h, b)
    s = np.float32(2.0 ** j)
    o2 = oracle.quantize(g * s, h * s, b)
    assert np.array_equal(o1["q"], o2["q"])
    assert o2["R"] == o1["R"] * s
    assert o1["Sq"] == o2["Sq"]
    assert o2["E2"] == pytest.approx(o1["E2"] * float(s) ** 2, rel=1e-12)


def test_one_bit_gives_plus_minus_R():
    g, h = _case(500)
    out = oracle.quantize(g, h, 1)
    R = out["R"]
    assert set(np.unique(out["delta"])) <= {-R, R}
    assert np.array_equal(out["delta"] > 0, (g - h) + R >= R)  # sign of the innovation (ties up)
    assert out["Sq"] == 500
    assert out["lhs"] == pytest.approx(500 * float(R) ** 2, rel=1e-12)


@pytest.mark.parametrize("b", [1, 3, 8])
def test_single_coordinate_is_reproduced(b):
    g = np.array([0.37], np.float32)
    h = np.array([-1.25], np.float32)
    out = oracle.quantize(g, h, b)
    assert out["R"] == np.float32(1.62)
    assert out["q"][0] == 2 ** b - 1
    assert abs(float(out["delta"][0]) - 1.62) <= 2 ** -22
    assert abs(float(out["h_new"][0]) - 0.37) <= 2 ** -22


def test_zero_innovation():
    g = RNG.standard_normal(64).astype(np.float32)
    out = oracle.quantize(g, g.copy(), 4)
    assert out["status"] == oracle.OK and out["R"] == 0
    assert not out["q"].any() and not out["delta"].any()
    assert np.array_equal(out["h_new"], g)
    assert out["Sq"] == 0 and out["E2"] == 0 and out["lhs"] == 0


def test_nonfinite_radius_is_reported():
    g, h = _case(16)
    g[3] = np.inf
    assert oracle.quantize(g, h, 4)["status"] == oracle.ENONFINITE
    g[3] = np.nan
    assert oracle.quantize(g, h, 4)["status"] == oracle.ENONFINITE
    g[3] = np.float32(3e38)
    h[3] = np.float32(-3e38)
    assert oracle.quantize(g, h, 4)["status"] == oracle.ENONFINITE


@pytest.mark.parametrize("b", [1, 2, 3, 4, 8, 16])
def test_squared_norms_match_plain_sums(b):
    L = 2 ** b - 1
    g, h = _case(5000, 0.3, 0.1)
    out = oracle.quantize(g, h, b)
    d = out["delta"].astype(np.longdouble)
    assert out["lhs"] == pytest.approx(float(np.sum(d * d)), rel=1e-6)
    assert out["Sq"] == int(np.sum((2 * out["q"].astype(np.int64) - L) ** 2))
    e = g.astype(np.float64) - out["h_new"].astype(np.float64)
    assert out["E2"] == pytest.approx(float(np.sum(e * e)), rel=1e-4)


def test_error_sum_is_exact_on_its_grid():
    """E2 = 2^(2(x-K)) * sum rint(eps 2^(K-x))^2 with 2^(x-1) <= step < 2^x."""
    b, p = 3, 777
    g, h = _case(p)
    out = oracle.quantize(g, h, b)
    step = np.float32(np.float32(2) * out["R"]) / np.float32(2 ** b - 1)
    x = int(np.frexp(step)[1])
    K = oracle.eps_K(p)
    assert K == 20
    e = (g - out["h_new"]).astype(np.float32)
    n = np.rint(np.ldexp(e, K - x)).astype(np.int64)
    assert out["E2"] == float(np.sum(n * n)) * 2.0 ** (2 * (x - K))


def test_eps_K_keeps_the_integer_sum_below_2_64():
    for p in [1, 2, 1000, 2 ** 20, 2 ** 24, 2 ** 24 + 1, 2 ** 30, 2 ** 40]:
        K = oracle.eps_K(p)
        assert K <= 20
        assert p * (1.04 * 2 ** K) ** 2 < 2 ** 64
    assert oracle.eps_K(2 ** 24) == 19 and oracle.eps_K(2 ** 23) == 20


@pytest.mark.parametrize("b", [1, 2, 3, 4, 5, 7, 8, 12, 16])
def test_wire_format_is_an_lsb_first_bitstream(b):
    p = 1234
    q = RNG.integers(0, 2 ** b, p).astype(np.uint32)
    words = oracle.pack(q, b)
    assert words.size == (p * b + 31) // 32
    big = 0
    for i, v in enumerate(q.tolist()):
        big |= v << (i * b)
    ref = np.frombuffer(big.to_bytes(words.size * 4, "little"), dtype="<u4")
    assert np.array_equal(words, ref)
    assert np.array_equal(oracle.unpack(words, p, b), q)


def test_exact_mode_is_the_identity_quantizer():
    g, h = _case(333)
    out = oracle.quantize(g, h, oracle.B_EXACT)
    assert np.array_equal(out["h_new"], g)
    assert np.array_equal(out["delta"], g - h)
    assert out["E2"] == 0
    assert out["lhs"] == pytest.approx(float(np.sum((g - h).astype(np.float64) ** 2)), rel=1e-12)
