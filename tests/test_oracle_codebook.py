"""Pins for the oracle's Lloyd-Max codebook and Haar rotation (CPU only).

Each check ties the oracle to something other than itself: a closed form, a
textbook table, an identity the paper states, or a value the paper prints.
"""
import math

import numpy as np
import pytest
from scipy import special

from oracle import ivftq_oracle as orc
from workloads import synth

DIMS = (64, 96, 128, 200)


def _cdf_sphere(t, d):
    """CDF of Lemma 1's density through the regularised incomplete beta function."""
    t = np.asarray(t, dtype=np.float64)
    return 0.5 + 0.5 * np.sign(t) * special.betainc(0.5, (d - 1) / 2.0, t * t)


def _first_moment_sphere(a, b, d):
    """Closed form of int_a^b t f_d(t) dt."""
    kappa = math.exp(math.lgamma(d / 2.0) - 0.5 * math.log(math.pi) - math.lgamma((d - 1) / 2.0))
    return kappa / (d - 1) * ((1 - a * a) ** ((d - 1) / 2.0) - (1 - b * b) ** ((d - 1) / 2.0))


def test_density_integrates_to_one_and_has_variance_one_over_d():
    for d in DIMS:
        t = np.linspace(-1, 1, 200001)
        f = orc.sphere_coord_density(t, d)
        assert abs(np.trapezoid(f, t) - 1.0) < 1e-8
        assert abs(np.trapezoid(t * t * f, t) - 1.0 / d) < 1e-9   # E[T^2] = 1/d on the sphere


@pytest.mark.parametrize("d", DIMS)
def test_one_bit_codebook_closed_form(d):
    # b=1: c = +-E|T| = +-Gamma(d/2) / (sqrt(pi) Gamma((d+1)/2)), approaching sqrt(2/(pi d))
    c, tau = orc.lloyd_max_codebook(1, d)
    closed = math.exp(math.lgamma(d / 2.0) - 0.5 * math.log(math.pi) - math.lgamma((d + 1) / 2.0))
    assert abs(c[1] - closed) < 1e-12 and abs(c[0] + closed) < 1e-12
    assert tau.shape == (1,) and abs(tau[0]) < 1e-15
    ratio = closed / math.sqrt(2.0 / (math.pi * d))
    assert 1.0 < ratio < 1.0 + 1.0 / d          # finite-d value sits just above the Gaussian limit


def test_one_bit_ratio_tends_to_gaussian_limit():
    ratios = []
    for d in (16, 64, 256, 1024, 4096):
        c, _ = orc.lloyd_max_codebook(1, d)
        ratios.append(c[1] / math.sqrt(2.0 / (math.pi * d)))
    assert all(a > b for a, b in zip(ratios[:-1], ratios[1:]))
    assert abs(ratios[-1] - 1.0) < 1e-4


@pytest.mark.parametrize("b", (1, 2, 3, 4))
def test_gaussian_mode_reproduces_textbook_lloyd_max(b):
    # Max (1960) optimal quantisers for a unit Gaussian: distortion and outermost level.
    textbook_D = {1: 0.3634, 2: 0.1175, 3: 0.03454, 4: 0.009497}[b]
    textbook_outer = {1: 0.7979, 2: 1.510, 3: 2.152, 4: 2.733}[b]
    d = 128
    c, tau = orc.lloyd_max_codebook(b, d, density="gauss")
    D = orc.codebook_distortion(c, tau, d, density="gauss")
    assert abs(D - textbook_D) < 5e-5
    assert abs(c[-1] * math.sqrt(d) - textbook_outer) < 1e-3
    if b == 4:
        assert abs(c[8] * math.sqrt(d) - 0.1284) < 1e-4     # innermost positive level


def test_paper_printed_distortion_neighbourhood(paper_numbers):
    # The paper quotes sqrt(D_4) ~ 0.102 and D_4 ~ 0.0104 for the Gaussian source.  The exact
    # Lloyd-Max value is 0.0095; 0.0104 is the high-resolution (Panter-Dite) figure
    # sqrt(3) pi / 2 * 4^-b = 0.0106 rounded down, so the oracle must land between.
    c, tau = orc.lloyd_max_codebook(4, 128, density="gauss")
    D = orc.codebook_distortion(c, tau, 128, density="gauss")
    panter_dite = math.sqrt(3.0) * math.pi / 2.0 * 4.0 ** -4
    assert D < paper_numbers["t2_D4"] < panter_dite + 3e-4
    assert abs(math.sqrt(paper_numbers["t2_D4"]) - paper_numbers["cs_sqrtD4"]) < 5e-4
    assert abs(math.sqrt(D) - paper_numbers["cs_sqrtD4"]) < 5e-3


@pytest.mark.parametrize("d", DIMS)
@pytest.mark.parametrize("b", (2, 3, 4))
def test_stationarity_against_closed_forms(b, d):
    """Boundaries are midpoints; centroids are conditional means computed another way
    (incomplete beta for the mass, closed-form first moment); orthogonality identities."""
    c, tau = orc.lloyd_max_codebook(b, d)
    K = 1 << b
    assert c.shape == (K,) and tau.shape == (K - 1,)
    assert np.all(np.diff(c) > 0)
    np.testing.assert_allclose(tau, 0.5 * (c[:-1] + c[1:]), atol=1e-15)
    np.testing.assert_allclose(c, -c[::-1], atol=1e-15)
    edges = np.concatenate(([-1.0], tau, [1.0]))
    mass = np.diff(_cdf_sphere(edges, d))
    first = np.array([_first_moment_sphere(edges[i], edges[i + 1], d) for i in range(K)])
    np.testing.assert_allclose(c, first / mass, rtol=0, atol=2e-11)
    np.testing.assert_allclose(orc.bin_masses(tau, d), mass, atol=1e-12)
    # every centroid lies inside its own bin (Lemma 2's premise)
    assert np.all(c > edges[:-1]) and np.all(c < edges[1:])
    # sum p_i c_i = 0 ; sum p_i c_i^2 = E[T C(T)] = (1 - D_b)/d   (proof of Theorem 2, bias term)
    D = orc.codebook_distortion(c, tau, d)
    assert abs(np.dot(mass, c)) < 1e-14
    assert abs(np.dot(mass, c * c) - (1.0 - D) / d) < 1e-12
    assert abs(np.dot(first, c) - (1.0 - D) / d) < 1e-12


@pytest.mark.parametrize("b,d", [(6, 8), (8, 8), (7, 96), (8, 128)])
def test_stationarity_at_many_levels_and_small_dimension(b, d):
    """K up to 256 and d = 8 (three standard deviations reach beyond the support): the result still
    meets the Lloyd-Max conditions, checked through the incomplete beta function and the closed-form
    first moment rather than the oracle's own quadrature."""
    c, tau = orc.lloyd_max_codebook(b, d)
    K = 1 << b
    assert np.all(np.isfinite(c)) and np.all(np.diff(c) > 0) and abs(c[-1]) < 1.0
    np.testing.assert_allclose(c, -c[::-1], atol=1e-15)
    edges = np.concatenate(([-1.0], tau, [1.0]))
    mass = np.diff(_cdf_sphere(edges, d))
    first = np.array([_first_moment_sphere(edges[i], edges[i + 1], d) for i in range(K)])
    np.testing.assert_allclose(c, first / mass, rtol=0, atol=5e-10)
    D = orc.codebook_distortion(c, tau, d)
    assert D < math.sqrt(3) * math.pi / 2 * 4.0 ** (-b)          # high-resolution bound
    assert abs(np.dot(mass, c * c) - (1.0 - D) / d) < 1e-12


@pytest.mark.parametrize("d", DIMS)
def test_distortion_decreases_with_bits_and_respects_high_resolution_bound(d):
    prev = None
    for b in (1, 2, 3, 4, 5):
        c, tau = orc.lloyd_max_codebook(b, d)
        D = orc.codebook_distortion(c, tau, d)
        if prev is not None:
            assert D < prev
            assert D > prev / 4.6          # each extra bit buys at most ~6 dB
        assert D <= math.sqrt(3.0) * math.pi / 2.0 * 4.0 ** -b
        prev = D
    # the sphere design beats the Gaussian design when the source really is the sphere marginal
    cg, tg = orc.lloyd_max_codebook(4, d, density="gauss")
    cs, ts = orc.lloyd_max_codebook(4, d)
    assert orc.codebook_distortion(cs, ts, d) < orc.codebook_distortion(cg, tg, d)


def test_codebook_depends_only_on_b_and_d_and_fp32_rounding():
    c32, t32 = orc.codebook_fp32(4, 96)
    c64, t64 = orc.lloyd_max_codebook(4, 96)
    assert c32.dtype == np.float32 and t32.dtype == np.float32
    np.testing.assert_array_equal(c32, c64.astype(np.float32))
    np.testing.assert_array_equal(t32, t64.astype(np.float32))
    with pytest.raises(ValueError):
        orc.lloyd_max_codebook(0, 96)
    with pytest.raises(ValueError):
        orc.lloyd_max_codebook(9, 96)


def test_quantize_is_nearest_centroid_with_ties_up():
    c, tau = orc.lloyd_max_codebook(3, 64)
    rng = np.random.default_rng(1)
    v = rng.normal(0, 1 / 8.0, size=5000)
    code = orc.quantize(v, tau)
    nearest = np.argmin(np.abs(v[:, None] - c[None, :]), axis=1)
    np.testing.assert_array_equal(code, nearest)
    # on a boundary the value belongs to the upper bin: [tau_i, tau_{i+1})
    np.testing.assert_array_equal(orc.quantize(tau, tau), np.arange(1, 8))
    np.testing.assert_array_equal(orc.quantize(np.nextafter(tau, -np.inf), tau), np.arange(0, 7))
    assert orc.quantize(np.array([-1.0]), tau)[0] == 0 and orc.quantize(np.array([1.0]), tau)[0] == 7


# ---------------------------------------------------------------- rotation


@pytest.mark.parametrize("d", (8, 64, 200))
def test_rotation_is_orthogonal_and_norm_preserving(d):
    G = synth.gaussian_matrix(3, d)
    Pi = orc.haar_rotation_from_gaussian(G)
    np.testing.assert_allclose(Pi @ Pi.T, np.eye(d), atol=1e-13)
    np.testing.assert_allclose(Pi.T @ Pi, np.eye(d), atol=1e-13)
    r = np.random.default_rng(0).normal(size=(50, d))
    np.testing.assert_allclose(np.linalg.norm(r @ Pi.T, axis=1), np.linalg.norm(r, axis=1), rtol=1e-13)
    # Pi^T G is upper triangular with positive diagonal: the unique QR with R_jj > 0,
    # which is what makes the factor Haar-distributed.
    R = Pi.T @ G
    assert np.max(np.abs(np.tril(R, -1))) < 1e-12
    assert np.all(np.diag(R) > 0)
    # Gram-Schmidt by hand on the first two columns gives the same first two columns
    q0 = G[:, 0] / np.linalg.norm(G[:, 0])
    w = G[:, 1] - q0 * (q0 @ G[:, 1])
    np.testing.assert_allclose(Pi[:, 0], q0, atol=1e-13)
    np.testing.assert_allclose(Pi[:, 1], w / np.linalg.norm(w), atol=1e-12)


def test_rotation_entries_have_haar_moments():
    d = 24
    first_col = []
    for seed in range(400):
        Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(seed, d))
        first_col.append(Pi[:, 0])
    first_col = np.array(first_col)            # Pi e_1 should be uniform on the sphere
    assert abs(first_col.mean()) < 0.01
    assert abs(first_col.var() - 1.0 / d) < 0.1 / d
    # fourth moment of a sphere coordinate: 3 / (d (d+2))
    assert abs((first_col ** 4).mean() - 3.0 / (d * (d + 2))) < 0.15 * 3.0 / (d * (d + 2))


# ---- Stage 2: sign-bit refinement (Appendix "Sign-bit refinement") -------------------------------


@pytest.mark.parametrize("b,d", [(1, 64), (2, 96), (3, 128), (4, 96), (4, 200)])
def test_half_bin_means_split_each_bin_consistently(b, d):
    c, tau = orc.lloyd_max_codebook(b, d)
    means, mass = orc.half_bin_means(c, tau, d)
    K = 1 << b
    edges = np.concatenate(([-1.0], tau, [1.0]))
    # each half-bin mean lies inside its half-bin
    assert np.all(means[:, 0] > edges[:-1]) and np.all(means[:, 0] < c)
    assert np.all(means[:, 1] > c) and np.all(means[:, 1] < edges[1:])
    # law of total expectation: the two halves average back to the bin's centroid, masses add up
    p = np.diff(_cdf_sphere(edges, d))                      # bin masses by the incomplete beta function
    np.testing.assert_allclose(mass.sum(axis=1), p, atol=1e-12)
    np.testing.assert_allclose((mass * means).sum(axis=1), p * c, atol=1e-12)
    # half-bin masses and first moments against closed forms
    for i in range(K):
        for s, (a_, b_) in enumerate(((edges[i], c[i]), (c[i], edges[i + 1]))):
            m0 = _cdf_sphere(np.array([a_, b_]), d)
            assert abs(mass[i, s] - (m0[1] - m0[0])) < 1e-12
            assert abs(means[i, s] - _first_moment_sphere(a_, b_, d) / (m0[1] - m0[0])) < 1e-10
    # symmetry of the density
    np.testing.assert_allclose(means[:, 0], -means[::-1, 1], atol=1e-13)


def test_one_bit_gaussian_refinement_matches_truncated_normal_means():
    """b = 1 under the Gaussian design: bins are the half-lines, the centroid is sigma*sqrt(2/pi), and
    the half-bin means are means of a normal truncated to [0, m) and [m, inf) (textbook formulas)."""
    d = 128
    sg = 1.0 / math.sqrt(d)
    c, tau = orc.lloyd_max_codebook(1, d, "gauss")
    assert abs(c[1] - sg * math.sqrt(2 / math.pi)) < 1e-12
    means, mass = orc.half_bin_means(c, tau, d, "gauss")
    a = c[1] / sg
    phi = lambda t: math.exp(-0.5 * t * t) / math.sqrt(2 * math.pi)
    Phi = lambda t: 0.5 * (1 + math.erf(t / math.sqrt(2)))
    inner = sg * (phi(0.0) - phi(a)) / (Phi(a) - Phi(0.0))
    outer = sg * phi(a) / (1.0 - Phi(a))
    assert abs(means[1, 0] - inner) < 1e-10 and abs(means[1, 1] - outer) < 1e-10
    assert abs(mass[1, 0] - (Phi(a) - 0.5)) < 1e-12


@pytest.mark.parametrize("b,d", [(2, 96), (3, 128), (4, 96)])
def test_refinement_sits_between_b_and_b_plus_one_bits(b, d):
    """The refined quantiser has 2^(b+1) levels but keeps the b-bit boundaries, so its distortion is
    below the b-bit one and cannot beat the optimal (b+1)-bit Lloyd-Max quantiser."""
    c, tau = orc.lloyd_max_codebook(b, d)
    levels, bnd = orc.refined_tables(c, tau, d)
    D_b = orc.codebook_distortion(c, tau, d)
    D_ref = orc.codebook_distortion(levels, bnd, d)
    c1, tau1 = orc.lloyd_max_codebook(b + 1, d)
    D_b1 = orc.codebook_distortion(c1, tau1, d)
    assert D_b1 < D_ref < D_b
    assert D_ref < 0.45 * D_b                                # one extra bit is worth close to a factor 4


@pytest.mark.parametrize("b,d", [(2, 64), (4, 128)])
def test_merged_table_form_equals_the_literal_definition(b, d):
    """code_refined = #{merged boundaries <= v} equals 2*code + 1[v >= c_code], and looking the level up
    equals the half-bin mean, for random values and for values exactly on centroids and boundaries."""
    c, tau = orc.lloyd_max_codebook(b, d)
    means, _ = orc.half_bin_means(c, tau, d)
    levels, bnd = orc.refined_tables(c, tau, d)
    rng = np.random.default_rng(b * 100 + d)
    v = np.concatenate([rng.standard_normal(20000) / math.sqrt(d), c, tau, np.nextafter(c, -1), np.nextafter(tau, -1), [-1, 1, 0]])
    code = orc.quantize(v[None, :], tau)[0]
    s = orc.sign_bits(v, code, c)
    refined = orc.quantize(v[None, :], bnd)[0]
    np.testing.assert_array_equal(refined, 2 * code.astype(np.int64) + s)
    np.testing.assert_array_equal(levels[refined], means[code, s])
    assert orc.bits_per_vector(4, 96, True) == 4 * 96 + 96 + 32    # the same total as (b+1)*d + 32
