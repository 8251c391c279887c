"""Brute-force checks of the error model behind the Magnitude-aware Clipping Strategy.

The run-time clip rule is closed-form (Eq. "gaus", Eq. "fats"); alpha never
appears at run time, so these tests validate the MODEL the rules come from
(Eq. "e", Eq. "e2", the printed Inverted-T derivative, Eq. "inequal") by grid
search, not the clip value itself.
"""
import numpy as np

from oracle import mcs_model as m

EPS, GMAX, A_, B_ = 0.05, 1.0, 8.0, 0.3


def test_printed_derivative_matches_numeric_derivative_of_the_model():
    p = m.invT_density(EPS, GMAX, A_, B_)
    for alpha in (0.2, 2.0):
        for s in (0.2, 0.5, 0.8):
            h = 1e-4
            num = (m.E_model(s + h, alpha, p, GMAX, breaks=(EPS,)) - m.E_model(s - h, alpha, p, GMAX, breaks=(EPS,))) / (2 * h)
            assert abs(num - m.dE_ds_invT(s, alpha, EPS, GMAX, A_, B_)) < 1e-5 * abs(num) + 1e-8


def _root(alpha):
    f = lambda s: m.dE_ds_invT(s, alpha, EPS, GMAX, A_, B_)
    lo, hi = EPS * 1.01, GMAX
    if f(hi) <= 0:
        return GMAX
    assert f(lo) < 0
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        lo, hi = (lo, mid) if f(mid) > 0 else (mid, hi)
    return lo


def test_root_of_derivative_is_the_grid_argmin_of_the_model():
    p = m.invT_density(EPS, GMAX, A_, B_)
    for alpha in (0.5, 2.0):
        grid = np.linspace(EPS * 1.01, GMAX, 1001)
        E = [m.E_model(s, alpha, p, GMAX, breaks=(EPS,)) for s in grid]
        best = grid[int(np.argmin(E))]
        assert abs(best - _root(alpha)) <= 2 * (grid[1] - grid[0])


def test_empirical_error_of_real_quantization_agrees_with_the_model():
    # samples of the piecewise-uniform density, actually quantized with Eq. "suq": the arg-min of the
    # measured error lands near the model's optimum (difference = the rectangle-rule assumption)
    rng = np.random.default_rng(0)
    mass_a, mass_b = A_ * EPS, B_ * (GMAX - EPS)
    n = 400_000
    inner = rng.random(n) < mass_a / (mass_a + mass_b)
    mag = np.where(inner, rng.uniform(0, EPS, n), rng.uniform(EPS, GMAX, n))
    g = mag * rng.choice([-1.0, 1.0], n)
    alpha = 2.0
    grid = np.linspace(0.6, 1.0, 81)
    best = grid[int(np.argmin([m.E_emp(g, s, alpha) for s in grid]))]
    assert abs(best - _root(alpha)) < 0.03


def test_gaussian_optimum_moves_to_gmax_as_alpha_grows():
    # Eq. "inequal": beta = s/|g|max increases with alpha; for large alpha the optimum IS |g|max,
    # which is why bell-shaped channels take s = |g|max (Eq. "gaus").
    rng = np.random.default_rng(1)
    g = rng.normal(0, 1, 200_000)
    gm = np.abs(g).max()
    grid = np.linspace(0.3 * gm, gm, 141)
    betas = []
    for alpha in (0.0, 0.5, 1.0, 2.0, 4.0):
        E = [m.E_emp(g, s, alpha) for s in grid]
        betas.append(grid[int(np.argmin(E))] / gm)
    assert all(b1 >= b0 - 1e-9 for b0, b1 in zip(betas, betas[1:]))
    assert betas[0] < 0.8 and betas[-1] > 0.99


def test_long_tail_prefers_a_clip_below_gmax():
    # the motivation for clipping sharp / long-tailed channels: unweighted error is minimised well below |g|max
    rng = np.random.default_rng(2)
    lap = rng.laplace(0, 1e-3, 200_000)
    g = np.where(rng.random(200_000) < 0.01, 50 * lap, lap)
    gm = np.abs(g).max()
    grid = np.linspace(0.05 * gm, gm, 96)
    best = grid[int(np.argmin([m.E_emp(g, s, 0.0) for s in grid]))]
    assert best < 0.5 * gm
