"""Brute-force checks of the error model behind the Magnitude-aware Clipping Strategy.

The run-time clip rule is closed-form (Eq. "gaus", Eq. "fats"); alpha never
appears at run time, so these tests validate the MODEL the rules come from
(Eq. "e", Eq. "e2", the printed Inverted-T derivative, Eq. "inequal") by grid
search, not the clip value itself.
"""
import numpy as np

from oracle import mcs_model as m

import pytest  # noqa: F401  (the `ref` fixture comes from conftest)

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


# ----------------------------------------------------------------------------- the search routine of the oracle

def test_clip_search_is_the_literal_objective_on_its_grid(ref):
    """daq_ref_clip_search against the literal fp64 evaluation of Eq. "e" in mcs_model (independent code: numpy, the
    quantizer written from Eq. "suq" as printed).  The two quantizers differ only at exact ties, of which random data
    has none; what remains is the fp32 rounding of the de-quantized value (2^-24 of a value up to 254 times the typical
    error), hence the 5e-5."""
    rng = np.random.default_rng(21)
    g = np.stack([rng.normal(0, 10.0 ** rng.uniform(-3, -1), (3, 9, 8)) for _ in range(4)], axis=1).astype(np.float32)
    for alpha in (0.0, 1.5, 40.0):
        err, best_s, best_j = ref.clip_search(g, alpha, 16)
        for c in range(4):
            gm = np.abs(g[:, c]).max()
            for j in range(1, 17):
                s = float(np.float32(gm) * (np.float32(j) / np.float32(16)))
                want = m.E_emp(g[:, c].astype(np.float64), s, alpha)
                assert abs(err[c, j - 1] - want) <= 5e-5 * want
            assert best_j[c] == int(np.argmin(err[c])) + 1
            assert best_s[c] == np.float32(gm) * (np.float32(best_j[c]) / np.float32(16))


def test_clip_search_on_a_hand_example(ref):
    # one channel, values 1, 2, 127 and J = 127: candidate j has s = j.  With s = 127 every value is a grid point
    # (error 0).  With s = 2: 1 -> code 64 (63.5 is a tie, to even) = 64*2/127, 2 -> exact, 127 -> clipped to 2.
    g = np.array([1.0, 2.0, 127.0], np.float32).reshape(3, 1, 1, 1)
    err, best_s, best_j = ref.clip_search(g, 0.0, 1)
    assert err[0, 0] == 0.0 and best_j[0] == 1 and best_s[0] == 127.0
    err, best_s, best_j = ref.clip_search(2 * g / 127, 0.0, 1)          # |g|max = 2: the same codes, scaled
    assert err[0, 0] < 1e-9
    g2 = np.array([1.0, 2.0, 4.0], np.float32).reshape(3, 1, 1, 1)
    err, _, _ = ref.clip_search(g2, 0.0, 2)                              # candidates s = 2 and s = 4
    e_s2 = (abs(1 - 64 * 2 / 127) + 0 + (4 - 2)) / 3                     # 63.5 -> 64 (tie to even); 4 is clipped to 2
    e_s4 = (abs(1 - 32 * 4 / 127) + abs(2 - 64 * 4 / 127) + 0) / 3       # 31.75 -> 32, 63.5 -> 64
    assert abs(err[0, 0] - e_s2) < 1e-7 and abs(err[0, 1] - e_s4) < 1e-7
    # the weight: alpha = ln 2 doubles the term of |g| = 1, quadruples |g| = 2, x16 for |g| = 4
    errw, _, _ = ref.clip_search(g2, float(np.log(2.0)), 2)
    assert abs(errw[0, 0] - (2 * abs(1 - 64 * 2 / 127) + 16 * 2) / 3) < 1e-5


def test_clip_search_reproduces_the_premises_of_the_rules(ref):
    # bell-shaped channel, large alpha: the optimum is |g|max (Eq. "inequal" -> Eq. "gaus"); long-tailed channel,
    # alpha = 0: far below |g|max (why such channels are clipped, Eq. "fats")
    rng = np.random.default_rng(22)
    bell = rng.normal(0, 1e-2, (8, 1, 40, 40))
    lap = rng.laplace(0, 1e-3, (8, 1, 40, 40))
    tail = np.where(rng.random(lap.shape) < 0.01, 50 * lap, lap)
    g = np.concatenate([bell, tail], axis=1).astype(np.float32)
    _, _, bj_hi = ref.clip_search(g, 4.0 / 1e-2, 64)
    assert bj_hi[0] == 64
    _, _, bj_0 = ref.clip_search(g, 0.0, 64)
    assert bj_0[1] < 32 and bj_0[0] < 64
