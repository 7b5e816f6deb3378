"""Pins of the controller oracle against closed forms, exact rational arithmetic and brute force
(Sec. 3.3, "Adaptive Acceleration Activation" and "Dual-Linkage Acceleration").  The paper prints
no worked numbers for these equations, so the pins are identities and special cases that a
dropped term, a shifted index or a wrong sign would break."""
import math
from fractions import Fraction

import pytest

from oracle import nova_controller as K


# ---------------------------------------------------------------------------------------------
# growth rate, baseline, smoothing: telescoping identities with exact rationals
# ---------------------------------------------------------------------------------------------
def _rational_sequence():
    # an arbitrary, non-monotone sequence of exact rationals (binary fractions: exact in float64)
    return [Fraction(n, 64) for n in (3, 40, 70, 96, 91, 120, 131, 133, 140, 138, 141)]


def test_growth_rates_are_first_differences():
    hb = _rational_sequence()
    g = K.growth_rates([float(h) for h in hb])
    assert len(g) == len(hb) - 1
    for i, gi in enumerate(g):
        # element i is g_{i+2} = Hbar_{i+2} - Hbar_{i+1}
        assert Fraction(gi) == hb[i + 1] - hb[i]


@pytest.mark.parametrize("t_est", [2, 3, 5, 8])
def test_baseline_telescopes(t_est):
    # sum_{t=2..t_est} g_t = Hbar_{t_est} - Hbar_1
    hb = _rational_sequence()
    eta = K.baseline_growth([float(h) for h in hb], t_est)
    assert eta == pytest.approx(float((hb[t_est - 1] - hb[0]) / (t_est - 1)), rel=1e-15)


@pytest.mark.parametrize("t", [3, 4, 7, 11])
def test_smoothed_growth_telescopes(t):
    # (g_t + g_{t-1}) / 2 = (Hbar_t - Hbar_{t-2}) / 2
    hb = _rational_sequence()
    gs = K.smoothed_growth([float(h) for h in hb], t)
    assert Fraction(gs) == (hb[t - 1] - hb[t - 3]) / 2


def test_baseline_rejects_short_input():
    with pytest.raises(ValueError):
        K.baseline_growth([1.0, 2.0], 3)
    with pytest.raises(ValueError):
        K.baseline_growth([1.0, 2.0], 1)


# ---------------------------------------------------------------------------------------------
# activation scale
# ---------------------------------------------------------------------------------------------
def _brute_t_star(hb, t_est, alpha):
    """Exact-rational restatement by exhaustive search over t (no early exit, then the minimum)."""
    T = len(hb)
    if T < t_est + 1:
        return None
    g = {t: hb[t - 1] - hb[t - 2] for t in range(2, T + 1)}
    eta = sum(g[t] for t in range(2, t_est + 1)) / (t_est - 1)
    hits = [t for t in range(t_est + 1, T + 1) if (g[t] + g[t - 1]) / 2 <= alpha * eta]
    return min(hits) if hits else None


def test_linear_growth_never_stabilises():
    # Hbar_t = a + b t with b > 0: g = eta = g~ = b > alpha b
    hb = [0.25 + 0.5 * t for t in range(1, 14)]
    assert K.activation_scale(hb, 5, 0.5) is None


def test_flat_entropy_activates_at_first_candidate():
    # b = 0: g~ = 0 <= alpha * 0
    assert K.activation_scale([2.0] * 10, 5, 0.5) == 6


def test_geometric_saturation_closed_form():
    # Hbar_t = 1 - r^t: g_t = r^(t-1) (1 - r), eta = (r - r^t_est) / (t_est - 1),
    # g~_t = r^(t-2) (1 - r^2) / 2; the first t >= t_est + 1 below alpha * eta
    r, t_est, alpha = Fraction(1, 2), 5, Fraction(1, 2)
    hb = [1 - r ** t for t in range(1, 16)]
    eta = (r - r ** t_est) / (t_est - 1)
    expect = next(t for t in range(t_est + 1, 16) if r ** (t - 2) * (1 - r * r) / 2 <= alpha * eta)
    assert K.activation_scale([float(h) for h in hb], t_est, float(alpha)) == expect == 6
    # slower saturation pushes the inflection later
    r = Fraction(7, 8)
    hb = [1 - r ** t for t in range(1, 40)]
    eta = (r - r ** t_est) / (t_est - 1)
    expect = next(t for t in range(t_est + 1, 40) if r ** (t - 2) * (1 - r * r) / 2 <= alpha * eta)
    assert K.activation_scale([float(h) for h in hb], t_est, float(alpha)) == expect
    assert expect > 6


@pytest.mark.parametrize("seed", range(25))
def test_activation_scale_matches_exhaustive_rational_search(seed):
    import random
    rng = random.Random(seed)
    T = rng.randint(2, 14)
    hb = [Fraction(rng.randint(0, 512), 64) for _ in range(T)]
    t_est = rng.randint(2, 6)
    alpha = Fraction(rng.randint(1, 15), 16)
    assert K.activation_scale([float(h) for h in hb], t_est, float(alpha)) == _brute_t_star(hb, t_est, alpha)


def test_activation_is_online():
    # appending later scales never changes an already detected t*
    hb = [1 - 0.5 ** t for t in range(1, 12)]
    t_star = K.activation_scale(hb, 5, 0.5)
    for T in range(t_star, len(hb) + 1):
        assert K.activation_scale(hb[:T], 5, 0.5) == t_star
    assert K.activation_scale(hb[:t_star - 1], 5, 0.5) is None


# ---------------------------------------------------------------------------------------------
# scale-linkage ratio
# ---------------------------------------------------------------------------------------------
def test_scale_ratio_closed_values():
    # at the first accelerated scale the sigmoid is exactly 1/2
    assert K.scale_ratio(7, 6, 0.0, 0.8, 0.1) == 0.5
    # sigmoid(ln 3) = 3/4 and tanh(ln 2) = 3/5: (t - t* - 1) / tau = ln 3, g = ln 2
    r = K.scale_ratio(8, 6, math.log(2.0), 1.0 / math.log(3.0), 0.1)
    assert r == pytest.approx(0.75 - 0.1 * 0.6, abs=1e-15)
    # sigmoid(-ln 3) = 1/4, tanh(-ln 2) = -3/5
    r = K.scale_ratio(6, 6, -math.log(2.0), 1.0 / math.log(3.0), 0.25)
    assert r == pytest.approx(0.25 + 0.25 * 0.6, abs=1e-15)


def test_scale_ratio_symmetry_and_limits():
    tau, lam = 0.8, 0.1
    for d in (1, 2, 5):
        for g in (0.0, 0.3, -1.2):
            a = K.scale_ratio(10 + d, 9, g, tau, lam)      # t - (t*+1) = +d
            b = K.scale_ratio(10 - d, 9, -g, tau, lam)     # t - (t*+1) = -d
            assert a + b == pytest.approx(1.0, abs=1e-15)  # sigma(x) + sigma(-x) = 1, tanh odd
    # far past the activation scale the base ratio saturates at 1
    assert K.scale_ratio(200, 6, 0.7, tau, lam) == pytest.approx(1.0 - lam * math.tanh(0.7), abs=1e-15)
    # small g: tanh g = g - g^3/3 + O(g^5)
    g = 1e-3
    assert K.scale_ratio(7, 6, g, tau, 1.0) == pytest.approx(0.5 - (g - g ** 3 / 3), abs=1e-15)


def test_scale_ratio_monotone():
    vals = [K.scale_ratio(t, 6, 0.2, 0.8, 0.1) for t in range(4, 14)]
    assert all(b > a for a, b in zip(vals, vals[1:]))            # later scales prune more
    vals = [K.scale_ratio(9, 6, g, 0.8, 0.1) for g in (-1.0, -0.1, 0.0, 0.1, 1.0)]
    assert all(b < a for a, b in zip(vals, vals[1:]))            # faster entropy growth prunes less
    assert K.scale_ratio(9, 6, 0.4, 0.8, 0.0) == K.sigmoid(2 / 0.8)


# ---------------------------------------------------------------------------------------------
# layer-linkage ratio
# ---------------------------------------------------------------------------------------------
def test_layer_ratio_special_cases():
    assert K.layer_ratio(0.4, [1.7]) == 0.4                                   # j = 1
    assert K.layer_ratio(0.4, [1.5, 1.5, 1.5, 1.5]) == pytest.approx(0.4)     # no deviation
    assert K.layer_ratio(0.4, [1.0, 3.0, 4.0]) == pytest.approx(0.0)          # twice the mean: Delta = 1
    assert K.layer_ratio(0.4, [1.0, 3.0, 0.0]) == pytest.approx(0.8)          # zero entropy: Delta = -1
    assert K.layer_ratio(0.4, [0.0, 0.0, 2.0]) == 0.4                         # mu = 0: falls back
    with pytest.raises(ValueError):
        K.layer_ratio(0.4, [])


@pytest.mark.parametrize("seed", range(10))
def test_layer_ratio_exact_rationals(seed):
    import random
    rng = random.Random(100 + seed)
    j = rng.randint(2, 9)
    hb = [Fraction(rng.randint(1, 400), 32) for _ in range(j)]
    ratio_t = Fraction(rng.randint(0, 64), 64)
    mu = sum(hb[:-1]) / (j - 1)
    expect = ratio_t * (1 - (hb[-1] - mu) / mu)
    assert K.layer_ratio(float(ratio_t), [float(h) for h in hb]) == pytest.approx(float(expect), rel=1e-14, abs=1e-15)


def test_layer_ratio_uses_only_preceding_layers_for_the_mean():
    # changing the current layer's entropy must not move mu
    a = K.layer_ratio(0.5, [2.0, 4.0, 3.0])       # mu = 3, Delta = 0
    b = K.layer_ratio(0.5, [2.0, 4.0, 6.0])       # mu = 3, Delta = 1
    assert a == pytest.approx(0.5) and b == pytest.approx(0.0)


# ---------------------------------------------------------------------------------------------
# keep count
# ---------------------------------------------------------------------------------------------
def test_keep_count_edges():
    assert K.keep_count(0.0, 4096) == 4096
    assert K.keep_count(1.0, 4096) == 0
    assert K.keep_count(-0.3, 100) == 100           # clamped
    assert K.keep_count(1.7, 100) == 0              # clamped
    assert K.keep_count(0.5, 7) == 4                # floor(3.5) = 3 pruned


@pytest.mark.parametrize("N", [1, 7, 169, 4096])
def test_keep_count_is_ceil_of_kept_fraction(N):
    # N - floor(r N) = ceil((1 - r) N) for exact rational r
    for num in range(0, 65):
        r = Fraction(num, 64)
        assert K.keep_count(float(r), N) == math.ceil((1 - r) * N)


@pytest.mark.parametrize("N", [7, 169, 4096, 65536])
def test_keep_count_clamps_and_keeps_everything_for_nan(N):
    assert K.keep_count(float("nan"), N) == N
    assert K.keep_count(-2.0, N) == N and K.keep_count(3.0, N) == 0
    assert K.keep_count(0.0, N) == N and K.keep_count(1.0, N) == 0
