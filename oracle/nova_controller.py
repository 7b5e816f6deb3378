"""CPU oracle for NOVA's ratio controllers (TEST INFRASTRUCTURE ONLY).

Plain float64 Python written from the paper's definitions; shares no code with
the HIP path and is never imported by the product package.

What each function follows (all in Sec. 3.3):
  growth_rates        -- "Adaptive Acceleration Activation": discrete entropy growth
                         rate g_t = Hbar_t - Hbar_{t-1}, t = 2..T.
  baseline_growth     -- same paragraph: eta, the mean of g_2..g_{t_est}.
  smoothed_growth     -- same paragraph: g~_t = (g_t + g_{t-1}) / 2 for t >= t_est + 1.
  activation_scale    -- same paragraph: t* = the earliest t >= t_est + 1 with
                         g~_t <= alpha * eta; acceleration starts at scale t* + 1.
  scale_ratio         -- "Dual-Linkage Acceleration", scale-linkage ratio:
                         Ratio_t = sigmoid((t - (t* + 1)) / tau) - lambda * tanh(g_t).
  layer_ratio         -- same paragraph, layer-linkage ratio: mu_{t,j-1} is the mean of
                         the preceding layers' scale mean entropies, Delta_{t,j} the
                         relative deviation of layer j from it,
                         Ratio_{t,j} = Ratio_t (j = 1), Ratio_t - Delta_{t,j} Ratio_t (j >= 2).
  keep_count          -- the integer number of tokens kept for a reduction ratio (exact arithmetic on the
                         float64 ratio).

Scales and layers are numbered from 1 as in the paper; Hbar[0] is Hbar_1.

Readings taken where the paper is silent (they are listed in the repository's design notes):
  * t* is detected online: the decision for scale t uses Hbar_1..Hbar_t only; when no scale
    satisfies the condition there is no t* (None) and nothing is accelerated.
  * eta is used as printed, whatever its sign.
  * mu_{t,j-1} = 0 makes Delta undefined: the layer ratio then falls back to Ratio_t.
  * a ratio is clamped to [0, 1] before it is turned into a count, and the count of
    pruned tokens is floor(ratio * N): k = N - floor(ratio * N).
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence


def growth_rates(hbar: Sequence[float]) -> List[float]:
    """[g_2, ..., g_T] for Hbar_1..Hbar_T (element i is g_{i+2})."""
    return [float(hbar[i]) - float(hbar[i - 1]) for i in range(1, len(hbar))]


def _g(hbar: Sequence[float], t: int) -> float:
    """g_t for a 1-based scale index t >= 2."""
    return float(hbar[t - 1]) - float(hbar[t - 2])


def baseline_growth(hbar: Sequence[float], t_est: int) -> float:
    """eta = (1 / (t_est - 1)) * sum_{t=2..t_est} g_t; needs t_est >= 2 and T >= t_est."""
    if t_est < 2 or len(hbar) < t_est:
        raise ValueError("baseline needs 2 <= t_est <= T")
    total = 0.0
    for t in range(2, t_est + 1):
        total += _g(hbar, t)
    return total / (t_est - 1)


def smoothed_growth(hbar: Sequence[float], t: int) -> float:
    """g~_t = (g_t + g_{t-1}) / 2 for a 1-based t >= 3."""
    return (_g(hbar, t) + _g(hbar, t - 1)) / 2.0


def activation_scale(hbar: Sequence[float], t_est: int, alpha: float) -> Optional[int]:
    """t* (1-based) or None: the earliest t >= t_est + 1 with g~_t <= alpha * eta."""
    T = len(hbar)
    if T < t_est + 1:
        return None
    eta = baseline_growth(hbar, t_est)
    for t in range(t_est + 1, T + 1):
        if smoothed_growth(hbar, t) <= alpha * eta:
            return t
    return None


def sigmoid(x: float) -> float:
    return 1.0 / (1.0 + math.exp(-x))


def scale_ratio(t: int, t_star: int, g_t: float, tau: float, lam: float) -> float:
    """Ratio_t = sigmoid((t - (t* + 1)) / tau) - lambda * tanh(g_t)."""
    return sigmoid((t - (t_star + 1)) / tau) - lam * math.tanh(g_t)


def layer_ratio(ratio_t: float, hbar_layers: Sequence[float]) -> float:
    """Ratio_{t,j} for j = len(hbar_layers): hbar_layers holds Hbar_{t,1}..Hbar_{t,j}."""
    j = len(hbar_layers)
    if j < 1:
        raise ValueError("needs the current layer's mean entropy")
    if j == 1:
        return float(ratio_t)
    mu = sum(float(h) for h in hbar_layers[:-1]) / (j - 1)
    if mu == 0.0:
        return float(ratio_t)
    delta = (float(hbar_layers[-1]) - mu) / mu
    return float(ratio_t) - delta * float(ratio_t)


def clamp_ratio(ratio: float) -> float:
    return min(1.0, max(0.0, ratio))


def keep_count(ratio: float, N: int) -> int:
    """k = N - floor(clamp(ratio) * N); a NaN ratio (an undefined entropy upstream) prunes nothing."""
    if math.isnan(ratio):
        return N
    return N - int(math.floor(clamp_ratio(ratio) * N))
