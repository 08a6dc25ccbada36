"""Skip-set selection from per-layer confidences (TEST INFRASTRUCTURE; Section 3.2, Eq. 5-10).

Steps, in the paper's order and notation:
  Eq. 5   c_hat_i = (c_i - mu_c) / (sigma_c + eps)
  Eq. 6   g = second-order discrete gradient of c_hat, min-max rescaled to [0, 1]
  Eq. 7   w_i = w_base + w_max * g_i * (l_i / num_layers)
  Eq. 8-9 local mean / std of c_hat over the window around i, excluding i
  Eq. 10  skip i  iff  c_hat_i < mu_local_i - lambda * sigma_local_i
followed by the skip-ratio bounds (minimum 40 %, Section 4.1.1; best range 40-60 %, Section 3.2)
and "sorted by index" output.  Where the paper leaves a detail open the reading taken is
listed in the design notes; this file implements exactly those readings:
  * population standard deviations; eps = 1e-8 in Eq. 5 and in the min-max rescale;
  * discrete gradient = numpy.gradient stencil (central inside, one-sided at the ends),
    applied twice, absolute value taken before rescaling;
  * w_max = kappa * (number of leading candidate layers whose confidence stays within
    flat_tol of the first one);
  * w_i is floored to an integer half-width: neighbours are j != i with |j - i| <= w_i;
  * first and last layer are not candidates when protect_ends is set (Appendix B considers
    38 of 40 layers);
  * ratio bounds are enforced by adding / removing layers in order of the margin
    c_hat_i - (mu_local_i - lambda * sigma_local_i), ties by index.
All sums are sequential left-to-right IEEE doubles so that an independent implementation can
reproduce every decision.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np


@dataclass
class SelectParams:
    lam: float = 0.3            # lambda of Eq. 10 (0.25 < lambda < 0.5, Section 4.1.1)
    w_base: float = 2.0         # Section 4.1.1
    kappa: float = 1.0          # w_max = kappa * n_flat
    flat_tol: float = 1e-3
    min_ratio: float = 0.40     # Section 4.1.1
    max_ratio: float = 0.60     # Section 3.2
    protect_ends: bool = True   # Appendix B
    eps: float = 1e-8
    fixed_w_max: float = -1.0   # >= 0 overrides kappa * n_flat (w_max = 0 gives a constant window)


def _seq_sum(v: Sequence[float]) -> float:
    s = 0.0
    for a in v:
        s += a
    return s


def _mean_std(v: Sequence[float]) -> Tuple[float, float]:
    n = len(v)
    if n == 0:
        return 0.0, 0.0
    mu = _seq_sum(v) / n
    var = _seq_sum([(a - mu) * (a - mu) for a in v]) / n
    return mu, math.sqrt(var)


def _gradient(y: List[float]) -> List[float]:
    if len(y) < 2:
        return [0.0] * len(y)
    return [float(a) for a in np.gradient(np.asarray(y, dtype=np.float64))]


def select_skip(conf: Sequence[float], params: SelectParams = SelectParams(), detail: bool = False):
    """conf[L] -> uint8 mask[L] (1 = skip).  With detail=True also returns the intermediates."""
    L = len(conf)
    p = params
    cand = list(range(1, L - 1)) if p.protect_ends else list(range(L))
    n = len(cand)
    mask = np.zeros(L, np.uint8)
    if n == 0:
        return (mask, {}) if detail else mask
    c = [float(conf[l]) for l in cand]

    mu, sigma = _mean_std(c)                                           # Eq. 5
    chat = [(ci - mu) / (sigma + p.eps) for ci in c]

    g = [abs(a) for a in _gradient(_gradient(chat))]                   # Eq. 6
    gmin, gmax = min(g), max(g)
    g = [(a - gmin) / (gmax - gmin + p.eps) for a in g]

    n_flat = 0
    for ci in c:
        if abs(ci - c[0]) <= p.flat_tol:
            n_flat += 1
        else:
            break
    w_max = p.fixed_w_max if p.fixed_w_max >= 0.0 else p.kappa * n_flat

    w = [int(math.floor(p.w_base + w_max * g[i] * (cand[i] / L))) for i in range(n)]   # Eq. 7

    mu_loc, sd_loc, margin = [], [], []
    for i in range(n):                                                 # Eq. 8-10
        nb = [chat[j] for j in range(max(0, i - w[i]), min(n, i + w[i] + 1)) if j != i]
        m_i, s_i = _mean_std(nb)
        mu_loc.append(m_i)
        sd_loc.append(s_i)
        margin.append(chat[i] - (m_i - p.lam * s_i))
    chosen = [i for i in range(n) if margin[i] < 0.0]

    n_min = min(n, int(math.ceil(p.min_ratio * L - 1e-9)))
    n_max = min(n, int(math.floor(p.max_ratio * L + 1e-9)))
    n_min = min(n_min, n_max)
    order = sorted(range(n), key=lambda i: (margin[i], i))
    if len(chosen) < n_min:
        have = set(chosen)
        for i in order:
            if len(have) >= n_min:
                break
            have.add(i)
        chosen = sorted(have)
    elif len(chosen) > n_max:
        have = set(chosen)
        chosen = sorted([i for i in order if i in have][:n_max])
    for i in chosen:
        mask[cand[i]] = 1
    if detail:
        return mask, {"cand": cand, "chat": chat, "g": g, "n_flat": n_flat, "w_max": w_max, "w": w,
                      "mu_local": mu_loc, "sigma_local": sd_loc, "margin": margin,
                      "n_min": n_min, "n_max": n_max}
    return mask


def uniform_skip(L: int, params: SelectParams = SelectParams()) -> np.ndarray:
    """Initial draft model: every second candidate layer skipped (Section 3, "uniformly skipping
    layers"), never more than the maximum ratio."""
    cand = list(range(1, L - 1)) if params.protect_ends else list(range(L))
    n_max = min(len(cand), int(math.floor(params.max_ratio * L + 1e-9)))
    mask = np.zeros(L, np.uint8)
    picked = [cand[i] for i in range(0, len(cand), 2)][:n_max]
    for l in picked:
        mask[l] = 1
    return mask
