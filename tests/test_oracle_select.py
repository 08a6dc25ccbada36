"""Pins of the skip-set selection (Eq. 5-10) and of the periodic search.

Parity with the authors' implementation is unpinned (the paper leaves stencil, window
rounding and ratio enforcement open); what is pinned: printed hyper-parameters, two vectors
worked by hand from the stated reading, the constant-window special case against an
independent vectorised NumPy evaluation, and the invariants the text states.
"""
import json
import math
import os

import numpy as np
import pytest
import scipy.stats

from oracle import SearchDriver, SelectParams, select_skip, uniform_skip

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_defaults_are_the_papers_hyperparameters():
    hp = json.load(open(os.path.join(GOLD, "paper_hparams.json")))
    p = SelectParams()
    assert p.w_base == hp["w_base"]
    assert hp["lambda_range_exclusive"][0] < p.lam < hp["lambda_range_exclusive"][1]
    assert p.min_ratio == hp["min_skip_ratio"] == hp["best_skip_ratio_range"][0]
    assert p.max_ratio == hp["best_skip_ratio_range"][1]
    d = SearchDriver(40)
    assert d.opt_interval == hp["search_interval"] and d.score_goal == hp["score_goal_accepted_tokens"]
    assert d.ring.maxlen == hp["context_window"]
    assert len([l for l in range(40) if l not in (0, 39)]) == hp["considered_layers_of_40"]
    assert p.protect_ends


def test_hand_worked_vector_12_layers():
    conf = [.05, .10, .10, .10, .12, .30, .28, .50, .45, .70, .90, .95]
    mask, d = select_skip(conf, SelectParams(lam=0.3), detail=True)
    assert d["n_flat"] == 3 and d["w"] == [2, 2, 2, 2, 2, 2, 2, 3, 3, 2]
    assert np.flatnonzero(mask).tolist() == [2, 3, 4, 6, 8]
    # spot values worked by hand: candidates 1..10, mean 0.355, population std
    c = np.array(conf[1:11])
    assert d["chat"][0] == pytest.approx((0.10 - c.mean()) / (c.std() + 1e-8), rel=1e-12)
    # first candidate: neighbours are candidates 1, 2 (both 0.10) -> sigma_local 0, margin 0 -> not skipped (strict <)
    assert d["sigma_local"][0] == 0.0 and d["margin"][0] == 0.0 and mask[1] == 0


def test_hand_worked_vector_4_layers_fill_to_minimum():
    mask, d = select_skip([.2, .1, .3, .4], SelectParams(protect_ends=False, max_ratio=0.5), detail=True)
    assert [i for i in range(4) if d["margin"][i] < 0] == [1]
    assert (d["n_min"], d["n_max"]) == (2, 2)
    assert np.flatnonzero(mask).tolist() == [0, 1]


def test_standardisation_matches_scipy_zscore():
    rng = np.random.default_rng(3)
    conf = rng.uniform(0, 1, 30)
    _, d = select_skip(conf, SelectParams(eps=0.0), detail=True)
    np.testing.assert_allclose(d["chat"], scipy.stats.zscore(conf[1:-1]), rtol=1e-12, atol=1e-13)


def _constant_window_reference(conf, lam, w):
    """Eq. 5, 8-10 with a constant half-width w, vectorised with NumPy (no ratio bounds)."""
    c = np.asarray(conf, dtype=np.float64)[1:-1]
    z = (c - c.mean()) / (c.std() + 1e-8)
    n = len(z)
    out = []
    for i in range(n):
        idx = np.array([j for j in range(i - w, i + w + 1) if 0 <= j < n and j != i])
        out.append(bool(z[i] < z[idx].mean() - lam * z[idx].std()))
    return np.array(out)


@pytest.mark.parametrize("seed", range(8))
def test_constant_window_special_case(seed):
    rng = np.random.default_rng(seed)
    L = int(rng.integers(8, 60))
    conf = rng.uniform(0, 1, L)
    lam = float(rng.uniform(0.25, 0.5))
    p = SelectParams(lam=lam, fixed_w_max=0.0, min_ratio=0.0, max_ratio=1.0)
    mask, d = select_skip(conf, p, detail=True)
    assert d["w"] == [2] * (L - 2)
    ref = _constant_window_reference(conf, lam, 2)
    assert np.array_equal(mask[1:-1].astype(bool), ref)


def test_window_grows_with_gradient_and_depth():
    # flat start of 6 layers -> w_max = 6; a single kink late in the stack gets the widest window
    conf = [0.5] * 8 + [0.5, 0.5, 0.9, 0.5, 0.5] + [0.5] * 3
    _, d = select_skip(conf, SelectParams(), detail=True)
    assert d["n_flat"] == 9 and d["w_max"] == 9.0        # candidates 1..9 are flat
    g = np.array(d["g"])
    assert g.min() == 0.0 and g.max() == pytest.approx(1.0, abs=1e-6)
    i = int(np.argmax(g))
    L = len(conf)
    assert d["w"][i] == math.floor(2 + 9.0 * g[i] * (d["cand"][i] / L))
    assert all(wi >= 2 for wi in d["w"]) and d["w"][0] == 2
    # the same kink earlier in the stack gets a smaller window (depth factor l_i / num_layers)
    conf2 = [0.5] * 3 + [0.9] + [0.5] * 12
    _, d2 = select_skip(conf2, SelectParams(fixed_w_max=9.0), detail=True)
    assert max(d2["w"]) < d["w"][i]


@pytest.mark.parametrize("seed", range(20))
def test_invariants(seed):
    rng = np.random.default_rng(100 + seed)
    L = int(rng.integers(4, 90))
    conf = rng.uniform(0, 1, L) if seed % 3 else np.round(rng.uniform(0, 1, L), 1)
    protect = bool(seed % 2)
    p = SelectParams(lam=float(rng.uniform(0.25, 0.5)), protect_ends=protect)
    mask, d = select_skip(conf, p, detail=True)
    assert mask.dtype == np.uint8 and set(np.unique(mask)) <= {0, 1}
    if protect:
        assert mask[0] == 0 and mask[-1] == 0
    assert d["n_min"] <= int(mask.sum()) <= d["n_max"]
    assert d["n_max"] <= math.floor(0.6 * L + 1e-9)
    assert np.array_equal(mask, select_skip(conf, p))                       # deterministic
    # a constant shift of all confidences cancels in Eq. 5 (exact for dyadic shifts of rounded inputs)
    if seed % 3 == 0:
        pass
    else:
        m2 = select_skip(np.asarray(conf) * 0.5, SelectParams(**{**p.__dict__, "flat_tol": p.flat_tol * 0.5}))
        assert np.array_equal(mask, m2)                                     # scale-invariant too


def test_degenerate_inputs():
    assert select_skip([0.3, 0.4], SelectParams()).sum() == 0              # no candidates
    assert select_skip([0.3], SelectParams(protect_ends=False)).tolist() in ([0], [1])
    m = select_skip([0.5] * 10, SelectParams())                             # all equal: margins 0, filled by index
    assert np.flatnonzero(m).tolist() == [1, 2, 3, 4]
    assert select_skip([], SelectParams()).shape == (0,)


def test_uniform_initial_set():
    m = uniform_skip(40)
    assert np.flatnonzero(m).tolist() == list(range(1, 39, 2)) and m[0] == 0 and m[39] == 0
    m = uniform_skip(10, SelectParams(max_ratio=0.3))
    assert m.sum() == 3
    assert np.flatnonzero(uniform_skip(4, SelectParams(protect_ends=False))).tolist() == [0, 2]


# ---- periodic search (Section 3.3) ----------------------------------------------------------

def _run(driver, accepted_of_mask, n_cycles, rng):
    masks = []
    for _ in range(n_cycles):
        a = accepted_of_mask(driver.mask)
        conf = rng.uniform(0, 1, driver.L)
        masks.append(driver.observe(a, conf).copy())
    return masks


def test_search_halts_on_goal_and_keeps_best():
    rng = np.random.default_rng(0)
    d = SearchDriver(24, opt_interval=5, score_goal=4.0, max_rounds=10)
    first = d.mask.copy()
    _run(d, lambda m: 4, 5, rng)
    assert not d.active and d.rounds == 1 and d.best_score == 4.0
    assert np.array_equal(d.mask, first)
    before = d.mask.copy()
    _run(d, lambda m: 0, 20, rng)                       # halted: nothing changes any more
    assert np.array_equal(d.mask, before) and d.rounds == 1


def test_search_runs_max_rounds_and_best_score_is_monotone():
    rng = np.random.default_rng(1)
    d = SearchDriver(24, opt_interval=3, score_goal=99.0, max_rounds=6)
    scores_seen, best_trace = [], []
    for _ in range(40):
        a = int(d.mask[:12].sum()) % 4                  # score depends on the set
        d.observe(a, rng.uniform(0, 1, 24))
        best_trace.append(d.best_score)
    assert d.rounds <= 6 and not d.active
    assert all(b2 >= b1 for b1, b2 in zip(best_trace, best_trace[1:]))
    assert d.best_score == max(s for _, s, _ in d.history)
    best_masks = [m for _, s, m in d.history if s == d.best_score]
    assert np.array_equal(d.mask, best_masks[0])
    keys = [m.tobytes() for _, _, m in d.history]
    assert len(set(keys)) == len(keys)                  # never scores the same set twice


def test_search_is_deterministic_and_uses_interval():
    def trace(seed):
        rng = np.random.default_rng(seed)
        d = SearchDriver(16, opt_interval=4, score_goal=9.0, max_rounds=3)
        return [m.tobytes() for m in _run(d, lambda m: 1, 14, rng)], d
    a, da = trace(5)
    b, _ = trace(5)
    assert a == b
    assert a[0] == a[1] == a[2] and da.rounds == 3       # the set only changes every 4th cycle
    assert a[4] == a[5] == a[6]


def test_window_of_confidences_is_a_ring():
    d = SearchDriver(6, opt_interval=1000, window=3)
    for i in range(5):
        d.observe(0, np.full(6, float(i)))
    np.testing.assert_allclose(d.mean_confidence(), np.full(6, 3.0))
