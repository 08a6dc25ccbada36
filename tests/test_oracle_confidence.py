"""Pins of the entropy confidence (Eq. 1-4) and of the per-layer confidence built on it."""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import OracleModel, OracleSSD, confidence_from_logits, argmax_lowest
from synth import ModelShape, WORKLOADS, make_prompt, make_weights

EPS = 1e-10


def test_uniform_logits_give_closed_form_near_zero():
    for V in (7, 1024, 32000):
        c, mp, am = confidence_from_logits(np.full(V, 3.25), eps=EPS)
        assert c == pytest.approx(1.0 + math.log(1.0 / V + EPS) / math.log(V), abs=1e-12)
        assert abs(c) < 1e-5 and mp == pytest.approx(1.0 / V) and am == 0


def test_peaked_logits_give_one():
    z = np.full(1000, -50.0)
    z[321] = 50.0
    c, mp, am = confidence_from_logits(z)
    assert c == pytest.approx(1.0, abs=1e-9) and mp == pytest.approx(1.0) and am == 321


def test_two_equal_maxima_closed_form_and_lowest_index_tie():
    V = 4096
    z = np.full(V, -1e4)
    z[[100, 7]] = 1e4
    c, mp, am = confidence_from_logits(z)
    assert c == pytest.approx(1.0 - math.log(2.0) / math.log(V), abs=1e-9)
    assert mp == pytest.approx(0.5) and am == 7
    assert argmax_lowest(np.array([1.0, 5.0, 5.0, 2.0])) == 1


def test_matches_scipy_entropy_and_softmax_and_stays_in_unit_interval():
    rng = np.random.default_rng(0)
    for V, scale in ((50, 1.0), (1024, 3.0), (32000, 0.5), (32000, 8.0)):
        z = rng.normal(0, scale, V).astype(np.float32).astype(np.float64)
        c, mp, am = confidence_from_logits(z, eps=EPS)
        p = scipy.special.softmax(z)
        ref = 1.0 - scipy.stats.entropy(p) / math.log(V)      # epsilon-free Shannon entropy
        assert abs(c - ref) <= V * EPS / math.log(V) + 1e-12   # epsilon shifts H by at most V*eps
        assert 0.0 <= c <= 1.0
        assert mp == pytest.approx(p.max(), rel=1e-12) and am == int(np.argmax(z))


def test_invariant_to_adding_a_constant():
    rng = np.random.default_rng(1)
    z = np.round(rng.normal(0, 2, 500) * 64) / 64            # exactly representable, so is z + 16
    a = confidence_from_logits(z)
    b = confidence_from_logits(z + 16.0)
    assert a[0] == pytest.approx(b[0], abs=1e-13) and a[2] == b[2]


def test_clamp_tames_infinite_and_huge_logits():
    z = np.array([np.inf, 0.0, -np.inf, 1e30, -1e30])
    c, mp, am = confidence_from_logits(z, clamp=1e4)
    # +inf and 1e30 both clamp to 1e4: two equal maxima among 5
    assert np.isfinite(c) and c == pytest.approx(1.0 - math.log(2) / math.log(5), abs=1e-9)
    assert mp == pytest.approx(0.5) and am == 0
    c2, _, _ = confidence_from_logits(np.array([3.0, 1.0, 0.5]), clamp=1.0)   # clamp changes the result
    c3, _, _ = confidence_from_logits(np.array([1.0, 1.0, 0.5]), clamp=1e4)
    assert c2 == pytest.approx(c3, abs=1e-15)


def test_logits_are_rounded_to_fp32_first():
    z = np.array([1.0 + 2.0 ** -30, 1.0, 0.0])        # the first two are equal once cast to fp32
    _, mp, am = confidence_from_logits(z)
    assert am == 0 and mp == pytest.approx(math.e / (2 * math.e + 1))


def _brute_force_conf(hidden, gain, lm_head, rms_eps):
    h = hidden / np.sqrt(np.mean(hidden * hidden) + rms_eps) * gain
    z = (lm_head @ h).astype(np.float32).astype(np.float64)
    p = scipy.special.softmax(z)
    return 1.0 - scipy.stats.entropy(p) / math.log(len(z)), p.max(), int(np.argmax(z))


@pytest.mark.parametrize("shape", [WORKLOADS["tiny"].shape, ModelShape(3, 64, 4, 2, 96, 211, dtype="bf16")])
def test_layer_confidence_equals_brute_force_per_layer_head(shape):
    # larger init so that the intermediate distributions are far from uniform
    w = make_weights(shape, 4, norm_gain_std=0.2, init_std=0.25)
    m = OracleModel(shape, w, 48)
    s = OracleSSD(m)
    s.prefill(make_prompt(shape.vocab, 20, 8).tolist())
    d = s.draft(np.zeros(shape.n_layers, np.uint8), 3)
    y = s.verify(d)
    gain = w["final_norm"].double().numpy()
    head = w["lm_head"].double().numpy()
    for row in range(4):
        conf, per = s.layer_confidence(row)
        for l in range(shape.n_layers):
            for t in range(2):
                c, mp, am = _brute_force_conf(s.last_taps[row, l, t], gain, head, shape.rms_eps)
                assert per["conf"][l, t] == pytest.approx(c, abs=1e-6)
                assert per["maxprob"][l, t] == pytest.approx(mp, rel=1e-9)
                assert per["argmax"][l, t] == am
            assert conf[l] == pytest.approx((per["conf"][l, 0] + per["conf"][l, 1]) / 2, abs=1e-15)
        conf1, _ = s.layer_confidence(row, taps=1)
        assert np.array_equal(conf1, per["conf"][:, 1])
        # the last layer's output tap is the hidden state the verify logits came from
        assert per["argmax"][shape.n_layers - 1, 1] == y[row]
    assert np.ptp(per["conf"]) > 1e-3


def test_last_tap_reproduces_verify_logits_exactly():
    wl = WORKLOADS["tiny"]
    w = make_weights(wl.shape, wl.seed)
    m = OracleModel(wl.shape, w, 64)
    toks = make_prompt(wl.shape.vocab, 10, 3).tolist()
    out = m.forward(toks, 0, want_taps=True, want_hidden=True)
    assert np.array_equal(out["taps"][:, -1, 1], out["hidden"])
    r = m.confidence(out["taps"][:, -1, 1], want_logits=True)
    assert np.array_equal(r["logits"], out["logits"])


def test_taps_of_a_skipped_layer_equal_its_input():
    wl = WORKLOADS["tiny"]
    w = make_weights(wl.shape, wl.seed)
    m = OracleModel(wl.shape, w, 16)
    out = m.forward([5, 6], 0, skip_mask=np.array([0, 1, 0, 0], np.uint8), want_taps=True)
    t = out["taps"]
    assert np.array_equal(t[:, 1, 0], t[:, 0, 1]) and np.array_equal(t[:, 1, 1], t[:, 0, 1])
    assert not np.array_equal(t[:, 2, 0], t[:, 1, 1])


def test_window_confidence_is_the_mean_over_the_last_committed_positions():
    """Context window (Section 4.1.1): the windowed confidence equals the mean of per-position confidences
    recomputed by brute force -- a full-sequence recompute of the committed tokens with the library-op
    reference, scipy's softmax for Eq. 1-4 -- over the last W processed positions (from the last prompt position
    on), whatever mix of accepted and rejected drafts produced them."""
    from tests._reference import reference_confidence, reference_forward
    wl = WORKLOADS["tiny"]
    shape = wl.shape
    w = make_weights(shape, wl.seed)
    prompt = make_prompt(shape.vocab, 9, 3).tolist()
    P = len(prompt)
    for W in (5, 100):
        s = OracleSSD(OracleModel(shape, w, 96), window=W)
        s.prefill(prompt)
        accepted = []
        for mask in ([0, 0, 0, 0], [0, 1, 0, 0], [0, 0, 0, 0], [0, 1, 1, 0], [0, 0, 0, 0]):
            d = s.draft(np.array(mask, np.uint8), 3)
            accepted.append(s.accept(d, s.verify(d))[0])
        assert len(set(accepted)) > 1                       # both full and partial acceptance occurred
        conf, per_tap, n = s.window_confidence()
        # positions processed with a committed input: P-1 (last prompt token) .. n-2 (the pending token is not yet)
        first, last = P - 1, s.n - 2
        assert n == min(W, last - first + 1)
        _, taps = reference_forward(shape, w, s.tokens[:-1], kv_storage="model")
        pos = list(range(last - n + 1, last + 1))
        ref = np.array([[[reference_confidence(shape, w, taps[p, l, t]) for t in range(2)]
                         for l in range(shape.n_layers)] for p in pos])
        np.testing.assert_allclose(per_tap, ref.mean(axis=0), rtol=0, atol=1e-12)
        np.testing.assert_allclose(conf, ref.mean(axis=(0, 2)), rtol=0, atol=1e-12)
