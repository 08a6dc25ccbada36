"""The stored tiny-workload fixture (tests/golden/tiny_oracle.json, written by tests/golden/make_golden.py, which calls
the oracle only) is pinned twice: the oracle still reproduces it, and every value in it is recomputed here by brute
force -- full-sequence recomputes with the library-op reference of tests/_reference.py (no cache, no incremental
state), scipy's softmax for Eq. 1-4 -- so the fixture does not rest on the oracle's own output."""
import importlib.util
import json
import os

import numpy as np
import pytest

from synth import WORKLOADS, make_weights
from tests._reference import reference_confidence, reference_forward

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _fixture():
    return json.load(open(os.path.join(GOLD, "tiny_oracle.json")))


def test_tiny_fixture_is_reproduced():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(GOLD, "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    ref = _fixture()
    for key in ("prompt", "vanilla_tokens", "first_draft", "first_target", "skip_mask", "ssd_accepted_per_cycle"):
        assert now[key] == ref[key], key
    assert now["layer_confidence_row0"] == pytest.approx(ref["layer_confidence_row0"], abs=1e-12)
    assert len(ref["vanilla_tokens"]) == 32 and ref["first_draft"] == ref["first_target"][:4]


def _argmax_lowest(z):
    return int(np.flatnonzero(z == z.max())[0])


def test_tiny_fixture_equals_brute_force_recompute():
    fx = _fixture()
    wl = WORKLOADS["tiny"]
    shape = wl.shape
    w = make_weights(shape, wl.seed)
    prompt = fx["prompt"]
    P, k = len(prompt), wl.k
    # vanilla greedy tokens: one full recompute per new token
    seq = list(prompt)
    for _ in range(wl.new_tokens):
        seq.append(_argmax_lowest(reference_forward(shape, w, seq)[0][-1]))
    assert seq[P:] == fx["vanilla_tokens"]
    # first cycle with the empty skip set: the draft is the full model, so its tokens are the greedy continuation,
    # and the verify rows [pending, d_1..d_k] give the next k + 1 greedy tokens
    assert fx["first_draft"] == seq[P + 1:P + 1 + k]
    assert fx["first_target"] == seq[P + 1:P + 2 + k]
    # confidence of the first verify row (position P, the pending token): Eq. 1-4 on its two taps per layer
    _, taps = reference_forward(shape, w, seq[:P + 1 + k])
    tap_conf = [[reference_confidence(shape, w, taps[P, l, t]) for t in range(2)] for l in range(shape.n_layers)]
    np.testing.assert_allclose(tap_conf, fx["tap_confidence_row0"], rtol=0, atol=1e-12)
    np.testing.assert_allclose(np.mean(tap_conf, axis=1), fx["layer_confidence_row0"], rtol=0, atol=1e-12)
    # greedy SSD with the stored skip set: drafts by recomputing the draft rows on top of the verified prefix
    mask = np.array(fx["skip_mask"], np.uint8)
    committed = seq[:P + 1]
    accepted = []
    while len(committed) - P < wl.new_tokens:
        n = len(committed)
        rows = list(committed)
        for _ in range(k):
            z, _ = reference_forward(shape, w, rows, skip_mask=mask, n_verified=n - 1)
            rows.append(_argmax_lowest(z[-1]))
        d = rows[n:]
        zt, _ = reference_forward(shape, w, rows)
        y = [_argmax_lowest(zt[j]) for j in range(n - 1, n + k)]
        a = 0
        while a < k and d[a] == y[a]:
            a += 1
        committed += d[:a] + [y[a]]
        accepted.append(a)
    assert accepted == fx["ssd_accepted_per_cycle"]
    assert committed[P:P + wl.new_tokens] == fx["vanilla_tokens"]
