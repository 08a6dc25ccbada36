"""The oracle still reproduces the stored tiny-workload fixture (written by tests/golden/make_golden.py,
which calls the oracle only)."""
import importlib.util
import json
import os

import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_tiny_fixture_is_reproduced():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(GOLD, "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    ref = json.load(open(os.path.join(GOLD, "tiny_oracle.json")))
    for key in ("prompt", "vanilla_tokens", "first_draft", "first_target", "skip_mask", "ssd_accepted_per_cycle"):
        assert now[key] == ref[key], key
    assert now["layer_confidence_row0"] == pytest.approx(ref["layer_confidence_row0"], abs=1e-12)
    assert len(ref["vanilla_tokens"]) == 32 and ref["first_draft"] == ref["first_target"][:4]
