"""Writes tests/golden/tiny_oracle.json from the CPU oracle alone (no HIP code is imported).

Regression fixture for the "tiny" workload: greedy tokens, per-layer confidences of the first
verify row, the skip set chosen from them and the accepted counts of greedy SSD with that set.
Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import OracleModel, OracleSSD, SelectParams, generate_ssd, generate_vanilla, select_skip  # noqa: E402
from synth import WORKLOADS, make_prompt, make_weights  # noqa: E402


def compute():
    wl = WORKLOADS["tiny"]
    w = make_weights(wl.shape, wl.seed)
    prompt = make_prompt(wl.shape.vocab, wl.prompt_len, wl.seed).tolist()
    max_seq = wl.prompt_len + wl.new_tokens + wl.k + 2
    vanilla = generate_vanilla(OracleModel(wl.shape, w, max_seq), prompt, wl.new_tokens)
    s = OracleSSD(OracleModel(wl.shape, w, max_seq))
    s.prefill(prompt)
    zero = np.zeros(wl.shape.n_layers, np.uint8)
    d = s.draft(zero, wl.k)
    y = s.verify(d)
    conf, per = s.layer_confidence(0)
    params = SelectParams(protect_ends=wl.protect_ends, max_ratio=0.5)
    mask = select_skip(conf, params)
    toks, st = generate_ssd(OracleModel(wl.shape, w, max_seq), prompt, wl.new_tokens, wl.k, mask)
    assert toks == vanilla
    return {"workload": "tiny", "prompt": prompt, "vanilla_tokens": vanilla, "first_draft": d,
            "first_target": y, "layer_confidence_row0": [float(c) for c in conf],
            "tap_confidence_row0": per["conf"].tolist(), "skip_mask": mask.tolist(),
            "ssd_accepted_per_cycle": st["accepted_per_cycle"]}


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle.json")
    with open(out, "w") as f:
        json.dump(compute(), f, indent=1)
    print("wrote", out)
