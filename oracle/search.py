"""Interval-based periodic search for the skip set (TEST INFRASTRUCTURE; Section 3.3).

PARITY UNPINNED against the authors' implementation: the paper gives the control flow in
prose only (Figure 2, Section 3 and 3.3) and no values for the maximum number of rounds.
The reading implemented here:
  * start from uniform layer skipping;
  * every generation cycle contributes its accepted-token count and one per-layer confidence
    vector; the vectors of the most recent `window` cycles (context window of 100,
    Section 4.1.1) are averaged when a new set is searched;
  * a skip set is used for `opt_interval` cycles; then score = mean accepted tokens per cycle;
    the best-scoring set so far is remembered;
  * the search halts when score >= score_goal (4 accepted tokens, Section 4.1.1) or after
    max_rounds rounds, and the best set is used from then on;
  * otherwise the next set comes from Eq. 5-10 on the averaged confidences; a set that was
    already scored is shrunk (its member with the largest margin is dropped) until it is new,
    and the search halts if that would go below the minimum skip ratio.
"""
from __future__ import annotations

from collections import deque
from typing import Optional

import numpy as np

from .select_skip import SelectParams, select_skip, uniform_skip


class SearchDriver:
    def __init__(self, n_layers: int, params: SelectParams = SelectParams(), opt_interval: int = 30,
                 score_goal: float = 4.0, max_rounds: int = 10, window: int = 100):
        self.L = n_layers
        self.params = params
        self.opt_interval = opt_interval
        self.score_goal = score_goal
        self.max_rounds = max_rounds
        self.ring = deque(maxlen=window)
        self.mask = uniform_skip(n_layers, params)
        self.best_mask = self.mask.copy()
        self.best_score = -1.0
        self.active = True
        self.rounds = 0
        self.iters = 0
        self.acc = 0
        self.evaluated = set()
        self.history = []          # (round, score, mask) per finished interval

    def mean_confidence(self) -> np.ndarray:
        out = np.zeros(self.L, np.float64)
        for l in range(self.L):
            s = 0.0
            for v in self.ring:
                s += float(v[l])
            out[l] = s / len(self.ring)
        return out

    def observe(self, n_accepted: int, conf: Optional[np.ndarray]) -> np.ndarray:
        """Feed one finished cycle; returns the mask to use for the next cycle."""
        if not self.active:
            return self.mask
        if conf is not None:
            self.ring.append(np.asarray(conf, dtype=np.float64).copy())
        self.acc += int(n_accepted)
        self.iters += 1
        if self.iters < self.opt_interval:
            return self.mask
        score = self.acc / self.iters
        self.iters = 0
        self.acc = 0
        self.rounds += 1
        self.evaluated.add(self.mask.tobytes())
        self.history.append((self.rounds, score, self.mask.copy()))
        if score > self.best_score:
            self.best_score = score
            self.best_mask = self.mask.copy()
        if score >= self.score_goal or self.rounds >= self.max_rounds or len(self.ring) == 0:
            self.active = False
            self.mask = self.best_mask.copy()
            return self.mask
        new, det = select_skip(self.mean_confidence(), self.params, detail=True)
        while new.tobytes() in self.evaluated:
            members = [i for i in range(len(det["cand"])) if new[det["cand"][i]]]
            if len(members) <= det["n_min"]:
                self.active = False
                self.mask = self.best_mask.copy()
                return self.mask
            drop = max(members, key=lambda i: (det["margin"][i], i))
            new = new.copy()
            new[det["cand"][drop]] = 0
        self.mask = new
        return self.mask
