"""Greedy self-speculative decoding on top of the reference decoder (TEST INFRASTRUCTURE).

Follows the generation step of Figure 2 / Section 3: the draft model (target model minus the
skip set S) proposes k tokens one at a time, the full model scores the pending token plus the
k proposals in one pass, and the longest prefix of proposals that equals the full model's own
greedy choices is kept, followed by the full model's token at the first mismatch (greedy
verification keeps the target model's output, Section 4.2.2).

State convention: committed tokens t_0..t_{n-1}; the cache holds verified K/V for positions
0..n-2; the last committed token is "pending" (not yet in the cache).
"""
from __future__ import annotations

from collections import deque
from typing import Callable, List, Optional, Sequence

import numpy as np

from .decoder import OracleModel, argmax_lowest, DEFAULT_CLAMP, DEFAULT_EPS


class OracleSSD:
    def __init__(self, model: OracleModel, window: int = 100):
        self.m = model
        # context window of the confidence extraction (Section 4.1.1: 100 tokens): hidden-state taps [L][2][d] of the
        # last `window` positions that the full model has processed with a committed input token -- the last prompt
        # position and every verified row whose token was kept
        self.window_taps = deque(maxlen=int(window))
        self.tokens: List[int] = []
        self.last_taps: Optional[np.ndarray] = None    # [rows][L][2][d] of the last verify / prefill
        self.last_logits: Optional[np.ndarray] = None
        self.last_draft_logits: List[np.ndarray] = []   # logits of each step of the last draft
        self.drafted = 0
        self.accepted = 0
        self.cycles = 0

    # number of committed tokens
    @property
    def n(self) -> int:
        return len(self.tokens)

    @property
    def pending(self) -> int:
        return self.tokens[-1]

    def prefill(self, prompt: Sequence[int], chunk=None, on_chunk=None) -> int:
        """Full model over the prompt; commits the first new token.  chunk: feed the prompt in pieces of that many
        rows (the cache makes this the same computation); on_chunk(rows_done) is called after each piece, so that a
        caller can report progress on a large model."""
        prompt = [int(t) for t in prompt]
        step = len(prompt) if not chunk else int(chunk)
        for a in range(0, len(prompt), step):
            out = self.m.forward(prompt[a:a + step], a, want_taps=True)
            if on_chunk is not None:
                on_chunk(min(a + step, len(prompt)))
        first = argmax_lowest(out["logits"][-1])
        self.tokens = prompt + [first]
        self.last_taps = out["taps"][-1:]
        self.last_logits = out["logits"][-1:]
        self.window_taps.clear()
        self.window_taps.append(self.last_taps[0])
        return first

    def decode(self) -> int:
        """One vanilla autoregressive step with the full model; commits its token."""
        out = self.m.forward([self.pending], self.n - 1)
        t = argmax_lowest(out["logits"][0])
        self.last_logits = out["logits"]
        self.tokens.append(t)
        return t

    def draft(self, skip_mask, k: int, want_maxprob=False):
        """k greedy tokens from the draft model; its K/V rows land at positions n-1..n+k-2."""
        d, mp = [], []
        tok, pos = self.pending, self.n - 1
        self.last_draft_logits = []
        for _ in range(k):
            out = self.m.forward([tok], pos, skip_mask=skip_mask)
            z = out["logits"][0]
            self.last_draft_logits.append(z)
            tok = argmax_lowest(z)
            if want_maxprob:
                e = np.exp(z - z.max())
                mp.append(float(e.max() / e.sum()))
            d.append(tok)
            pos += 1
        return (d, mp) if want_maxprob else d

    def draft_adaptive(self, skip_mask, k_max: int, gamma: float):
        """Confidence-aware drafting (Section 3: candidates are generated "following the confidence-aware approach"
        of the draft-exit baseline): tokens are drafted one at a time and drafting stops after the first token whose
        draft soft-max probability is below gamma, or after k_max tokens.  The low-confidence token itself is kept
        (it has been generated; verification decides).  Returns (tokens, their max-probabilities)."""
        d, mp = [], []
        tok, pos = self.pending, self.n - 1
        self.last_draft_logits = []
        while len(d) < k_max:
            z = self.m.forward([tok], pos, skip_mask=skip_mask)["logits"][0]
            self.last_draft_logits.append(z)
            tok = argmax_lowest(z)
            e = np.exp(z - z.max())
            p = float(e.max() / e.sum())
            d.append(tok)
            mp.append(p)
            pos += 1
            if p < gamma:
                break
        return d, mp

    def verify(self, draft: Sequence[int]):
        """Full model over [pending, d_1..d_k]; returns its greedy token after each row."""
        rows = [self.pending] + [int(t) for t in draft]
        out = self.m.forward(rows, self.n - 1, want_taps=True)
        self.last_taps = out["taps"]
        self.last_logits = out["logits"]
        return [argmax_lowest(z) for z in out["logits"]]

    def accept(self, draft: Sequence[int], target: Sequence[int]):
        """a = longest prefix with d_j == y_{j-1}; commit d_1..d_a and y_a. Returns (a, y_a)."""
        k = len(draft)
        assert len(target) == k + 1
        a = 0
        while a < k and int(draft[a]) == int(target[a]):
            a += 1
        self.tokens.extend(int(t) for t in draft[:a])
        self.tokens.append(int(target[a]))
        # verify rows 0..a were fed committed tokens (the pending one and the accepted drafts): they enter the window
        taps = getattr(self, "last_taps", None)
        if taps is not None and len(taps) == k + 1:
            for j in range(a + 1):
                self.window_taps.append(taps[j])
        self.drafted += k
        self.accepted += a
        self.cycles += 1
        return a, int(target[a])

    def force_commit(self, toks: Sequence[int]):
        self.tokens.extend(int(t) for t in toks)

    def layer_confidence(self, row: int = 0, clamp=DEFAULT_CLAMP, eps=DEFAULT_EPS, taps: int = 2):
        """Per-layer confidence of one row of the last verify/prefill.

        taps=2: mean of the confidences of the post-attention and post-MLP hidden states
        (the "FFNN and Attention" hidden states of Section 3.1); taps=1: post-MLP only.
        Returns (conf[L], per_tap dict with conf/maxprob/argmax arrays shaped [L][2]).
        """
        t = self.last_taps[row]                      # [L][2][d]
        L = t.shape[0]
        r = self.m.confidence(t.reshape(L * 2, -1), clamp=clamp, eps=eps)
        c = r["conf"].reshape(L, 2)
        per = {k_: v.reshape(L, 2) for k_, v in r.items()}
        conf = (c[:, 0] + c[:, 1]) / 2.0 if taps == 2 else c[:, 1].copy()
        return conf, per


    def window_confidence(self, clamp=DEFAULT_CLAMP, eps=DEFAULT_EPS, taps: int = 2):
        """Per-layer confidence over the context window (Section 4.1.1): Eq. 1-4 on every tapped hidden state of
        every position in the window, averaged over the positions; a layer's value is the mean of its two taps
        (taps=2) or its post-MLP tap (taps=1).  Returns (conf[L], per-tap means [L][2], positions in the window)."""
        n = len(self.window_taps)
        t = np.stack(list(self.window_taps))           # [n][L][2][d]
        L = t.shape[1]
        c = self.m.confidence(t.reshape(n * L * 2, -1), clamp=clamp, eps=eps)["conf"].reshape(n, L, 2)
        per_tap = c.mean(axis=0)
        conf = (per_tap[:, 0] + per_tap[:, 1]) / 2.0 if taps == 2 else per_tap[:, 1].copy()
        return conf, per_tap, n


def generate_vanilla(model: OracleModel, prompt: Sequence[int], n_new: int) -> List[int]:
    s = OracleSSD(model)
    s.prefill(prompt)
    while s.n - len(prompt) < n_new:
        s.decode()
    return s.tokens[len(prompt):len(prompt) + n_new]


def generate_ssd(model: OracleModel, prompt: Sequence[int], n_new: int, k: int, skip_mask,
                 on_cycle: Optional[Callable] = None):
    """Greedy SSD until n_new tokens exist (the surplus of the last cycle is dropped).

    skip_mask: array[L] of 0/1, or a callable(state) -> mask evaluated before every cycle.
    on_cycle(state, draft, target, a) is called after each accept (search drivers hook in here).
    Returns (new tokens, dict(accepted per cycle, drafted, accepted, cycles)).
    """
    s = OracleSSD(model)
    s.prefill(prompt)
    per_cycle = []
    P = len(prompt)
    while s.n - P < n_new:
        mask = skip_mask(s) if callable(skip_mask) else skip_mask
        d = s.draft(mask, k)
        y = s.verify(d)
        a, _ = s.accept(d, y)
        per_cycle.append(a)
        if on_cycle is not None:
            on_cycle(s, d, y, a)
    stats = {"accepted_per_cycle": per_cycle, "drafted": s.drafted, "accepted": s.accepted,
             "cycles": s.cycles}
    return s.tokens[P:P + n_new], stats
