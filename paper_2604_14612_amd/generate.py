"""Host-side generation loops over the C-ABI calls (no arithmetic here: every step runs in the library).

generate_conflayers follows the generation process of Section 3 / Figure 2: start from uniform layer skipping,
draft k tokens with the current skip set (or with the confidence-aware draft exit when gamma is given), verify
them in one pass of the full model, accept greedily, and -- while the search is active -- feed the cycle's
accepted count and the per-layer confidence of its first verify row to the interval-based search (Section 3.3),
which may install a new skip set.  With windowed=True the confidences come from the context window instead (Section
4.1.1: the hidden states of the last 100 positions, kept on the device): nothing is computed per cycle, and one pass
over the whole window runs on the cycle that completes a search interval.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

from .binding import Context, Search, search_defaults, select_defaults


def generate_vanilla(ctx: Context, prompt: Sequence[int], n_new: int) -> List[int]:
    """n_new greedy tokens from the full model, one per step."""
    out = [ctx.ssd_prefill(prompt)]
    while len(out) < n_new:
        out.append(ctx.ssd_decode())
    return out[:n_new]


def generate_conflayers(ctx: Context, prompt: Sequence[int], n_new: int, k: int = 4, search: Optional[Search] = None,
                        gamma: Optional[float] = None, windowed: bool = False, opt_interval: int = 30):
    """n_new greedy tokens by self-speculative decoding with the skip set under search.

    search: a Search handle (default: the paper's hyper-parameters for this depth); gamma: draft-exit threshold of
    the confidence-aware drafting, None = always k drafts; windowed: take the confidences from ssd_window_confidence (the
    context needs conf_window > 0, the Search handle window = 1 and the same opt_interval as given here).  Returns (tokens, stats) where stats has the number of
    cycles, drafted and accepted tokens, search rounds and the final skip mask."""
    L = ctx.shape.n_layers
    own = search is None
    if own:
        search = Search(L, search_defaults(opt_interval=opt_interval, **({"window": 1} if windowed else {})), select_defaults())
    out = [ctx.ssd_prefill(prompt)]
    cycles = drafted = accepted = 0
    while len(out) < n_new:
        mask = search.mask()
        if gamma is None:
            d = ctx.ssd_draft_step(mask, k)
        else:
            d, _ = ctx.ssd_draft_adaptive(mask, k, gamma)
        y = ctx.ssd_verify(d)
        a, nxt = ctx.ssd_accept(d, y)
        if not search.active:
            conf = None
        elif windowed:      # one pass over the window, on the cycle that completes an interval
            conf = ctx.ssd_window_confidence() if (cycles + 1) % opt_interval == 0 else None
        else:
            conf = ctx.ssd_layer_confidence(0, 1)[0]
        search.observe(a, conf)
        out += d[:a] + [nxt]
        cycles += 1
        drafted += len(d)
        accepted += a
    rounds, best = search.status()
    stats = {"cycles": cycles, "drafted": drafted, "accepted": accepted, "search_rounds": rounds,
             "search_best_score": best, "skip_mask": search.mask()}
    if own:
        search.close()
    return out[:n_new], stats
