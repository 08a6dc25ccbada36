"""GPU parity on the benchmark workloads themselves (BASELINE configs 2-5): the full "small" workload,
the 7B / 13B / 70B shapes at reduced depth (the CPU oracle needs seconds per row at full depth), one
full-depth 7B pass on a short prompt, and size-independent properties on the full 7B, 13B and 70B workloads
in the launch configuration bench.py times."""
import time

import numpy as np
import pytest

from oracle import OracleSSD, SearchDriver, SelectParams, select_skip
from synth import WORKLOADS, make_prompt, reduced_depth
from tests._parity import (assert_logits_close, decisive, lockstep_ssd, make_pair, make_pair_gpu_generated)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ssd():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2604_14612_amd as lib
    lib.lib()
    return lib


def test_small_workload_full_config(ssd):
    """Config 2 as specified: 24 layers, prompt 256, 128 new tokens, k = 4, confidence-selected skip set
    (at most 50 % of the layers), every cycle in lock-step with the oracle."""
    wl = WORKLOADS["small"]
    shape = wl.shape
    orc, ctx = make_pair(shape, wl.seed, wl.prompt_len + wl.new_tokens + 2 * wl.k + 8, max_k=wl.k)
    prompt = make_prompt(shape.vocab, wl.prompt_len, wl.seed).tolist()
    op = SelectParams(max_ratio=wl.max_skip_ratio, protect_ends=wl.protect_ends)
    cp = ssd.select_defaults(max_ratio=wl.max_skip_ratio, protect_ends=int(wl.protect_ends))
    chosen = {}

    def policy(o, c, cycle, a):
        if cycle != 0:
            return None
        conf_o, _ = o.layer_confidence(0)
        conf_g = c.ssd_layer_confidence(0, 1)[0]
        np.testing.assert_allclose(conf_g, conf_o, atol=5e-3)
        mask_o = select_skip(conf_o, op)
        assert np.array_equal(ssd.ssd_select_skip(conf_o, cp), mask_o)     # identical inputs -> identical set
        chosen["mask"], chosen["gpu_mask"] = mask_o, ssd.ssd_select_skip(conf_g.astype(np.float64), cp)
        return mask_o

    t0 = time.time()
    st = lockstep_ssd(ctx, orc, prompt, wl.new_tokens, wl.k, np.zeros(shape.n_layers, np.uint8), shape.dtype,
                      next_mask=policy)
    n_skip = int(chosen["mask"].sum())
    print("small: cycles", st["cycles"], "unpinned", st["unpinned_cycles"], "max err %.2e" % st["max_err"],
          "skipped", n_skip, "mean accepted %.2f" % np.mean(st["accepted"]), "gpu-conf mask equal",
          bool(np.array_equal(chosen["mask"], chosen["gpu_mask"])), "%.0f s" % (time.time() - t0))
    assert 0.4 * shape.n_layers - 1e-9 <= n_skip <= 0.5 * shape.n_layers + 1e-9
    assert st["unpinned_cycles"] <= max(2, st["cycles"] // 10)
    assert len(st["tokens"]) >= wl.new_tokens


@pytest.mark.parametrize("name,layers,mask", [("llama7b", 3, [0, 1, 0]), ("llama70b", 2, [0, 1]),
                                              ("llama3_8b", 2, [0, 1]), ("llama7b_f16", 3, [0, 1, 0])])
def test_large_shapes_at_reduced_depth(ssd, name, layers, mask):
    """Real widths (7B: d 4096, FFN 11008, MHA; 70B: d 8192, FFN 28672, 64 query / 8 KV heads), few layers."""
    wl = WORKLOADS[name]
    shape = reduced_depth(wl.shape, layers)
    orc, ctx = make_pair_gpu_generated(shape, wl.seed, 96, max_k=4)
    prompt = make_prompt(shape.vocab, 37, wl.seed).tolist()
    st = lockstep_ssd(ctx, orc, prompt, 6, 4, np.zeros(layers, np.uint8), shape.dtype)
    assert all(a == 4 for a in st["accepted"]) or st["unpinned_cycles"] > 0
    ctx.ssd_reset()                                              # same weights, fresh sequence on both sides
    st2 = lockstep_ssd(ctx, orc, prompt[:21], 8, 4, np.array(mask, np.uint8), shape.dtype)
    o = OracleSSD(orc)
    print(name, "x", layers, "layers: max err %.2e / %.2e" % (st["max_err"], st2["max_err"]), "accepted", st["accepted"],
          st2["accepted"], "unpinned", st["unpinned_cycles"], st2["unpinned_cycles"])
    # per-layer confidence of the last verify, all rows
    ctx.ssd_reset()
    o.prefill(prompt[:9])
    ctx.ssd_prefill(prompt[:9])
    d = o.draft(np.zeros(layers, np.uint8), 2)
    ctx.ssd_draft_step(np.zeros(layers, np.uint8), 2)
    o.verify(d)
    ctx.ssd_verify(d)
    conf_g = ctx.ssd_layer_confidence(0, 3)
    for row in range(3):
        np.testing.assert_allclose(conf_g[row], o.layer_confidence(row)[0], atol=5e-3)


def test_13b_shape_iterative_search(ssd):
    """Config 4's refinement loop at reduced depth: the library's search (fed the oracle's confidences) installs
    exactly the oracle driver's skip sets, and generation stays in lock-step while the set changes."""
    wl = WORKLOADS["llama13b"]
    L = 6
    shape = reduced_depth(wl.shape, L)
    orc, ctx = make_pair_gpu_generated(shape, wl.seed, 160, max_k=4)
    prompt = make_prompt(shape.vocab, 30, wl.seed).tolist()
    od = SearchDriver(L, SelectParams(), opt_interval=2, score_goal=4.0, max_rounds=10, window=100)
    cd = ssd.Search(L, ssd.search_defaults(opt_interval=2, max_rounds=10), ssd.select_defaults())
    assert np.array_equal(od.mask, cd.mask())
    masks = [od.mask.copy()]

    def policy(o, c, cycle, a):
        conf_o, _ = o.layer_confidence(0)
        conf_g = c.ssd_layer_confidence(0, 1)[0]
        np.testing.assert_allclose(conf_g, conf_o, atol=5e-3)
        m_o = od.observe(a, conf_o)
        m_c = cd.observe(a, conf_o)
        assert np.array_equal(m_o, m_c) and od.active == cd.active
        masks.append(m_o.copy())
        return m_o

    st = lockstep_ssd(ctx, orc, prompt, 24, 4, od.mask.copy(), shape.dtype, next_mask=policy)
    distinct = len({m.tobytes() for m in masks})
    print("13B-shape search: cycles", st["cycles"], "rounds", od.rounds, "distinct sets", distinct, "active", od.active,
          "best", od.best_score, "accepted", st["accepted"], "unpinned", st["unpinned_cycles"])
    assert od.rounds >= 2 and od.rounds <= 10
    assert st["unpinned_cycles"] <= max(2, st["cycles"] // 5)


def test_7b_full_depth_short_prompt(ssd):
    """All 32 layers at full width against the oracle: a 48-token prompt, one draft / verify / accept cycle.
    (With only a dozen cached positions a single bf16 rounding of a K/V element that lands on the other side
    of a tie carries 1/12 of an attention output; 32 layers of that reach the 2e-2 bound, so the prompt is
    long enough for the softmax to average over it as the real workloads do.)"""
    wl = WORKLOADS["llama7b"]
    orc, ctx = make_pair_gpu_generated(wl.shape, wl.seed, 72, max_k=4)
    prompt = make_prompt(wl.shape.vocab, 48, wl.seed).tolist()
    mask = np.zeros(32, np.uint8)
    mask[1:31:2] = 1
    t0 = time.time()
    st = lockstep_ssd(ctx, orc, prompt, 2, 4, mask, "bf16")
    print("7B full depth: max err %.2e" % st["max_err"], "accepted", st["accepted"], "unpinned", st["unpinned_cycles"],
          "%.0f s" % (time.time() - t0))


@pytest.mark.parametrize("name,n_new", [("llama7b", 40), ("llama13b", 16), ("llama70b", 12), ("llama3_8b", 24),
                                        ("llama7b_f16", 24)])
def test_full_workload_properties(ssd, name, n_new):
    """Configs 3-5 at full size in bench.py's launch configuration (full prompt, graphs on): properties that hold
    at any size.  Empty skip set => everything accepted; greedy SSD reproduces the library's own vanilla tokens
    for any skip set (lossless verification); repeated prefills are bit-identical; stale cache entries are never
    read (they are NaN-poisoned before every cycle)."""
    import torch
    from synth import make_weights
    wl = WORKLOADS[name]
    shape = wl.shape
    L = shape.n_layers
    t0 = time.time()
    w = make_weights(shape, wl.seed, device="cuda")
    prompt = make_prompt(shape.vocab, wl.prompt_len, wl.seed).tolist()
    ctx = ssd.Context(shape, w, wl.prompt_len + 4 * n_new + 32, max_k=8)
    van = [ctx.ssd_prefill(prompt)]
    logits0 = ctx.ssd_copy_logits(0, 1).copy()
    assert np.all(np.isfinite(logits0))
    while len(van) < n_new:
        van.append(ctx.ssd_decode())
    uniform = ssd.ssd_uniform_skip(L)
    for k, mask in ((4, np.zeros(L, np.uint8)), (8, uniform), (2, uniform)):
        ctx.ssd_reset()
        got = [ctx.ssd_prefill(prompt)]
        assert np.array_equal(ctx.ssd_copy_logits(0, 1), logits0)          # deterministic prefill
        acc = []
        while len(got) < n_new:
            ctx.ssd_kv_poison_stale()
            d = ctx.ssd_draft_step(mask, k)
            y = ctx.ssd_verify(d)
            a, nx = ctx.ssd_accept(d, y)
            assert d[:a] == y[:a] and nx == y[a] and (a == k or d[a] != y[a])
            acc.append(a)
            got += d[:a] + [nx]
        first_diff = next((i for i, (x, y_) in enumerate(zip(got[:n_new], van)) if x != y_), n_new)
        print(name, "full: k", k, "skipped", int(mask.sum()), "accepted", sum(acc), "of", k * len(acc),
              "first diff vs vanilla", first_diff, "%.0f s" % (time.time() - t0))
        # the single-row and the multi-row kernels round differently: after a near-tie flips one token the two
        # sequences legitimately part ways, so only the prefix up to the first flip is comparable
        assert first_diff >= min(8, n_new)
        if not mask.any():
            assert sum(acc) >= 0.85 * k * len(acc)
    s = ctx.ssd_get_stats()
    assert s["n_tokens"] >= wl.prompt_len + n_new
    del ctx, w
    torch.cuda.empty_cache()


def test_13b_full_iterative_refinement(ssd):
    """Config 4 at full size: the skip set is refined for up to 10 rounds of 30 cycles while tokens are generated;
    the stream stays the vanilla stream (lossless verification) and the search ends within its round limit."""
    import torch
    from synth import make_weights
    wl = WORKLOADS["llama13b"]
    shape = wl.shape
    w = make_weights(shape, wl.seed, device="cuda")
    prompt = make_prompt(shape.vocab, wl.prompt_len, wl.seed).tolist()
    n_new = 330                                                   # > 10 rounds x 30 cycles at one token per cycle
    ctx = ssd.Context(shape, w, wl.prompt_len + n_new + 64, max_k=wl.k)
    t0 = time.time()
    van = ssd.generate_vanilla(ctx, prompt, n_new)
    ctx.ssd_reset()
    sr = ssd.Search(shape.n_layers, ssd.search_defaults(max_rounds=10), ssd.select_defaults())
    got, st = ssd.generate_conflayers(ctx, prompt, n_new, k=wl.k, search=sr)
    first_diff = next((i for i, (a, b) in enumerate(zip(got, van)) if a != b), n_new)
    n_skip = int(st["skip_mask"].sum())
    print("13B refinement: cycles", st["cycles"], "rounds", st["search_rounds"], "best", st["search_best_score"],
          "skipped", n_skip, "accepted", st["accepted"], "first diff vs vanilla", first_diff, "%.0f s" % (time.time() - t0))
    assert 1 <= st["search_rounds"] <= 10 and not sr.active
    assert 0.4 * shape.n_layers - 1e-9 <= n_skip <= 0.6 * shape.n_layers + 1e-9
    assert first_diff >= 32
    del ctx, w
    torch.cuda.empty_cache()
