"""GPU parity on the benchmark workloads themselves (BASELINE configs 2-5): the full "small" workload,
the 7B / 13B / 70B shapes at reduced depth (several cycles, confidence, search) and at FULL depth (32, 40 and 80
layers, one cycle per draft length after a 48-token prompt: the CPU oracle needs seconds per row there), and
size-independent properties on the full 7B, 13B and 70B workloads in the launch configuration bench.py times."""
import time

import numpy as np
import pytest

from oracle import OracleSSD, SearchDriver, SelectParams, select_skip
from synth import WORKLOADS, make_prompt, reduced_depth
from tests._parity import (TOL, assert_logits_close, decisive, lockstep_ssd, make_pair, make_pair_gpu_generated,
                           progress)

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


def _uniform_mask(L):
    m = np.zeros(L, np.uint8)
    m[1:L - 1:2] = 1
    return m


def _full_depth(ssd, name, k_seq, prompt_len=48):
    """Every layer of a benchmark shape at full width in lock-step with the oracle (K/V storage = the model's type):
    one prompt, then one draft / verify / accept cycle per entry of k_seq with every second layer skipped in the
    draft.  All logit rows within the bf16 bound, tokens and accepted counts exact wherever the oracle's margin is
    decisive."""
    wl = WORKLOADS[name]
    L = wl.shape.n_layers
    t0 = time.time()
    progress("%s full depth: drawing weights, copying them to the host" % name)
    orc, ctx = make_pair_gpu_generated(wl.shape, wl.seed, prompt_len + sum(k_seq) + len(k_seq) + 8, max_k=max(k_seq))
    prompt = make_prompt(wl.shape.vocab, prompt_len, wl.seed).tolist()
    t1 = time.time()
    progress("%s full depth: set-up done in %.0f s" % (name, t1 - t0))
    st = lockstep_ssd(ctx, orc, prompt, 0, k_seq, _uniform_mask(L), wl.shape.dtype, report=name + " full depth")
    print(name, "full depth (%d layers), prompt %d, k" % (L, prompt_len), k_seq, ": max err %.2e" % st["max_err"],
          "accepted", st["accepted"], "unpinned", st["unpinned_cycles"], "tokens checked", st["tokens_checked"],
          "setup %.0f s, lock-step %.0f s" % (t1 - t0, time.time() - t1), flush=True)
    progress("%s full depth: max logit err %.2e over %d draft + %d verify rows, accepted %s, unpinned cycles %d" % (
        name, st["max_err"], st["draft_rows"], st["verify_rows"], st["accepted"], st["unpinned_cycles"]))
    assert st["cycles"] == len(k_seq) and st["verify_rows"] == sum(k_seq) + len(k_seq)
    assert st["unpinned_cycles"] <= 1
    ctx.close()
    orc.close()
    import torch
    del ctx, orc
    torch.cuda.empty_cache()
    return st


def test_7b_full_depth_k_2_4_8(ssd):
    """Config 3: all 32 layers, k = 2, 4 and 8 (one cycle each after a 48-token prompt)."""
    _full_depth(ssd, "llama7b", [2, 4, 8])


def test_13b_full_depth_40_layers(ssd):
    """Config 4's model: all 40 layers."""
    _full_depth(ssd, "llama13b", [4])


def test_70b_full_depth_80_layers(ssd):
    """Config 5's model: all 80 layers, grouped-query attention (64 query / 8 KV heads), 138 GB of bf16 weights on
    the GPU and the same bits on the host for the oracle."""
    _full_depth(ssd, "llama70b", [4])


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
    tol_a, tol_r = TOL[shape.dtype]

    def near_tie(z, t1, t2):
        """True if tokens t1 and t2 are within the logit tolerance of each other in the library's own logits z
        (two kernels that are each within tolerance of the exact logits can order such a pair differently)."""
        return abs(float(z[t1]) - float(z[t2])) <= tol_a + tol_r * float(np.abs(z).max())

    progress("%s properties: %d vanilla tokens done at %.0f s" % (name, n_new, time.time() - t0))
    for k, mask in ((4, np.zeros(L, np.uint8)), (8, uniform), (2, uniform)):
        progress("%s properties: k=%d, %d layers skipped" % (name, k, int(mask.sum())))
        ctx.ssd_reset()
        got = [ctx.ssd_prefill(prompt)]
        assert np.array_equal(ctx.ssd_copy_logits(0, 1), logits0)          # deterministic prefill
        acc = []
        diverged = None          # index of the first token that differs from the vanilla stream
        while len(got) < n_new:
            ctx.ssd_kv_poison_stale()
            d = ctx.ssd_draft_step(mask, k)
            y = ctx.ssd_verify(d)
            zv = ctx.ssd_copy_logits(0, k + 1)
            a, nx = ctx.ssd_accept(d, y)
            assert d[:a] == y[:a] and nx == y[a] and (a == k or d[a] != y[a])
            if not mask.any() and a < k:
                # empty skip set: the draft model IS the full model, so a rejected draft can only be a near-tie
                # that the single-row and the multi-row kernels order differently
                assert near_tie(zv[a], d[a], y[a]), "empty skip set: draft rejected at a decisive margin"
            if diverged is None:
                # lossless verification: every committed token is the library's own vanilla token, until the first
                # near-tie that the two kernel families order differently (after it the streams legitimately part)
                for j, t in enumerate(d[:a] + [nx]):
                    i = len(got) + j
                    if i < n_new and t != van[i]:
                        assert near_tie(zv[j], t, van[i]), "SSD token differs from vanilla at a decisive margin"
                        diverged = i
                        break
            acc.append(a)
            got += d[:a] + [nx]
        print(name, "full: k", k, "skipped", int(mask.sum()), "accepted", sum(acc), "of", k * len(acc),
              "first diff vs vanilla", diverged, "%.0f s" % (time.time() - t0), flush=True)
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
