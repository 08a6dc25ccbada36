"""Pins of the reference decoder against library routines, closed forms and invariants.

None of these tests touches the HIP library.  The independent reference (tests/_reference.py) is built from
PyTorch library ops in float64 (rms_norm, scaled_dot_product_attention, silu, linear,
embedding) with the rotary embedding written as a complex multiplication, i.e. a different
formulation from the oracle's pairwise rotation.  Both K/V storage modes of the oracle are pinned:
"exact" (cache in fp64, the plain definition) and "model" (cache rounded to the weight type).
"""
import dataclasses

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import OracleModel, OracleSSD, generate_ssd, generate_vanilla
from synth import ModelShape, WORKLOADS, make_prompt, make_weights
from tests._reference import reference_forward, reference_logits


SHAPES = [
    ModelShape(3, 64, 4, 4, 96, 50, dtype="fp32"),
    ModelShape(2, 96, 6, 2, 160, 77, dtype="fp32", rope_base=500.0, rms_eps=1e-3),   # GQA 3:1
    ModelShape(2, 64, 2, 1, 88, 40, dtype="bf16"),                                    # MQA, bf16 storage
    ModelShape(2, 64, 4, 2, 72, 48, dtype="fp16"),                                    # GQA, fp16 storage
]


@pytest.mark.parametrize("kv", ["exact", "model"])
@pytest.mark.parametrize("shape", SHAPES)
def test_matches_library_op_reference(shape, kv):
    # init_std 0.3 and jittered gains make every term (gain, rope, softmax scale) visible
    w = make_weights(shape, 11, norm_gain_std=0.2, init_std=0.3)
    toks = make_prompt(shape.vocab, 13, 5).tolist()
    ref, ref_taps = reference_forward(shape, w, toks, kv_storage=kv)
    m = OracleModel(shape, w, 32, kv_storage=kv)
    out = m.forward(toks, 0, want_taps=True)
    assert np.abs(out["logits"] - ref).max() <= 1e-9 * max(1.0, np.abs(ref).max())
    assert np.abs(out["taps"] - ref_taps).max() <= 1e-9 * max(1.0, np.abs(ref_taps).max())
    assert np.abs(ref).max() > 0.1        # the comparison is not vacuous
    if kv == "model" and shape.dtype != "fp32":
        # the storage mode matters: the two readings differ by far more than the pin's tolerance
        assert np.abs(ref - reference_logits(shape, w, toks, "exact")).max() > 1e-6


@pytest.mark.parametrize("kv", ["exact", "model"])
def test_tiny_workload_matches_library_op_reference(tiny_workload, kv):
    wl = tiny_workload
    w = make_weights(wl.shape, wl.seed)
    toks = make_prompt(wl.shape.vocab, wl.prompt_len, wl.seed).tolist()
    ref = reference_logits(wl.shape, w, toks, kv)
    got = OracleModel(wl.shape, w, 64, kv_storage=kv).forward(toks, 0)["logits"]
    assert np.abs(got - ref).max() <= 1e-11


def test_draft_rows_match_library_op_reference():
    """Draft model of Section 3 by full recompute: rows after the verified prefix leave out the skipped layers and
    attend the full model's K/V of the prefix plus their own; both storage modes."""
    shape = SHAPES[1]
    w = make_weights(shape, 4, norm_gain_std=0.2, init_std=0.3)
    toks = make_prompt(shape.vocab, 11, 8).tolist()
    mask = np.array([1, 0], np.uint8)
    for kv in ("exact", "model"):
        ref, _ = reference_forward(shape, w, toks, kv, skip_mask=mask, n_verified=7)
        m = OracleModel(shape, w, 16, kv_storage=kv)
        m.forward(toks[:7], 0)
        for p in range(7, 11):
            z = m.forward([toks[p]], p, skip_mask=mask)["logits"][0]
            assert np.abs(z - ref[p]).max() <= 1e-9 * max(1.0, np.abs(ref).max())
        full = reference_logits(shape, w, toks, kv)
        assert np.abs(full[7:] - ref[7:]).max() > 1e-3     # the skip set changes the result


def test_cache_rounding_is_the_library_cast_and_is_applied():
    """orc_round_bf16 against torch's fp32 -> bf16 cast (random values, exact ties, both parities), and the
    cache of a bf16 model holds only bf16-representable numbers that differ from the unrounded K/V."""
    from oracle import round_bf16
    g = torch.Generator().manual_seed(7)
    x = torch.randn(4000, generator=g, dtype=torch.float64) * torch.logspace(-6, 6, 4000, dtype=torch.float64)
    ties = torch.tensor([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 2.0 ** -20 * (1 + 5 * 2.0 ** -8),
                         1.0 + 2.0 ** -8 + 2.0 ** -30, 1.0 + 2.0 ** -8 - 2.0 ** -30, 0.0, 255.5, 3.3895e38],
                        dtype=torch.float64)
    x = torch.cat([x, ties])
    ref = x.to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([round_bf16(v) for v in x.tolist()])
    assert np.array_equal(got, ref)
    assert round_bf16(1.0 + 2.0 ** -8) == 1.0 and round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6   # ties to even
    # fp16: random values across the normal and subnormal range, ties, overflow to infinity
    from oracle import round_fp16
    xh = torch.cat([torch.randn(4000, generator=g, dtype=torch.float64) * torch.logspace(-9, 5, 4000, dtype=torch.float64),
                    torch.tensor([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, -(1.0 + 2.0 ** -11), 2.0 ** -24, 2.0 ** -25,
                                  3 * 2.0 ** -25, 65504.0, 65519.9, 65520.0, 1e6, 0.0, 2.0 ** -14 - 2.0 ** -26],
                                 dtype=torch.float64)])
    refh = xh.to(torch.float32).to(torch.float16).to(torch.float64).numpy()
    goth = np.array([round_fp16(v) for v in xh.tolist()])
    assert np.array_equal(goth, refh)
    assert round_fp16(1.0 + 2.0 ** -11) == 1.0 and round_fp16(65520.0) == np.inf and round_fp16(2.0 ** -25) == 0.0
    for shape, st in ((SHAPES[2], torch.bfloat16), (SHAPES[3], torch.float16)):
        w = make_weights(shape, 11, norm_gain_std=0.2, init_std=0.3)
        toks = make_prompt(shape.vocab, 9, 5).tolist()
        m = OracleModel(shape, w, 16)
        m.forward(toks, 0)
        for c in (m.kcache(), m.vcache()):
            c = np.asarray(c).reshape(shape.n_layers, 16, -1)[:, :9]
            assert np.array_equal(c, torch.from_numpy(c.copy()).to(st).to(torch.float64).numpy())
            assert np.abs(c).max() > 0.1
    # an fp32 model's cache holds fp32-representable numbers
    m32 = OracleModel(SHAPES[0], make_weights(SHAPES[0], 1, init_std=0.3), 16)
    m32.forward(toks[:5], 0)
    c = np.asarray(m32.kcache()).reshape(SHAPES[0].n_layers, 16, -1)[:, :5]
    assert np.array_equal(c, c.astype(np.float32).astype(np.float64)) and np.abs(c).max() > 0.1


def test_incremental_equals_full_recompute():
    shape = SHAPES[1]
    w = make_weights(shape, 3, norm_gain_std=0.1, init_std=0.2)
    toks = make_prompt(shape.vocab, 12, 1).tolist()
    full = OracleModel(shape, w, 16).forward(toks, 0)["logits"]
    m = OracleModel(shape, w, 16)
    for p, t in enumerate(toks):
        z = m.forward([t], p)["logits"][0]
        assert np.array_equal(z, full[p])          # same row routine, same order: bit-exact
    # mixed chunking
    m2 = OracleModel(shape, w, 16)
    a = m2.forward(toks[:5], 0)["logits"]
    b = m2.forward(toks[5:], 5)["logits"]
    assert np.array_equal(np.concatenate([a, b]), full)


def test_all_layers_skipped_is_embedding_through_head():
    shape = SHAPES[0]
    w = make_weights(shape, 5, norm_gain_std=0.3, init_std=0.5)
    m = OracleModel(shape, w, 8)
    t = 17
    z = m.forward([t], 0, skip_mask=np.ones(shape.n_layers, np.uint8))["logits"][0]
    e = w["embed"][t].double().numpy()
    h = e / np.sqrt(np.mean(e * e) + shape.rms_eps) * w["final_norm"].double().numpy()
    np.testing.assert_allclose(z, w["lm_head"].double().numpy() @ h, rtol=1e-12, atol=1e-12)
    # a skipped layer writes nothing to the cache
    assert not m.kcache().any() and not m.vcache().any()


def test_sub_block_skipping():
    """Attention and MLP sub-blocks skipped separately (two mask entries per layer): against the library-op
    reference on draft rows, against the whole-layer mask, and against a closed form with every attention
    sub-block skipped (no token then sees another: the row is its embedding pushed through the MLPs alone)."""
    shape = SHAPES[1]
    L = shape.n_layers
    w = make_weights(shape, 4, norm_gain_std=0.2, init_std=0.3)
    toks = make_prompt(shape.vocab, 11, 8).tolist()
    for sub in ([1, 0, 0, 1], [0, 1, 1, 0], [0, 0, 1, 0], [1, 1, 0, 1]):
        sub = np.array(sub, np.uint8)
        for kv in ("exact", "model"):
            ref, ref_taps = reference_forward(shape, w, toks, kv, skip_mask=sub, n_verified=7)
            m = OracleModel(shape, w, 16, kv_storage=kv)
            m.forward(toks[:7], 0)
            out = m.forward(toks[7:], 7, skip_mask=sub, want_taps=True)
            assert np.abs(out["logits"] - ref[7:]).max() <= 1e-9 * max(1.0, np.abs(ref).max())
            assert np.abs(out["taps"] - ref_taps[7:]).max() <= 1e-9 * max(1.0, np.abs(ref_taps).max())
    # a layer of the skip set = both of its sub-blocks
    whole = np.array([0, 1], np.uint8)
    a = OracleModel(shape, w, 16)
    b = OracleModel(shape, w, 16)
    za = a.forward(toks, 0, skip_mask=whole)["logits"]
    zb = b.forward(toks, 0, skip_mask=np.repeat(whole, 2))["logits"]
    assert np.array_equal(za, zb) and np.array_equal(a.kcache(), b.kcache())
    # every attention sub-block skipped: closed form, and nothing is written to the cache
    only_mlp = np.tile(np.array([1, 0], np.uint8), L)
    m = OracleModel(shape, w, 16)
    z = m.forward(toks[:3], 2, skip_mask=only_mlp)["logits"]
    assert not m.kcache().any() and not m.vcache().any()
    for r, t in enumerate(toks[:3]):
        x = w["embed"][t].double().numpy()
        for l in range(L):
            h = x / np.sqrt(np.mean(x * x) + shape.rms_eps) * w["mlp_norm"][l].double().numpy()
            g, u = w["wg"][l].double().numpy() @ h, w["wu"][l].double().numpy() @ h
            x = x + w["wd"][l].double().numpy() @ (g / (1.0 + np.exp(-g)) * u)
        h = x / np.sqrt(np.mean(x * x) + shape.rms_eps) * w["final_norm"].double().numpy()
        np.testing.assert_allclose(z[r], w["lm_head"].double().numpy() @ h, rtol=1e-11, atol=1e-11)
    # every MLP sub-block skipped changes the result in another way (both masks differ from the full model)
    only_attn = np.tile(np.array([0, 1], np.uint8), L)
    full = OracleModel(shape, w, 16).forward(toks, 0)["logits"]
    part = OracleModel(shape, w, 16).forward(toks, 0, skip_mask=only_attn)["logits"]
    assert np.abs(full - part).max() > 1e-3


def test_rope_is_identity_at_position_zero_and_preserves_norm():
    shape = ModelShape(1, 64, 2, 2, 96, 30, dtype="fp32")
    w = make_weights(shape, 9, init_std=0.4)
    m = OracleModel(shape, w, 8)
    toks = [3, 3, 3, 3]
    m.forward(toks, 0)
    e = w["embed"][3].double()
    h = F.rms_norm(e, (64,), w["attn_norm"][0].double(), eps=shape.rms_eps)
    k_raw = F.linear(h, w["wk"][0].double()).view(2, 32).numpy()
    v_raw = F.linear(h, w["wv"][0].double()).view(2, 32).numpy()
    # exact storage: the cache holds the fp64 values; model storage: the cache of an fp32 model stores fp32
    # numbers, agreement to one fp32 rounding (2^-24 relative)
    for kv, rtol in (("exact", 1e-12), ("model", 6e-8)):
        mm = OracleModel(shape, w, 8, kv_storage=kv)
        mm.forward(toks, 0)
        K = mm.kcache()[0]
        np.testing.assert_allclose(K[0], k_raw, rtol=rtol, atol=1e-14)           # angle 0
        for p in range(1, 4):                                                   # same token => same raw k
            np.testing.assert_allclose(np.linalg.norm(K[p], axis=-1), np.linalg.norm(k_raw, axis=-1), rtol=rtol)
            assert np.abs(K[p] - k_raw).max() > 1e-3
        for p in range(4):                                                      # V is never rotated
            np.testing.assert_allclose(mm.vcache()[0][p], v_raw, rtol=rtol, atol=1e-14)


def test_gqa_equals_mha_with_replicated_kv_heads():
    g = ModelShape(2, 64, 4, 2, 96, 40, dtype="fp32")
    w = make_weights(g, 21, init_std=0.3)
    mha = dataclasses.replace(g, n_kv_heads=4)
    w2 = dict(w)
    hd = g.head_dim
    for name in ("wk", "wv"):
        w2[name] = [t.view(2, hd, -1).repeat_interleave(2, dim=0).reshape(4 * hd, -1).contiguous() for t in w[name]]
    toks = make_prompt(40, 9, 2).tolist()
    a = OracleModel(g, w, 16).forward(toks, 0)["logits"]
    b = OracleModel(mha, w2, 16).forward(toks, 0)["logits"]
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)


# ---- greedy self-speculative decoding -----------------------------------------------------

def _tiny():
    wl = WORKLOADS["tiny"]
    w = make_weights(wl.shape, wl.seed)
    return wl, w, make_prompt(wl.shape.vocab, wl.prompt_len, wl.seed).tolist()


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_ssd_is_lossless_for_any_mask(k):
    wl, w, p = _tiny()
    m = OracleModel(wl.shape, w, 128)
    van = generate_vanilla(m, p, 24)
    rng = np.random.default_rng(k)
    masks = [np.zeros(4, np.uint8), np.array([0, 1, 1, 0], np.uint8), np.ones(4, np.uint8)]
    masks += [rng.integers(0, 2, 4).astype(np.uint8) for _ in range(3)]
    masks += [rng.integers(0, 2, 8).astype(np.uint8) for _ in range(3)]      # attention / MLP sub-blocks separately
    for mask in masks:
        got, st = generate_ssd(OracleModel(wl.shape, w, 128), p, 24, k, mask)
        assert got == van, mask
        assert st["drafted"] == st["cycles"] * k


@pytest.mark.parametrize("k", [1, 3, 4])
def test_empty_skip_set_accepts_everything(k):
    wl, w, p = _tiny()
    m = OracleModel(wl.shape, w, 128)
    _, st = generate_ssd(m, p, 20, k, np.zeros(4, np.uint8))
    assert all(a == k for a in st["accepted_per_cycle"])
    assert st["accepted"] == st["drafted"]


def test_adaptive_drafting_truncates_the_fixed_length_draft_and_stays_lossless():
    """Confidence-aware drafting: gamma = 0 is the fixed-k draft, gamma > 1 drafts one token, any gamma gives a
    prefix of the fixed-k draft whose length is set by the first max-probability below gamma (max-probabilities
    recomputed here with scipy's softmax), and generation with it still equals vanilla decoding."""
    from scipy.special import softmax
    wl, w, _ = _tiny()
    shape = wl.shape
    prompt = make_prompt(shape.vocab, 9, 3).tolist()
    mask = np.array([0, 1, 0, 0], np.uint8)
    s = OracleSSD(OracleModel(shape, w, 64))
    s.prefill(prompt)
    fixed = s.draft(mask, 8)
    probs = [float(softmax(z).max()) for z in s.last_draft_logits]
    assert s.draft_adaptive(mask, 8, 0.0)[0] == fixed
    d1, p1 = s.draft_adaptive(mask, 8, 1.5)
    assert d1 == fixed[:1] and abs(p1[0] - probs[0]) < 1e-12
    for gamma in sorted(probs)[1::2]:
        d, mp = s.draft_adaptive(mask, 8, gamma + 1e-12)
        stop = next(i for i, p in enumerate(probs) if p < gamma + 1e-12)
        assert d == fixed[:stop + 1] and np.allclose(mp, probs[:stop + 1], rtol=1e-12)
        assert all(p >= gamma for p in mp[:-1]) and mp[-1] < gamma + 1e-12
    # lossless with a varying draft length
    van = generate_vanilla(OracleModel(shape, w, 96), prompt, 24)
    s = OracleSSD(OracleModel(shape, w, 96))
    s.prefill(prompt)
    gamma = float(np.median(probs))
    lens = []
    while s.n - len(prompt) < 24:
        d, _ = s.draft_adaptive(mask, 6, gamma)
        lens.append(len(d))
        s.accept(d, s.verify(d))
    assert s.tokens[len(prompt):len(prompt) + 24] == van
    assert len(set(lens)) > 1          # the rule actually varied the length


def test_stale_cache_entries_are_never_read():
    wl, w, p = _tiny()
    mask = np.array([0, 1, 0, 1], np.uint8)
    ref, _ = generate_ssd(OracleModel(wl.shape, w, 128), p, 20, 4, mask)
    m = OracleModel(wl.shape, w, 128)

    def poison(state, d, y, a):
        state.m.kv_poison(state.n - 1)          # valid entries are 0..n-2

    got, _ = generate_ssd(m, p, 20, 4, mask, on_cycle=poison)
    assert got == ref


def test_accept_rule_on_hand_cases():
    s = OracleSSD.__new__(OracleSSD)
    s.tokens, s.drafted, s.accepted, s.cycles = [9], 0, 0, 0
    assert s.accept([5, 6, 7], [5, 6, 7, 8]) == (3, 8) and s.tokens == [9, 5, 6, 7, 8]
    assert s.accept([1, 2, 3], [1, 9, 3, 4]) == (1, 9) and s.tokens[-2:] == [1, 9]
    assert s.accept([1, 2], [0, 2, 3]) == (0, 0)
    # a later match after a mismatch does not count
    assert s.accept([4, 4, 4], [4, 5, 4, 4]) == (1, 5)
    assert (s.drafted, s.accepted, s.cycles) == (11, 5, 4)


def test_bad_arguments_are_rejected():
    wl, w, p = _tiny()
    m = OracleModel(wl.shape, w, 8)
    with pytest.raises(ValueError):
        m.forward([1] * 9, 0)
    with pytest.raises(ValueError):
        m.forward([wl.shape.vocab], 0)
