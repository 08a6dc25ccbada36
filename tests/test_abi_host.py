"""CPU-side checks of the C ABI: exported symbols, argument validation, call-order errors, and
the host policy (selection + search) against the oracle's NumPy/Python twin."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2604_14612_amd as ssd
from paper_2604_14612_amd.binding import ssd_config
from oracle import SearchDriver, SelectParams, select_skip, uniform_skip
from synth import WORKLOADS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ssd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ssd_[a-z_]+)\s*\(", header))
    assert declared == set(ssd.SYMBOLS), declared ^ set(ssd.SYMBOLS)
    l = ssd.lib()
    for name in declared:
        assert getattr(l, name) is not None
    # ... and nothing else: kernel stubs, launchers and tuning hooks are not part of the dynamic symbol table
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", ssd.LIB_PATH], capture_output=True, text=True, check=True).stdout
    exported = {ln.split()[-1] for ln in out.splitlines() if ln.strip()}
    assert exported == declared, sorted(exported ^ declared)[:10]


def _cfg(**kw):
    s = WORKLOADS["tiny"].shape
    c = ssd.make_config(s, 128, 4)
    for k, v in kw.items():
        setattr(c, k, v)
    return c


@pytest.mark.parametrize("bad", [dict(head_dim=48), dict(n_kv_heads=3), dict(d_model=250), dict(vocab=1001),
                                 dict(max_k=0), dict(max_k=16), dict(weight_dtype=3), dict(conf_taps=3),
                                 dict(n_layers=0), dict(max_seq=1), dict(rms_eps=0.0)])
def test_create_rejects_bad_config(bad):
    h = C.c_void_p()
    c = _cfg(**bad)
    assert ssd.lib().ssd_create(C.byref(c), None, C.byref(h)) == ssd.SSD_EINVAL
    assert not h.value
    assert ssd.lib().ssd_workspace_bytes(C.byref(c)) == 0


def test_workspace_size_covers_cache_and_grows_with_max_seq():
    s = WORKLOADS["llama7b"].shape
    a = ssd.lib().ssd_workspace_bytes(C.byref(ssd.make_config(s, 1024, 8)))
    b = ssd.lib().ssd_workspace_bytes(C.byref(ssd.make_config(s, 2048, 8)))
    kv = 2 * s.n_layers * s.d_kv * 2
    assert a > 1024 * kv and b - a >= 1024 * kv


def test_call_order_and_argument_errors_without_a_gpu():
    l = ssd.lib()
    h = C.c_void_p()
    c = _cfg()
    assert l.ssd_create(C.byref(c), None, C.byref(h)) == 0
    tok = np.zeros(4, np.int32)
    out = np.zeros(8, np.int32)
    mask = np.zeros(4, np.uint8)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    assert l.ssd_set_workspace(h, None, 1 << 30) == ssd.SSD_ENOMEM
    assert l.ssd_set_workspace(h, C.c_void_p(256), 16) == ssd.SSD_ENOMEM
    assert b"workspace" in l.ssd_last_error(h)
    assert l.ssd_prefill(h, p(tok), 4, p(out)) == ssd.SSD_ESTATE
    assert l.ssd_decode(h, p(out)) == ssd.SSD_ESTATE
    assert l.ssd_draft_step(h, p(mask), 4, p(out), None) == ssd.SSD_ESTATE
    assert l.ssd_verify(h, p(tok), 4, p(out)) == ssd.SSD_ESTATE
    assert l.ssd_accept(h, p(tok), p(out), 4, p(out), p(out)) == ssd.SSD_ESTATE
    assert l.ssd_layer_confidence(h, 0, 1, p(out), None, None, None) == ssd.SSD_ESTATE
    assert l.ssd_copy_logits(h, 0, 1, p(out)) == ssd.SSD_ESTATE
    assert l.ssd_reset(h) == ssd.SSD_ESTATE
    assert l.ssd_prefill(h, None, 4, p(out)) == ssd.SSD_EINVAL
    assert l.ssd_draft_step(h, p(mask), 0, p(out), None) == ssd.SSD_EINVAL
    kout = np.zeros(1, np.int32)
    assert l.ssd_draft_adaptive(h, p(mask), 4, C.c_float(0.5), p(out), None, p(kout)) == ssd.SSD_ESTATE
    assert l.ssd_draft_adaptive(h, p(mask), 0, C.c_float(0.5), p(out), None, p(kout)) == ssd.SSD_EINVAL
    assert l.ssd_draft_adaptive(h, p(mask), 4, C.c_float(float("nan")), p(out), None, p(kout)) == ssd.SSD_EINVAL
    assert l.ssd_draft_adaptive(h, p(mask), 4, C.c_float(0.5), p(out), None, None) == ssd.SSD_EINVAL
    assert l.ssd_load_weights(h, None) == ssd.SSD_EINVAL
    st = ssd.binding.ssd_stats()
    assert l.ssd_get_stats(h, C.byref(st)) == 0 and st.state == 0 and st.n_tokens == 0
    l.ssd_destroy(h)
    assert l.ssd_prefill(None, p(tok), 4, p(out)) == ssd.SSD_EINVAL


# ---- selection: C++ policy == oracle ----------------------------------------------------------

def _pair(rng):
    lam = float(rng.uniform(0.2, 0.55))
    protect = bool(rng.integers(0, 2))
    maxr = float(rng.choice([0.5, 0.6, 1.0]))
    minr = float(rng.choice([0.0, 0.4]))
    fixed = float(rng.choice([-1.0, -1.0, 0.0, 5.0]))
    op = SelectParams(lam=lam, protect_ends=protect, max_ratio=maxr, min_ratio=minr, fixed_w_max=fixed)
    cp = ssd.select_defaults(lam=lam, protect_ends=int(protect), max_ratio=maxr, min_ratio=minr, fixed_w_max=fixed)
    return op, cp


def test_select_defaults_match_the_oracle_defaults():
    d, o = ssd.select_defaults(), SelectParams()
    assert (d.lambda_, d.w_base, d.kappa, d.flat_tol, d.min_ratio, d.max_ratio, bool(d.protect_ends), d.eps,
            d.fixed_w_max) == (o.lam, o.w_base, o.kappa, o.flat_tol, o.min_ratio, o.max_ratio, o.protect_ends, o.eps,
                               o.fixed_w_max)
    s = ssd.search_defaults()
    assert (s.opt_interval, s.score_goal, s.max_rounds, s.window) == (30, 4.0, 10, 100)


def test_select_skip_identical_to_oracle_on_random_confidences():
    rng = np.random.default_rng(7)
    for it in range(1500):
        L = int(rng.integers(1, 90))
        kind = it % 4
        if kind == 0:
            conf = rng.uniform(0, 1, L)
        elif kind == 1:
            conf = np.round(rng.uniform(0, 1, L), 2)              # many ties and flat runs
        elif kind == 2:
            conf = np.sort(rng.uniform(0, 1, L)) * 1e-2            # near-uniform distributions of random models
        else:
            conf = np.concatenate([np.full(L // 2, 0.3), rng.uniform(0, 1, L - L // 2)])
        op, cp = _pair(rng)
        ref, det = select_skip(conf, op, detail=True)
        got, margin = ssd.ssd_select_skip(conf, cp, want_margin=True)
        assert np.array_equal(ref, got), (it, L, conf.tolist())
        if det:
            full = np.zeros(L)
            full[det["cand"]] = det["margin"]
            assert np.array_equal(full, margin)                   # bit-identical margins


def test_select_skip_hand_vectors_and_errors():
    conf = [.05, .10, .10, .10, .12, .30, .28, .50, .45, .70, .90, .95]
    assert np.flatnonzero(ssd.ssd_select_skip(conf)).tolist() == [2, 3, 4, 6, 8]
    m = ssd.ssd_select_skip([.2, .1, .3, .4], ssd.select_defaults(protect_ends=0, max_ratio=0.5))
    assert np.flatnonzero(m).tolist() == [0, 1]
    with pytest.raises(ssd.SsdError):
        ssd.ssd_select_skip([0.1, float("nan"), 0.2])
    with pytest.raises(ssd.SsdError):
        ssd.ssd_select_skip([0.1, 0.2], ssd.select_defaults(min_ratio=0.7))
    for L in (1, 2, 3, 4, 10, 40, 80):
        for protect in (0, 1):
            a = ssd.ssd_uniform_skip(L, ssd.select_defaults(protect_ends=protect))
            assert np.array_equal(a, uniform_skip(L, SelectParams(protect_ends=bool(protect))))


def test_search_identical_to_oracle_on_random_traces():
    rng = np.random.default_rng(11)
    for trial in range(40):
        L = int(rng.integers(4, 60))
        interval = int(rng.integers(1, 6))
        rounds = int(rng.integers(1, 8))
        window = int(rng.integers(1, 12))
        goal = float(rng.choice([2.0, 3.5, 99.0]))
        op, cp = _pair(rng)
        od = SearchDriver(L, op, opt_interval=interval, score_goal=goal, max_rounds=rounds, window=window)
        cd = ssd.Search(L, ssd.search_defaults(opt_interval=interval, score_goal=goal, max_rounds=rounds, window=window), cp)
        assert np.array_equal(od.mask, cd.mask())
        # few distinct confidence vectors => repeated selections => the shrink path is exercised
        pool = [np.round(rng.uniform(0, 1, L), 1) for _ in range(2)]
        for cyc in range(60):
            a = int(rng.integers(0, 5))
            conf = pool[int(rng.integers(0, 2))] if cyc % 3 else None
            mo = od.observe(a, conf)
            mc = cd.observe(a, conf)
            assert np.array_equal(mo, mc), (trial, cyc)
            assert od.active == cd.active
        r, b = cd.status()
        assert r == od.rounds and b == od.best_score
        cd.close()
