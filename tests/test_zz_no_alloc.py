"""The entry point that allocates nothing (ssd_layer_confidence_static: scratch in a fixed device array inside the
library image) against the ordinary one (scratch in the caller's workspace), through the C ABI: identical results
on two calls in a row, the second with a smaller input; then a smaller model on the same GPU (the array keeps the
first model's contents), an fp32 model (the other kernel path), and the capacity error."""
import ctypes as C

import numpy as np
import pytest

from synth import ModelShape, WORKLOADS, make_prompt, make_weights
from tests._parity import to_gpu

pytestmark = pytest.mark.gpu


def _both(ctx, row_begin, n_rows):
    """Raw ctypes calls of the two entry points on the same taps -> (ordinary, static) result tuples."""
    l, L = ctx._l, ctx.shape.n_layers
    out = []
    for fn in (l.ssd_layer_confidence, l.ssd_layer_confidence_static):
        conf = np.full((n_rows, L), np.nan, np.float32)
        tc = np.full((n_rows, L, 2), np.nan, np.float32)
        tm = np.full((n_rows, L, 2), np.nan, np.float32)
        ta = np.full((n_rows, L, 2), -1, np.int32)
        rc = fn(ctx._h, row_begin, n_rows, conf.ctypes.data_as(C.c_void_p), tc.ctypes.data_as(C.c_void_p),
                tm.ctypes.data_as(C.c_void_p), ta.ctypes.data_as(C.c_void_p))
        assert rc == 0, (rc, l.ssd_last_error(ctx._h))
        out.append((conf, tc, tm, ta))
    return out


def _cycle(ctx, shape, k, plen, seed):
    prompt = make_prompt(shape.vocab, plen, seed).tolist()
    ctx.ssd_prefill(prompt)
    mask = np.zeros(shape.n_layers, np.uint8)
    mask[1::2] = 1
    d = ctx.ssd_draft_step(mask, k)
    ctx.ssd_verify(d)


def _check_equal(a, b):
    for x, y in zip(a, b):
        assert np.array_equal(x, y)          # same kernels, same tiles: bit-identical
    assert np.all(np.isfinite(a[0])) and np.all(a[3] >= 0)


def test_static_scratch_entry_point_matches_the_ordinary_one():
    import torch
    assert torch.cuda.is_available()
    import paper_2604_14612_amd as ssd
    big = ModelShape(40, 512, 8, 8, 1408, 4096)             # 80 tap rows: two batches of the 64-row static pass
    ctx = ssd.Context(big, to_gpu(make_weights(big, 3, norm_gain_std=0.1)), 96, 8)
    _cycle(ctx, big, 8, 33, 1)
    first = _both(ctx, 0, 9)                                # all nine verify rows
    _check_equal(*first)
    second = _both(ctx, 2, 3)                               # second call in a row, smaller input
    _check_equal(*second)
    assert np.array_equal(second[1][0], first[1][0][2:5])
    # a smaller model on the same GPU: the array still holds the first model's rows beyond what this one writes
    small = ModelShape(3, 1024, 8, 2, 2816, 2048)
    ctx2 = ssd.Context(small, to_gpu(make_weights(small, 4, norm_gain_std=0.1)), 64, 4)
    _cycle(ctx2, small, 4, 17, 2)
    _check_equal(*_both(ctx2, 0, 5))
    _check_equal(*_both(ctx, 0, 9))                         # and the first context again
    # fp32 weights: the plain multi-row path
    wl = WORKLOADS["tiny"]
    ctx3 = ssd.Context(wl.shape, to_gpu(make_weights(wl.shape, wl.seed)), 64, 4)
    _cycle(ctx3, wl.shape, 4, 32, 0)
    _check_equal(*_both(ctx3, 0, 5))
    # beyond the stated maximum: a clear error, nothing launched
    wide = ModelShape(32, 128, 2, 2, 256, 65536)            # 64 rows x 65 536 logits do not fit the array
    ctx4 = ssd.Context(wide, to_gpu(make_weights(wide, 5)), 32, 2)
    _cycle(ctx4, wide, 2, 5, 3)
    conf = np.zeros((1, 32), np.float32)
    rc = ctx4._l.ssd_layer_confidence_static(ctx4._h, 0, 1, conf.ctypes.data_as(C.c_void_p), None, None, None)
    assert rc == ssd.SSD_ECAPACITY
    assert ctx4.ssd_layer_confidence(0, 1).shape == (1, 32)  # the ordinary entry point still serves it
