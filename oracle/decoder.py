"""ctypes front end of the C reference decoder (TEST INFRASTRUCTURE, not a product path).

`OracleModel` wraps oracle/ssd_oracle.c: a double-precision Llama-style decoder with a
KV cache, a layer skip mask (draft model of Section 3), hidden-state taps and the
entropy confidence of Eq. 1-4.
"""
from __future__ import annotations

import ctypes as C
from typing import Optional, Sequence

import numpy as np

from .build import build


class _Cfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("max_seq", C.c_int32),
                ("rms_eps", C.c_double), ("rope_base", C.c_double), ("weight_dtype", C.c_int32),
                ("kv_storage", C.c_int32)]


# K/V cache storage of the reference model: "model" = rounded to the weight type (the reading of Section 4.1.1:
# a half-precision model's cache holds half-precision numbers), "exact" = kept in fp64 (nothing rounded: the
# plain definition of attention), or an explicit type
KV_STORAGE = {"exact": -1, "fp32": 0, "bf16": 1, "fp16": 2}


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        lib.orc_create.restype = C.c_void_p
        lib.orc_create.argtypes = [C.POINTER(_Cfg)] + [C.c_void_p] * 12
        lib.orc_destroy.argtypes = [C.c_void_p]
        lib.orc_kv_poison.argtypes = [C.c_void_p, C.c_int]
        lib.orc_kcache.restype = C.c_void_p
        lib.orc_kcache.argtypes = [C.c_void_p]
        lib.orc_vcache.restype = C.c_void_p
        lib.orc_vcache.argtypes = [C.c_void_p]
        for fn in (lib.orc_forward, lib.orc_forward_sub):
            fn.restype = C.c_int
            fn.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.orc_round_bf16.restype = C.c_double
        lib.orc_round_bf16.argtypes = [C.c_double]
        lib.orc_round_fp16.restype = C.c_double
        lib.orc_round_fp16.argtypes = [C.c_double]
        lib.orc_argmax.restype = C.c_int32
        lib.orc_argmax.argtypes = [C.c_void_p, C.c_int]
        lib.orc_confidence_from_logits.argtypes = [C.c_void_p, C.c_int, C.c_double, C.c_double,
                                                   C.c_void_p, C.c_void_p, C.c_void_p]
        lib.orc_confidence.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_double, C.c_double,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = lib
    return _lib


def _as_numpy(t):
    """torch tensor (fp32, bf16 or fp16, CPU) or ndarray -> contiguous ndarray; half types become raw uint16."""
    if isinstance(t, np.ndarray):
        return np.ascontiguousarray(t)
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


DEFAULT_CLAMP = 1e4     # the paper gives no clamp range (Section 3.1); reading stated in the design notes
DEFAULT_EPS = 1e-10     # epsilon of Eq. 2, not given in the paper


class OracleModel:
    """Reference decoder over caller-supplied weights (dict as produced by synth.make_weights)."""

    def __init__(self, shape, weights, max_seq: int, kv_storage: str = "model"):
        lib = _load()
        self.shape = shape
        self.max_seq = int(max_seq)
        wt = {"fp32": 0, "bf16": 1, "fp16": 2}[shape.dtype]
        self.kv_storage = shape.dtype if kv_storage == "model" else kv_storage
        kvs = KV_STORAGE[self.kv_storage]
        self._keep = []

        def mat(t):
            a = _as_numpy(t)
            assert a.dtype == (np.uint16 if wt else np.float32), a.dtype
            self._keep.append(a)
            return a.ctypes.data

        def vec(t):
            a = _as_numpy(t).astype(np.float32, copy=False)
            self._keep.append(a)
            return a.ctypes.data

        L = shape.n_layers

        def arr(name, conv):
            ptrs = (C.c_void_p * L)(*[conv(weights[name][l]) for l in range(L)])
            self._keep.append(ptrs)
            return C.cast(ptrs, C.c_void_p)

        cfg = _Cfg(L, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                   shape.vocab, self.max_seq, shape.rms_eps, shape.rope_base, wt, kvs)
        self._h = lib.orc_create(C.byref(cfg), mat(weights["embed"]), mat(weights["lm_head"]),
                                 vec(weights["final_norm"]), arr("attn_norm", vec), arr("wq", mat),
                                 arr("wk", mat), arr("wv", mat), arr("wo", mat), arr("mlp_norm", vec),
                                 arr("wg", mat), arr("wu", mat), arr("wd", mat))
        if not self._h:
            raise RuntimeError("orc_create failed")
        self._lib = lib

    def close(self):
        if getattr(self, "_h", None):
            self._lib.orc_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    # -- cache access (tests) ---------------------------------------------------------------
    def kv_poison(self, from_pos: int):
        self._lib.orc_kv_poison(self._h, int(from_pos))

    def kcache(self) -> np.ndarray:
        s = self.shape
        n = s.n_layers * self.max_seq * s.d_kv
        buf = (C.c_double * n).from_address(self._lib.orc_kcache(self._h))
        return np.frombuffer(buf, dtype=np.float64).reshape(s.n_layers, self.max_seq, s.n_kv_heads, s.head_dim)

    def vcache(self) -> np.ndarray:
        s = self.shape
        n = s.n_layers * self.max_seq * s.d_kv
        buf = (C.c_double * n).from_address(self._lib.orc_vcache(self._h))
        return np.frombuffer(buf, dtype=np.float64).reshape(s.n_layers, self.max_seq, s.n_kv_heads, s.head_dim)

    # -- forward ----------------------------------------------------------------------------
    def forward(self, tokens: Sequence[int], pos0: int, skip_mask=None, want_taps=False,
                want_logits=True, want_hidden=False):
        """Run rows `tokens` at positions pos0.. ; returns dict(logits, taps, hidden).

        skip_mask: n_layers entries (whole layers, the skip set S) or 2 * n_layers entries (attention and MLP
        sub-block of every layer separately, [2l] and [2l+1])."""
        s = self.shape
        tok = np.ascontiguousarray(np.asarray(tokens, dtype=np.int32))
        R = tok.shape[0]
        skip = None if skip_mask is None else np.ascontiguousarray(np.asarray(skip_mask, dtype=np.uint8))
        fwd = self._lib.orc_forward
        if skip is not None:
            assert skip.shape in ((s.n_layers,), (2 * s.n_layers,)), skip.shape
            if skip.shape[0] == 2 * s.n_layers:
                fwd = self._lib.orc_forward_sub
        taps = np.empty((R, s.n_layers, 2, s.d_model), np.float64) if want_taps else None
        logits = np.empty((R, s.vocab), np.float64) if want_logits else None
        hidden = np.empty((R, s.d_model), np.float64) if want_hidden else None
        rc = fwd(self._h, _ptr(tok), R, int(pos0), _ptr(skip), _ptr(taps), _ptr(logits), _ptr(hidden))
        if rc != 0:
            raise ValueError("orc_forward: bad arguments (rows, positions or token ids out of range)")
        return {"logits": logits, "taps": taps, "hidden": hidden}

    # -- confidence -------------------------------------------------------------------------
    def confidence(self, hidden: np.ndarray, clamp=DEFAULT_CLAMP, eps=DEFAULT_EPS, want_logits=False):
        """Eq. 1-4 on hidden-state rows [n][d] -> dict(conf, maxprob, argmax[, logits])."""
        hid = np.ascontiguousarray(hidden, dtype=np.float64).reshape(-1, self.shape.d_model)
        n = hid.shape[0]
        conf = np.empty(n, np.float64)
        mp = np.empty(n, np.float64)
        am = np.empty(n, np.int32)
        lg = np.empty((n, self.shape.vocab), np.float64) if want_logits else None
        self._lib.orc_confidence(self._h, _ptr(hid), n, float(clamp), float(eps), _ptr(conf), _ptr(mp),
                                 _ptr(am), _ptr(lg))
        out = {"conf": conf, "maxprob": mp, "argmax": am}
        if want_logits:
            out["logits"] = lg
        return out


def round_bf16(x: float) -> float:
    """The value a bf16 K/V cache entry holds for x: fp32 then bf16, round-to-nearest-even."""
    return float(_load().orc_round_bf16(float(x)))


def round_fp16(x: float) -> float:
    """The value an fp16 K/V cache entry holds for x: fp32 then fp16, round-to-nearest-even."""
    return float(_load().orc_round_fp16(float(x)))


def argmax_lowest(z: np.ndarray) -> int:
    z = np.ascontiguousarray(z, dtype=np.float64)
    return int(_load().orc_argmax(_ptr(z), z.shape[0]))


def confidence_from_logits(z: np.ndarray, clamp=DEFAULT_CLAMP, eps=DEFAULT_EPS):
    """Eq. 1-4 for one logit vector -> (confidence, max probability, argmax)."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    conf, mp, am = C.c_double(), C.c_double(), C.c_int32()
    _load().orc_confidence_from_logits(_ptr(z), z.shape[0], float(clamp), float(eps),
                                       C.byref(conf), C.byref(mp), C.byref(am))
    return conf.value, mp.value, am.value
