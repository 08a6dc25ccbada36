"""Thin ctypes binding of libssd.so: argument marshalling only.

Function names mirror include/ssd.h.  PyTorch appears only as the owner of device memory
(weights, workspace) and of the HIP stream; every step of the decoding path runs inside the
library's kernels.  There is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# SSD_LIB_PATH names another build of the same library (the sanitizer build of the CPU tests); default: in-tree
LIB_PATH = os.environ.get("SSD_LIB_PATH") or os.path.join(_HERE, "libssd.so")

SSD_OK, SSD_EINVAL, SSD_ESTATE, SSD_ECAPACITY, SSD_ENOMEM, SSD_EHIP = 0, -1, -2, -3, -4, -5
SSD_MAX_K = 15
KERNEL_IDS = {"gemv_qkv": 0, "attention": 1, "gemv_o": 2, "gemv_gateup": 3, "gemv_down": 4, "gemv_lmhead": 5,
              "vocab_reduce": 6, "rows_qkv": 7, "rows_o": 8, "rows_gateup": 9, "rows_down": 10, "rows_lmhead": 11}
SSD_PREFILL_ROWS = 512
_ERR_NAMES = {-1: "SSD_EINVAL", -2: "SSD_ESTATE", -3: "SSD_ECAPACITY", -4: "SSD_ENOMEM", -5: "SSD_EHIP"}


class SsdError(RuntimeError):
    def __init__(self, code: int, msg: str = ""):
        self.code = code
        super().__init__("%s (%d)%s" % (_ERR_NAMES.get(code, "SSD_E?"), code, ": " + msg if msg else ""))


class ssd_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("max_seq", C.c_int32), ("rms_eps", C.c_float),
                ("rope_base", C.c_float), ("weight_dtype", C.c_int32), ("conf_taps", C.c_int32),
                ("conf_clamp", C.c_float), ("conf_eps", C.c_float), ("max_k", C.c_int32), ("kv_dtype", C.c_int32),
                ("conf_window", C.c_int32)]


class ssd_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wq", C.POINTER(C.c_void_p)),
                ("wk", C.POINTER(C.c_void_p)), ("wv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)),
                ("mlp_norm", C.POINTER(C.c_void_p)), ("wg", C.POINTER(C.c_void_p)),
                ("wu", C.POINTER(C.c_void_p)), ("wd", C.POINTER(C.c_void_p))]


class ssd_stats(C.Structure):
    _fields_ = [("cycles", C.c_int64), ("drafted", C.c_int64), ("accepted", C.c_int64), ("committed", C.c_int64),
                ("decode_steps", C.c_int64), ("draft_steps", C.c_int64), ("verify_rows", C.c_int64),
                ("confidence_rows", C.c_int64), ("n_tokens", C.c_int32), ("state", C.c_int32)]


class ssd_select_params(C.Structure):
    _fields_ = [("lambda_", C.c_double), ("w_base", C.c_double), ("kappa", C.c_double), ("flat_tol", C.c_double),
                ("min_ratio", C.c_double), ("max_ratio", C.c_double), ("protect_ends", C.c_int32),
                ("eps", C.c_double), ("fixed_w_max", C.c_double)]


class ssd_search_params(C.Structure):
    _fields_ = [("opt_interval", C.c_int32), ("score_goal", C.c_double), ("max_rounds", C.c_int32),
                ("window", C.c_int32)]


# every symbol include/ssd.h declares: name -> (restype, argtypes)
_P = C.c_void_p
SYMBOLS = {
    "ssd_create": (C.c_int, [C.POINTER(ssd_config), _P, C.POINTER(_P)]),
    "ssd_workspace_bytes": (C.c_size_t, [C.POINTER(ssd_config)]),
    "ssd_set_workspace": (C.c_int, [_P, _P, C.c_size_t]),
    "ssd_load_weights": (C.c_int, [_P, C.POINTER(ssd_weights)]),
    "ssd_reset": (C.c_int, [_P]),
    "ssd_destroy": (None, [_P]),
    "ssd_last_error": (C.c_char_p, [_P]),
    "ssd_get_stats": (C.c_int, [_P, C.POINTER(ssd_stats)]),
    "ssd_prefill": (C.c_int, [_P, _P, C.c_int, _P]),
    "ssd_decode": (C.c_int, [_P, _P]),
    "ssd_draft_step": (C.c_int, [_P, _P, C.c_int, _P, _P]),
    "ssd_draft_step_sub": (C.c_int, [_P, _P, C.c_int, _P, _P]),
    "ssd_draft_adaptive": (C.c_int, [_P, _P, C.c_int, C.c_float, _P, _P, _P]),
    "ssd_verify": (C.c_int, [_P, _P, C.c_int, _P]),
    "ssd_accept": (C.c_int, [_P, _P, _P, C.c_int, _P, _P]),
    "ssd_force_commit": (C.c_int, [_P, _P, C.c_int, C.c_int, C.c_int32]),
    "ssd_copy_logits": (C.c_int, [_P, C.c_int, C.c_int, _P]),
    "ssd_layer_confidence": (C.c_int, [_P, C.c_int, C.c_int, _P, _P, _P, _P]),
    "ssd_layer_confidence_static": (C.c_int, [_P, C.c_int, C.c_int, _P, _P, _P, _P]),
    "ssd_window_confidence": (C.c_int, [_P, _P, _P, _P]),
    "ssd_select_defaults": (None, [C.POINTER(ssd_select_params)]),
    "ssd_select_skip": (C.c_int, [_P, C.c_int, C.POINTER(ssd_select_params), _P, _P, _P]),
    "ssd_uniform_skip": (C.c_int, [C.c_int, C.POINTER(ssd_select_params), _P]),
    "ssd_search_defaults": (None, [C.POINTER(ssd_search_params)]),
    "ssd_search_create": (C.c_int, [C.c_int, C.POINTER(ssd_search_params), C.POINTER(ssd_select_params), C.POINTER(_P)]),
    "ssd_search_destroy": (None, [_P]),
    "ssd_search_mask": (C.c_int, [_P, _P]),
    "ssd_search_observe": (C.c_int, [_P, C.c_int, _P, _P, _P]),
    "ssd_search_status": (C.c_int, [_P, _P, _P]),
    "ssd_hbm_read_probe": (C.c_int, [_P, C.c_size_t, C.c_int, _P, _P]),
    "ssd_kv_poison_stale": (C.c_int, [_P]),
    "ssd_profile_select": (C.c_int, [_P, C.c_int]),
    "ssd_profile_read": (C.c_int, [_P, _P, _P]),
    "ssd_set_graphs": (C.c_int, [_P, C.c_int]),
}

_lib = None


def lib():
    """Loads libssd.so (built by paper_2604_14612_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libssd.so is not built: run `python -m paper_2604_14612_amd.build` "
                              "(or __graft_entry__.build()); there is no fallback path")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


# ---- host-only policy calls ----------------------------------------------------------------

def select_defaults(**overrides) -> ssd_select_params:
    p = ssd_select_params()
    lib().ssd_select_defaults(C.byref(p))
    for k, v in overrides.items():
        setattr(p, "lambda_" if k in ("lam", "lambda") else k, v)
    return p


def search_defaults(**overrides) -> ssd_search_params:
    p = ssd_search_params()
    lib().ssd_search_defaults(C.byref(p))
    for k, v in overrides.items():
        setattr(p, k, v)
    return p


def ssd_select_skip(conf: Sequence[float], params: Optional[ssd_select_params] = None, want_margin=False):
    p = params or select_defaults()
    c = np.ascontiguousarray(np.asarray(conf, dtype=np.float64))
    L = c.shape[0]
    mask = np.zeros(L, np.uint8)
    n = C.c_int32()
    margin = np.zeros(L, np.float64) if want_margin else None
    rc = lib().ssd_select_skip(_np_ptr(c), L, C.byref(p), _np_ptr(mask), C.addressof(n), _np_ptr(margin))
    if rc:
        raise SsdError(rc)
    return (mask, margin) if want_margin else mask


def ssd_uniform_skip(n_layers: int, params: Optional[ssd_select_params] = None) -> np.ndarray:
    p = params or select_defaults()
    mask = np.zeros(n_layers, np.uint8)
    rc = lib().ssd_uniform_skip(n_layers, C.byref(p), _np_ptr(mask))
    if rc:
        raise SsdError(rc)
    return mask


def pack_weights(weights: dict, per_layer: bool = False) -> dict:
    """Copies the weight matrices into ONE device allocation, in the order a forward pass reads them (embedding,
    then per layer wq wk wv wo wg wu wd, then the LM head), each on a 2 MiB boundary, and returns a dict of views.
    Memory plumbing only: the library takes whatever pointers it is given; one arena streams a few per cent faster
    than a few hundred separate allocations.  per_layer=True makes one arena per layer instead and releases the
    source tensors of a layer as soon as they are copied (the lists of the input dict are emptied), for models of
    which two copies do not fit."""
    import torch
    per = ("wq", "wk", "wv", "wo", "wg", "wu", "wd")
    L = len(weights["wq"])
    ALIGN = 2 << 20     # every matrix starts on a 2 MiB boundary of the arena (measured: 256-byte packing cost 4 % at 13B)
    nbytes = lambda t: (t.numel() * t.element_size() + ALIGN - 1) // ALIGN * ALIGN
    dev = weights["embed"].device

    def fill(tensors):
        arena = torch.empty(sum(nbytes(t) for t in tensors) + ALIGN, dtype=torch.uint8, device=dev)
        views, off = [], (-arena.data_ptr()) % ALIGN
        for t in tensors:
            v = arena[off:off + t.numel() * t.element_size()].view(t.dtype).view(t.shape)
            v.copy_(t)
            off += nbytes(t)
            views.append(v)
        return arena, views

    out = {k: (list(v) if isinstance(v, list) else v) for k, v in weights.items()}
    if not per_layer:
        flat = [weights["embed"]] + [weights[k][l] for l in range(L) for k in per] + [weights["lm_head"]]
        arena, views = fill(flat)
        out["embed"], out["lm_head"] = views[0], views[-1]
        for l in range(L):
            for i, k in enumerate(per):
                out[k][l] = views[1 + l * len(per) + i]
        out["_arena"] = arena
        return out
    arenas = []
    for l in range(L):
        arena, views = fill([weights[k][l] for k in per])
        for i, k in enumerate(per):
            out[k][l] = views[i]
            weights[k][l] = None            # drop the source tensor of this layer
        arenas.append(arena)
        torch.cuda.synchronize()
        torch.cuda.empty_cache()            # hand the freed blocks back so that the next arena fits
    out["_arena"] = arenas
    return out


class Search:
    """ssd_search_* handle (Section 3.3 search check)."""

    def __init__(self, n_layers: int, search: Optional[ssd_search_params] = None,
                 select: Optional[ssd_select_params] = None):
        self.L = n_layers
        sp = search or search_defaults()
        sel = select or select_defaults()
        h = C.c_void_p()
        rc = lib().ssd_search_create(n_layers, C.byref(sp), C.byref(sel), C.byref(h))
        if rc:
            raise SsdError(rc)
        self._h = h
        self.active = True

    def mask(self) -> np.ndarray:
        m = np.zeros(self.L, np.uint8)
        rc = lib().ssd_search_mask(self._h, _np_ptr(m))
        if rc:
            raise SsdError(rc)
        return m

    def observe(self, n_accepted: int, conf=None) -> np.ndarray:
        c = None if conf is None else np.ascontiguousarray(np.asarray(conf, dtype=np.float64))
        m = np.zeros(self.L, np.uint8)
        act = C.c_int32()
        rc = lib().ssd_search_observe(self._h, int(n_accepted), _np_ptr(c), _np_ptr(m), C.addressof(act))
        if rc:
            raise SsdError(rc)
        self.active = bool(act.value)
        return m

    def status(self):
        r, b = C.c_int32(), C.c_double()
        lib().ssd_search_status(self._h, C.addressof(r), C.addressof(b))
        return r.value, b.value

    def close(self):
        if getattr(self, "_h", None):
            lib().ssd_search_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()


# ---- device context --------------------------------------------------------------------------

_DTYPE_CODE = {"fp32": 0, "bf16": 1, "fp16": 2}


def default_kv_dtype(shape) -> str:
    """Element type of the KV cache when the caller names none: fp32.  Only the weights are 16-bit in the benchmark
    workloads; activations, K and V included, stay fp32, which keeps deep models (40, 80 layers) within the logit
    tolerance of an unrounded reference.  "bf16" / "fp16" halve the cache traffic at the cost of that margin."""
    return "fp32"


def make_config(shape, max_seq: int, max_k: int = 8, conf_taps: int = 2, conf_clamp: float = 1e4,
                conf_eps: float = 1e-10, kv_dtype: Optional[str] = None, conf_window: int = 0) -> ssd_config:
    return ssd_config(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim,
                      shape.d_ffn, shape.vocab, int(max_seq), shape.rms_eps, shape.rope_base,
                      _DTYPE_CODE[shape.dtype], conf_taps, conf_clamp, conf_eps, max_k,
                      _DTYPE_CODE[kv_dtype or default_kv_dtype(shape)], int(conf_window))


class Context:
    """One decoding context on the current torch device/stream.

    weights: dict as produced by synth.make_weights, tensors already on the GPU.
    """

    def __init__(self, shape, weights, max_seq: int, max_k: int = 8, **cfg_kw):
        import torch
        self._torch = torch
        self._l = lib()
        self.shape = shape
        self.cfg = make_config(shape, max_seq, max_k, **cfg_kw)
        self.kv_dtype = {v: k for k, v in _DTYPE_CODE.items()}[self.cfg.kv_dtype]
        h = C.c_void_p()
        # a stream of its own (default priority): the legacy default stream cannot be graph-captured
        self.stream = torch.cuda.Stream()
        self._check(self._l.ssd_create(C.byref(self.cfg), C.c_void_p(self.stream.cuda_stream), C.byref(h)), None)
        self._h = h
        nbytes = self._l.ssd_workspace_bytes(C.byref(self.cfg))
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()      # weights / workspace were produced on other streams
        self._check(self._l.ssd_set_workspace(self._h, C.c_void_p(self.workspace.data_ptr()), nbytes))
        self._weights = weights   # keep tensors alive
        L = shape.n_layers
        exp_dt = {"bf16": torch.bfloat16, "fp16": torch.float16, "fp32": torch.float32}[shape.dtype]

        def dp(t, dt):
            assert t.is_cuda and t.is_contiguous() and t.dtype == dt, (t.device, t.dtype)
            return t.data_ptr()

        self._arrs = {}

        def arr(name, dt):
            a = (C.c_void_p * L)(*[dp(weights[name][l], dt) for l in range(L)])
            self._arrs[name] = a
            return C.cast(a, C.POINTER(C.c_void_p))

        w = ssd_weights(dp(weights["embed"], exp_dt), dp(weights["lm_head"], exp_dt),
                        dp(weights["final_norm"], torch.float32),
                        arr("attn_norm", torch.float32), arr("wq", exp_dt), arr("wk", exp_dt), arr("wv", exp_dt),
                        arr("wo", exp_dt), arr("mlp_norm", torch.float32), arr("wg", exp_dt), arr("wu", exp_dt),
                        arr("wd", exp_dt))
        self._check(self._l.ssd_load_weights(self._h, C.byref(w)))
        if os.environ.get("SSD_NO_GRAPHS"):       # e.g. under counter-collecting profilers
            self.ssd_set_graphs(False)

    def _check(self, rc, h="self"):
        if rc != 0:
            msg = ""
            if h is not None and getattr(self, "_h", None):
                msg = self._l.ssd_last_error(self._h).decode()
            raise SsdError(rc, msg)

    def close(self):
        if getattr(self, "_h", None):
            self._l.ssd_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    # -- calls, same names as the C ABI ---------------------------------------------------------
    def ssd_reset(self):
        self._check(self._l.ssd_reset(self._h))

    def ssd_prefill(self, tokens: Sequence[int]) -> int:
        t = np.ascontiguousarray(np.asarray(tokens, dtype=np.int32))
        out = C.c_int32()
        self._check(self._l.ssd_prefill(self._h, _np_ptr(t), t.shape[0], C.addressof(out)))
        return out.value

    def ssd_decode(self) -> int:
        out = C.c_int32()
        self._check(self._l.ssd_decode(self._h, C.addressof(out)))
        return out.value

    def ssd_draft_step(self, skip_mask, k: int, want_maxprob: bool = False):
        m = np.ascontiguousarray(np.asarray(skip_mask, dtype=np.uint8))
        L = self.shape.n_layers
        if m.shape not in ((L,), (2 * L,)):
            raise SsdError(SSD_EINVAL, "skip_mask must have n_layers entries (or 2 * n_layers: attention / MLP sub-blocks)")
        d = np.zeros(max(k, 1), np.int32)
        mp = np.zeros(max(k, 1), np.float32) if want_maxprob else None
        fn = self._l.ssd_draft_step if m.shape[0] == L else self._l.ssd_draft_step_sub
        self._check(fn(self._h, _np_ptr(m), int(k), _np_ptr(d), _np_ptr(mp)))
        return (d[:k].tolist(), mp[:k].tolist()) if want_maxprob else d[:k].tolist()

    def ssd_draft_adaptive(self, skip_mask, k_max: int, gamma: float):
        """-> (tokens, their draft max-probabilities); len(tokens) is the k to verify."""
        m = np.ascontiguousarray(np.asarray(skip_mask, dtype=np.uint8))
        if m.shape != (self.shape.n_layers,):
            raise SsdError(SSD_EINVAL, "skip_mask must have n_layers entries")
        d = np.zeros(max(k_max, 1), np.int32)
        mp = np.zeros(max(k_max, 1), np.float32)
        k = C.c_int32()
        self._check(self._l.ssd_draft_adaptive(self._h, _np_ptr(m), int(k_max), float(gamma), _np_ptr(d), _np_ptr(mp),
                                               C.addressof(k)))
        return d[:k.value].tolist(), mp[:k.value].tolist()

    def ssd_verify(self, draft: Sequence[int]):
        d = np.ascontiguousarray(np.asarray(draft, dtype=np.int32))
        k = d.shape[0]
        y = np.zeros(k + 1, np.int32)
        self._check(self._l.ssd_verify(self._h, _np_ptr(d), k, _np_ptr(y)))
        return y.tolist()

    def ssd_accept(self, draft: Sequence[int], target: Sequence[int]):
        d = np.ascontiguousarray(np.asarray(draft, dtype=np.int32))
        y = np.ascontiguousarray(np.asarray(target, dtype=np.int32))
        if y.shape[0] != d.shape[0] + 1:
            raise SsdError(SSD_EINVAL, "target must have k + 1 entries")
        a, nx = C.c_int32(), C.c_int32()
        self._check(self._l.ssd_accept(self._h, _np_ptr(d), _np_ptr(y), d.shape[0], C.addressof(a), C.addressof(nx)))
        return a.value, nx.value

    def ssd_force_commit(self, draft: Sequence[int], n_accepted: int, next_token: int):
        d = np.ascontiguousarray(np.asarray(draft, dtype=np.int32))
        self._check(self._l.ssd_force_commit(self._h, _np_ptr(d), d.shape[0], int(n_accepted), int(next_token)))

    def ssd_copy_logits(self, row_begin: int, n_rows: int) -> np.ndarray:
        out = np.empty((n_rows, self.shape.vocab), np.float32)
        self._check(self._l.ssd_copy_logits(self._h, int(row_begin), int(n_rows), _np_ptr(out)))
        return out

    def ssd_layer_confidence(self, row_begin: int = 0, n_rows: int = 1, detail: bool = False, static: bool = False):
        """static=True calls ssd_layer_confidence_static (no workspace scratch, no allocation) instead."""
        L = self.shape.n_layers
        conf = np.empty((n_rows, L), np.float32)
        tc = np.empty((n_rows, L, 2), np.float32) if detail else None
        tm = np.empty((n_rows, L, 2), np.float32) if detail else None
        ta = np.empty((n_rows, L, 2), np.int32) if detail else None
        fn = self._l.ssd_layer_confidence_static if static else self._l.ssd_layer_confidence
        self._check(fn(self._h, int(row_begin), int(n_rows), _np_ptr(conf), _np_ptr(tc), _np_ptr(tm), _np_ptr(ta)))
        return (conf, {"conf": tc, "maxprob": tm, "argmax": ta}) if detail else conf

    def ssd_window_confidence(self, detail: bool = False):
        """-> conf[L] over the context window (and, with detail, per-tap means [L][2] and the positions in the window)."""
        L = self.shape.n_layers
        conf = np.empty(L, np.float32)
        tc = np.empty((L, 2), np.float32) if detail else None
        n = C.c_int32()
        self._check(self._l.ssd_window_confidence(self._h, _np_ptr(conf), _np_ptr(tc), C.addressof(n)))
        return (conf, tc, n.value) if detail else conf

    def ssd_kv_poison_stale(self):
        self._check(self._l.ssd_kv_poison_stale(self._h))

    def ssd_set_graphs(self, enable: bool):
        self._check(self._l.ssd_set_graphs(self._h, 1 if enable else 0))

    def ssd_profile_select(self, kernel_id: int):
        self._check(self._l.ssd_profile_select(self._h, int(kernel_id)))

    def ssd_profile_read(self):
        n, ms = C.c_int64(), C.c_double()
        self._check(self._l.ssd_profile_read(self._h, C.addressof(n), C.addressof(ms)))
        return n.value, ms.value

    def ssd_get_stats(self) -> dict:
        s = ssd_stats()
        self._check(self._l.ssd_get_stats(self._h, C.byref(s)))
        return {name: getattr(s, name) for name, _ in ssd_stats._fields_}


def ssd_hbm_read_probe(tensor, iters: int = 10) -> float:
    """Mean milliseconds for one read-only pass over `tensor` (device memory)."""
    import torch
    ms = C.c_float()
    nbytes = tensor.numel() * tensor.element_size()
    rc = lib().ssd_hbm_read_probe(C.c_void_p(tensor.data_ptr()), nbytes, iters,
                                  C.c_void_p(torch.cuda.current_stream().cuda_stream), C.addressof(ms))
    if rc:
        raise SsdError(rc)
    return ms.value
