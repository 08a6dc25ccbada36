"""Shapes and seeded random tensors of the five synthetic workloads.

The paper evaluates on trained Llama-2/3 checkpoints and text datasets (Section 4.1.1);
neither is available offline, so random-weight decoders of the same shapes and uniform
random prompts stand in for them.  Everything here is a pure function of (shape, seed,
device): the oracle and the HIP library are both handed the tensors this module returns.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass
from typing import Dict, List

import torch


@dataclass(frozen=True)
class ModelShape:
    """Decoder-only transformer shape (Llama layout: RMSNorm, RoPE, SwiGLU)."""
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    d_ffn: int
    vocab: int
    dtype: str = "bf16"          # weight storage: "bf16", "fp16" or "fp32"
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    init_depth: int = 0          # depth the residual-projection init is scaled for (0 = n_layers)
    resid_scale: float = 1.0     # extra factor on the two projections that write into the residual stream

    @property
    def head_dim(self) -> int:
        return self.d_model // self.n_heads

    @property
    def d_kv(self) -> int:
        return self.n_kv_heads * self.head_dim

    def layer_params(self) -> int:
        d, f = self.d_model, self.d_ffn
        return 2 * d * d + 2 * d * self.d_kv + 3 * d * f + 2 * d

    def bytes_per_weight(self) -> int:
        return 4 if self.dtype == "fp32" else 2


@dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration: a shape plus its decoding recipe."""
    name: str
    shape: ModelShape
    seed: int
    prompt_len: int
    new_tokens: int
    k: int                        # draft length
    max_skip_ratio: float = 0.6
    protect_ends: bool = True
    note: str = ""


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload(
        "tiny", ModelShape(4, 256, 4, 4, 688, 1024, dtype="fp32"),
        seed=0, prompt_len=32, new_tokens=32, k=4, protect_ends=False,
        note="fp32, skip set from confidence over all 4 layers"),
    "small": Workload(
        "small", ModelShape(24, 1024, 16, 16, 2816, 32000),
        seed=1, prompt_len=256, new_tokens=128, k=4, max_skip_ratio=0.5,
        note="confidence-based skipping, at most 50% of layers"),
    "llama7b": Workload(
        "llama7b", ModelShape(32, 4096, 32, 32, 11008, 32000),
        seed=2, prompt_len=512, new_tokens=256, k=4,
        note="k in {2,4,8}; vanilla decode timed alongside"),
    "llama13b": Workload(
        "llama13b", ModelShape(40, 5120, 40, 40, 13824, 32000),
        seed=3, prompt_len=1024, new_tokens=256, k=4,
        note="iterative skip-set refinement, at most 10 rounds"),
    "llama70b": Workload(
        "llama70b", ModelShape(80, 8192, 64, 8, 28672, 32000),
        seed=4, prompt_len=2048, new_tokens=128, k=4,
        note="grouped-query attention, ~138 GB of bf16 weights"),
    # Beyond the five benchmark configurations.
    # A model in which depth is redundant, as it is in trained LLMs and is not in a random-init one: every layer
    # writes a thousand times less into the residual stream, so a draft model with half the layers mostly agrees
    # with the full model.  Shows the pipeline at high acceptance (search reaching its goal, SSD faster than vanilla).
    "llama7b_redundant": Workload(
        "llama7b_redundant", ModelShape(32, 4096, 32, 32, 11008, 32000, resid_scale=0.001),
        seed=2, prompt_len=512, new_tokens=256, k=4,
        note="7B shape, o_proj / down_proj scaled by 0.001 (depth made redundant)"),
    "llama7b_f16": Workload(
        "llama7b_f16", ModelShape(32, 4096, 32, 32, 11008, 32000, dtype="fp16"),
        seed=2, prompt_len=512, new_tokens=256, k=4,
        note="the 7B shape in the paper's own precision (FP16 weights and cache)"),
    # the second model family of Section 4.1.1 (grouped heads, 128 256-entry vocabulary: a 1 GB LM head, so the
    # confidence pass is four times dearer per row)
    "llama3_8b": Workload(
        "llama3_8b", ModelShape(32, 4096, 32, 8, 14336, 128256, rope_base=500000.0),
        seed=5, prompt_len=512, new_tokens=128, k=4,
        note="Llama-3-8B shape in bf16"),
}

_PER_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "wg", "wu", "wd")
_GLOBAL = ("embed", "lm_head", "final_norm")


def weight_tensor_names() -> List[str]:
    return list(_GLOBAL) + list(_PER_LAYER)


def reduced_depth(shape: ModelShape, n_layers: int) -> ModelShape:
    """The first n_layers layers of the same model (used where the full depth is too slow for the CPU
    oracle): widths, seeds and the init scale of the full-depth model are kept, so every tensor equals
    the full model's."""
    return dataclasses.replace(shape, n_layers=n_layers, init_depth=shape.init_depth or shape.n_layers)


def _tensor_seed(seed: int, layer: int, tensor_id: int) -> int:
    # distinct stream per tensor so that no single RNG call has to cover a whole model
    return (seed * 1_000_003 + (layer + 1) * 1009 + tensor_id) & 0x7FFFFFFF


def _normal(shape, std, seed, device, dtype):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    t = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    t.mul_(std)
    return t.to(dtype)


def make_weights(shape: ModelShape, seed: int, device: str = "cpu",
                 norm_gain_std: float = 0.0, init_std: float = 0.02) -> Dict[str, object]:
    """Random-init decoder weights.

    All matrices are row-major [out_features][in_features] and ~N(0, init_std); the two
    projections that write into the residual stream (wo, wd) are scaled by resid_scale/sqrt(2*depth),
    depth = init_depth or n_layers.
    Norm gains are 1 (+ norm_gain_std * N(0,1) when a test wants them non-trivial).
    bf16 / fp16 models are rounded to their type once (round-to-nearest-even) and that rounded tensor is
    what every consumer sees.  The stream differs between CPU and GPU generators: move the
    returned tensors, do not regenerate them on the other device.
    """
    dt = {"bf16": torch.bfloat16, "fp16": torch.float16, "fp32": torch.float32}[shape.dtype]
    L, d, f, V = shape.n_layers, shape.d_model, shape.d_ffn, shape.vocab
    dq, dkv = shape.n_heads * shape.head_dim, shape.d_kv
    res_std = shape.resid_scale * init_std / math.sqrt(2.0 * (shape.init_depth or L))

    def gain(layer, tid):
        if norm_gain_std == 0.0:
            return torch.ones(d, device=device, dtype=torch.float32)
        g = _normal((d,), norm_gain_std, _tensor_seed(seed, layer, tid), device, torch.float32)
        return g + 1.0

    w: Dict[str, object] = {
        "embed": _normal((V, d), init_std, _tensor_seed(seed, -1, 0), device, dt),
        "lm_head": _normal((V, d), init_std, _tensor_seed(seed, -1, 1), device, dt),
        "final_norm": gain(-1, 2),
    }
    for name in _PER_LAYER:
        w[name] = []
    for l in range(L):
        w["attn_norm"].append(gain(l, 10))
        w["wq"].append(_normal((dq, d), init_std, _tensor_seed(seed, l, 11), device, dt))
        w["wk"].append(_normal((dkv, d), init_std, _tensor_seed(seed, l, 12), device, dt))
        w["wv"].append(_normal((dkv, d), init_std, _tensor_seed(seed, l, 13), device, dt))
        w["wo"].append(_normal((d, dq), res_std, _tensor_seed(seed, l, 14), device, dt))
        w["mlp_norm"].append(gain(l, 15))
        w["wg"].append(_normal((f, d), init_std, _tensor_seed(seed, l, 16), device, dt))
        w["wu"].append(_normal((f, d), init_std, _tensor_seed(seed, l, 17), device, dt))
        w["wd"].append(_normal((d, f), res_std, _tensor_seed(seed, l, 18), device, dt))
    return w


def make_prompt(vocab: int, n: int, seed: int) -> torch.Tensor:
    """n i.i.d. uniform token ids in [0, vocab), int32, on the CPU."""
    g = torch.Generator()
    g.manual_seed(_tensor_seed(seed, -2, 99))
    return torch.randint(0, vocab, (n,), generator=g, dtype=torch.int32)
