"""Independent float64 reference of the decoder made of PyTorch library ops (CPU tests only).

Full-sequence recompute, no cache: rms_norm, scaled_dot_product_attention, silu, linear, embedding, with the rotary
embedding written as a complex multiplication -- a different formulation from the oracle's incremental, pairwise
one.  It shares no code with oracle/ and none with the HIP library; the CPU tests pin the oracle to it.
"""
import numpy as np
import torch
import torch.nn.functional as F

_ST = {"bf16": torch.bfloat16, "fp16": torch.float16, "fp32": torch.float32}


def _store(t, kv_storage):
    """What a K/V cache of the given storage type holds for t: exact, or the library's casts via fp32."""
    if kv_storage == "exact":
        return t
    return t.to(torch.float32).to(_ST[kv_storage]).to(torch.float64)


def reference_forward(shape, w, tokens, kv_storage="model", skip_mask=None, n_verified=None):
    """Logits [T][V] and hidden-state taps [T][L][2][d] of the token sequence, recomputed in full.

    kv_storage: "exact" (nothing rounded), "model" (K after the rotary embedding and V pass through the weight
    type, the half-precision cache of Section 4.1.1) or an explicit type name.
    skip_mask / n_verified: the draft model of Section 3 on rows n_verified.. -- those rows leave out the layers of
    the skip set (L entries) or single attention / MLP sub-blocks (2L entries, [2l] attention, [2l+1] MLP), and in an
    executed attention sub-block they attend the full model's K/V at positions < n_verified (the verified cache) and
    the draft rows' own K/V from n_verified on.  Rows < n_verified always run the full model.
    """
    dd = torch.float64
    if kv_storage == "model":
        kv_storage = shape.dtype
    T = len(tokens)
    L, H, Hkv, hd, d = shape.n_layers, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_model
    nv = T if n_verified is None else n_verified
    skip = np.zeros(2 * L, bool) if skip_mask is None else np.asarray(skip_mask).astype(bool)
    if skip.shape[0] == L:                 # whole layers: both sub-blocks
        skip = np.repeat(skip, 2)
    x = F.embedding(torch.tensor(tokens, dtype=torch.long), w["embed"].to(dd))
    pos = torch.arange(T, dtype=dd)
    inv = shape.rope_base ** (-torch.arange(0, hd, 2, dtype=dd) / hd)       # base^(-2i/hd)
    rot = torch.polar(torch.ones(T, hd // 2, dtype=dd), pos[:, None] * inv[None, :])  # e^{i p theta_i}

    def rope(t):                       # t: [T][heads][hd], pairs (i, i+hd/2)
        z = torch.complex(t[..., : hd // 2], t[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    taps = torch.zeros(T, L, 2, d, dtype=dd)
    for l in range(L):
        # rows that run a sub-block: all verified rows, and the draft rows unless it is skipped
        live_a = torch.ones(T, dtype=torch.bool)
        live_m = torch.ones(T, dtype=torch.bool)
        if skip[2 * l]:
            live_a[nv:] = False
        if skip[2 * l + 1]:
            live_m[nv:] = False
        h = F.rms_norm(x, (d,), w["attn_norm"][l].to(dd), eps=shape.rms_eps)
        q = rope(F.linear(h, w["wq"][l].to(dd)).view(T, H, hd))
        k = _store(rope(F.linear(h, w["wk"][l].to(dd)).view(T, Hkv, hd)), kv_storage)
        v = _store(F.linear(h, w["wv"][l].to(dd)).view(T, Hkv, hd), kv_storage)
        k = k.repeat_interleave(H // Hkv, dim=1)
        v = v.repeat_interleave(H // Hkv, dim=1)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True)[0]
        xa = x + F.linear(o.transpose(0, 1).reshape(T, H * hd), w["wo"][l].to(dd))
        xa = torch.where(live_a[:, None], xa, x)
        h = F.rms_norm(xa, (d,), w["mlp_norm"][l].to(dd), eps=shape.rms_eps)
        xm = xa + F.linear(F.silu(F.linear(h, w["wg"][l].to(dd))) * F.linear(h, w["wu"][l].to(dd)), w["wd"][l].to(dd))
        xm = torch.where(live_m[:, None], xm, xa)
        taps[:, l, 0], taps[:, l, 1] = xa, xm
        x = xm
    h = F.rms_norm(x, (d,), w["final_norm"].to(dd), eps=shape.rms_eps)
    return F.linear(h, w["lm_head"].to(dd)).numpy(), taps.numpy()


def reference_logits(shape, w, tokens, kv_storage="model"):
    return reference_forward(shape, w, tokens, kv_storage)[0]


def reference_confidence(shape, w, hidden, clamp=1e4, eps=1e-10):
    """Eq. 1-4 of one hidden state with scipy's softmax: final norm, LM head, fp32 cast, clamp, entropy."""
    from scipy.special import softmax
    dd = torch.float64
    h = F.rms_norm(torch.from_numpy(np.asarray(hidden)), (shape.d_model,), w["final_norm"].to(dd), eps=shape.rms_eps)
    z = F.linear(h, w["lm_head"].to(dd)).numpy().astype(np.float32).astype(np.float64)
    p = softmax(np.clip(z, -clamp, clamp))
    return 1.0 + float(np.sum(p * np.log(p + eps))) / np.log(shape.vocab)
