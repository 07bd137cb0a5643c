"""Oracle: Llama-style decoder forward with a KV cache (test infrastructure only).

The paper treats the two models as black boxes M_p(.), M_q(.) that return next-token
logits from one forward (Section 2, "Notations"); it names Llama-family decoders in
bf16 (Section 4.1, App. C model table).  This file writes that forward out plainly:
RMSNorm -> QKV -> RoPE -> causal attention over the cache (grouped-query) -> output
projection + residual -> RMSNorm -> SwiGLU FFN + residual; final RMSNorm -> LM head.

All matrices are [out_features, in_features] (y = x @ W.T).  Arithmetic runs in the
dtype of `Model.dtype` (float32 by default, float64 for pins).

Precision.  The paper runs its models in bfloat16 (App. C: weights loaded in bf16).  The plain
forward above keeps every activation in `dtype`; with `act_bf16=True` the same forward rounds
the activations that a bf16 deployment hands from one operator to the next to bfloat16
(round-to-nearest-even) - the input of each projection, q / k / v after RoPE (k, v are what
the cache holds), the soft-max weights that multiply v, the attention output and the SwiGLU
product - while sums, the residual stream, norms' statistics, soft-max and logits stay in
`dtype`.  The input of a projection is rounded as h * gain and the factor 1/rms is applied to
the projection's output (the projection is linear, so this is the same operator; bf16 has the
same relative step at any scale, so it is also the same amount of rounding).  The variant
exists to tell rounding noise from mistakes: the distance between the two variants is what
bf16 activations cost at a given depth, and an implementation with these rounding points
should sit much closer to the rounded variant than to the plain one.
"""
from __future__ import annotations

import numpy as np


class Model:
    """Weights of one decoder.  `w` mirrors the generator's dict layout, as NumPy arrays."""

    def __init__(self, w: dict, n_heads: int, n_kv_heads: int, head_dim: int,
                 rope_theta: float = 10000.0, rms_eps: float = 1e-5, dtype=np.float32, act_bf16: bool = False):
        self.dtype = dtype
        self.act_bf16 = act_bf16
        cv = lambda a: np.ascontiguousarray(np.asarray(a, dtype=dtype))
        self.tok_embed = cv(w["tok_embed"])
        self.lm_head = cv(w["lm_head"])
        self.final_norm = cv(w["final_norm"])
        self.layers = [{k: cv(v) for k, v in lay.items()} for lay in w["layers"]]
        self.n_heads, self.n_kv_heads, self.head_dim = n_heads, n_kv_heads, head_dim
        self.rope_theta, self.rms_eps = rope_theta, rms_eps
        self.vocab, self.d_model = self.tok_embed.shape


class KVCache:
    """Per-layer keys/values of the tokens fed so far.  Rollback only shortens `len`."""

    def __init__(self, model: Model, max_len: int):
        L, H, D = len(model.layers), model.n_kv_heads, model.head_dim
        self.k = np.zeros((L, max_len, H, D), dtype=model.dtype)
        self.v = np.zeros((L, max_len, H, D), dtype=model.dtype)
        self.len = 0

    def rollback(self, new_len: int):
        if not 0 <= new_len <= self.len:
            raise ValueError("rollback target outside [0, len]")
        self.len = new_len


def bf16_round(x):
    """Round to the nearest bfloat16 (ties to even), returned in x's dtype.  bfloat16 = the upper 16 bits of an
    IEEE float32; finite inputs only."""
    x = np.asarray(x)
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(x.dtype)


def rmsnorm(x, gain, eps):
    """x / sqrt(mean(x^2) + eps) * gain, per row."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + x.dtype.type(eps)) * gain


def norm_input(model, h, gain):
    """(a, scale) with norm(h) @ W.T == (a @ W.T) * scale: plainly a = rmsnorm(h) and scale = 1; with bf16
    activations a = bf16(h * gain) and scale = 1/rms(h), per row."""
    if not model.act_bf16:
        return rmsnorm(h, gain, model.rms_eps), h.dtype.type(1.0)
    ms = np.mean(h * h, axis=-1, keepdims=True)
    return bf16_round(h * gain), 1.0 / np.sqrt(ms + h.dtype.type(model.rms_eps))


def rope(x, positions, theta):
    """Rotate pairs (i, i + D/2) of the last axis by angle pos * theta^(-2i/D).  x: [M, H, D]."""
    D = x.shape[-1]
    half = D // 2
    i = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * i / D)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]      # [M, half]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def layer_forward(model: Model, cache: KVCache, l: int, w: dict, h, n: int):
    """One decoder layer over the M rows of h (the tokens at positions n .. n+M-1): appends their keys / values to
    layer l of the cache (cache.len is not moved) and returns the new residual stream.  `w`: the layer's matrices
    and gains as arrays of model.dtype.  forward() is embedding -> this for every layer -> head(); it is a function
    of its own so that a test can hand over a deep model's layers one at a time."""
    M = h.shape[0]
    H, Hkv, D = model.n_heads, model.n_kv_heads, model.head_dim
    group = H // Hkv
    pos = np.arange(n, n + M)
    scale = model.dtype(1.0 / np.sqrt(D))
    rb = bf16_round if model.act_bf16 else (lambda x: x)
    a, sc = norm_input(model, h, w["attn_norm"])
    q = ((a @ w["wq"].T) * sc).reshape(M, H, D)
    k = ((a @ w["wk"].T) * sc).reshape(M, Hkv, D)
    v = rb(((a @ w["wv"].T) * sc).reshape(M, Hkv, D))
    q = rb(rope(q, pos, model.rope_theta))
    k = rb(rope(k, pos, model.rope_theta))
    cache.k[l, n:n + M] = k
    cache.v[l, n:n + M] = v
    o = np.zeros((M, H, D), dtype=model.dtype)
    for i in range(M):
        T = n + i + 1                                          # token i sees positions 0..n+i
        for j in range(H):
            kv = j // group
            s = (cache.k[l, :T, kv] @ q[i, j]) * scale        # [T]
            s = s - s.max()
            p = np.exp(s)
            o[i, j] = (rb(p) @ cache.v[l, :T, kv]) / p.sum()   # = softmax(s) @ V; the weights on V rounded if asked
    h = h + rb(o.reshape(M, H * D)) @ w["wo"].T
    b, sc = norm_input(model, h, w["ffn_norm"])
    z = rb(silu((b @ w["w_gate"].T) * sc) * ((b @ w["w_up"].T) * sc))
    return h + z @ w["w_down"].T


def head(model: Model, h) -> np.ndarray:
    """Final norm and LM head: logits [M, vocab] of the rows of h."""
    a, sc = norm_input(model, h, model.final_norm)
    return (a @ model.lm_head.T) * sc


def forward(model: Model, cache: KVCache, tokens) -> np.ndarray:
    """Feed M new tokens at positions cache.len .. cache.len+M-1; return logits [M, vocab].

    Row i is the logit vector of the token that follows tokens[i] (it attends to
    everything in the cache plus tokens[0..i]).
    """
    tokens = np.asarray(tokens, dtype=np.int64)
    M = tokens.shape[0]
    n = cache.len
    if n + M > cache.k.shape[1]:
        raise ValueError("KV cache overflow")
    h = model.tok_embed[tokens]                                   # [M, d]
    for l, w in enumerate(model.layers):
        h = layer_forward(model, cache, l, w, h, n)
    cache.len = n + M
    return head(model, h)


class CachedModel:
    """A model plus its cache, with the feed / rollback interface the loops use."""

    def __init__(self, model: Model, max_len: int):
        self.model = model
        self.cache = KVCache(model, max_len)
        self.n_forwards = 0

    @property
    def len(self) -> int:
        return self.cache.len

    def feed(self, tokens) -> np.ndarray:
        self.n_forwards += 1
        return forward(self.model, self.cache, tokens)

    def rollback(self, new_len: int):
        self.cache.rollback(new_len)
