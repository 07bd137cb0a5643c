"""Seeded synthetic inputs: weights, prompts and uniform random numbers.

This module holds none of the decoding method's arithmetic.  It only turns
(seed, tensor id, element index) counters into numbers, so that the CPU oracle
and the HIP library can be handed literally the same inputs.  Everything is a
pure function of its arguments (a counter-based hash), so a value does not
depend on generation order, chunking, or which other tensors were drawn.

The workloads stand in for the paper's pretrained Llama-family pairs and its
benchmark prompts (App. C, model-configuration table): random-init decoder
weights of the same shapes, prompts of uniform token ids, batch 1.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, asdict
from typing import Dict, List, Optional

import torch

_M32 = 0xFFFFFFFF


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """Avalanche a tensor of 32-bit values held in int64 (a 32-bit finalizer)."""
    x = x ^ (x >> 16)
    x = (x * 0x85EBCA6B) & _M32
    x = x ^ (x >> 13)
    x = (x * 0xC2B2AE35) & _M32
    x = x ^ (x >> 16)
    return x


def _key32(*parts: int) -> int:
    """Fold python ints into one 32-bit key (host side, scalar)."""
    h = 0x9E3779B9
    for p in parts:
        p &= 0xFFFFFFFFFFFFFFFF
        for w in (p & _M32, (p >> 32) & _M32):
            h ^= w
            h ^= h >> 16
            h = (h * 0x85EBCA6B) & _M32
            h ^= h >> 13
            h = (h * 0xC2B2AE35) & _M32
            h ^= h >> 16
            h = (h + 0x7F4A7C15) & _M32
    return h


def hash_u32(key: int, index: torch.Tensor) -> torch.Tensor:
    """32-bit hash (in int64) of (key, index) for a tensor of int64 indices < 2^63."""
    lo = index & _M32
    hi = (index >> 32) & _M32
    h = _mix32(lo ^ key)
    h = _mix32((h + hi * 0x9E3779B9 + 0x7F4A7C15) & _M32)
    return h


def normal_tensor(shape, std: float, seed: int, tensor_id: int, dtype: torch.dtype,
                  device="cpu", chunk: int = 1 << 25) -> torch.Tensor:
    """i.i.d. N(0, std^2) tensor; element e is ndtri((hash(seed, tensor_id, e)+0.5)/2^32)*std."""
    numel = int(math.prod(shape))
    out = torch.empty(numel, dtype=dtype, device=device)
    key = _key32(seed, tensor_id, 0x6E6F726D)
    for s in range(0, numel, chunk):
        e = min(numel, s + chunk)
        idx = torch.arange(s, e, dtype=torch.int64, device=device)
        h = hash_u32(key, idx)
        del idx
        u = (h.to(torch.float64) + 0.5) * (1.0 / 4294967296.0)
        del h
        z = torch.special.ndtri(u)
        del u
        out[s:e] = (z * std).to(dtype)
        del z
    return out.view(*shape)


def uniform_array(n: int, seed: int, stream_id: int) -> torch.Tensor:
    """n float32 uniforms strictly inside (0,1): odd multiples of 2^-24 (exact in fp32), CPU tensor."""
    key = _key32(seed, stream_id, 0x756E6966)
    idx = torch.arange(n, dtype=torch.int64)
    h = hash_u32(key, idx)
    return (((h >> 9) * 2 + 1).to(torch.float32) * (1.0 / 16777216.0)).contiguous()


def prompt_tokens(n: int, vocab: int, seed: int) -> torch.Tensor:
    """n token ids uniform on [0, vocab), int32 CPU tensor."""
    key = _key32(seed, 0x70726F6D)
    idx = torch.arange(n, dtype=torch.int64)
    return (hash_u32(key, idx) % vocab).to(torch.int32).contiguous()


# --------------------------------------------------------------------------
# Model shapes
# --------------------------------------------------------------------------
@dataclass
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    d_ffn: int
    vocab: int
    head_dim: int = 0
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5

    def __post_init__(self):
        if self.head_dim == 0:
            self.head_dim = self.d_model // self.n_heads

    def params_per_layer(self) -> int:
        d, hq, hkv, dh, f = self.d_model, self.n_heads, self.n_kv_heads, self.head_dim, self.d_ffn
        return d * hq * dh * 2 + d * hkv * dh * 2 + 3 * d * f

    def streamed_params(self) -> int:
        """Matrix parameters read once per forward (layers + LM head; the embedding is gathered)."""
        return self.n_layers * self.params_per_layer() + self.vocab * self.d_model

    def kv_bytes_per_token(self, elem_bytes: int = 2) -> int:
        return 2 * self.n_layers * self.n_kv_heads * self.head_dim * elem_bytes


@dataclass
class PairConfig:
    name: str
    target: ModelShape
    draft: ModelShape
    draft_from_target_layers: int = 0   # >0: draft = first k target layers + shared embed / norm / LM head
    dtype: str = "bf16"                 # storage type of weights ("fp32" or "bf16")
    n_prompt: int = 0
    n_generate: int = 0
    gamma: int = 4
    temperature: float = 1.0
    logit_scale: float = 1.0
    seed_target: int = 1234
    seed_draft: int = 4321
    seed_prompt: int = 7
    seed_uniform: int = 99


def _truncate(shape: ModelShape, n_layers: int) -> ModelShape:
    d = asdict(shape)
    d["n_layers"] = n_layers
    return ModelShape(**d)


def config(name: str, depth: Optional[int] = None, draft_depth: Optional[int] = None) -> PairConfig:
    """The five workload pairs.  `depth`/`draft_depth` give a depth-truncated pair of the same widths."""
    if name == "tiny":
        t = ModelShape(4, 256, 4, 4, 688, 1024)
        c = PairConfig("tiny", t, _truncate(t, 1), draft_from_target_layers=1, dtype="fp32",
                       n_prompt=32, n_generate=64, gamma=4, logit_scale=8.0)
    elif name == "small":
        t = ModelShape(24, 2048, 16, 16, 5504, 32000)
        c = PairConfig("small", t, _truncate(t, 4), draft_from_target_layers=4,
                       n_prompt=512, n_generate=256, gamma=4)
    elif name == "7b_1b":
        c = PairConfig("7b_1b", ModelShape(32, 4096, 32, 32, 11008, 32000),
                       ModelShape(22, 2048, 32, 4, 5632, 32000), n_prompt=1024, n_generate=512, gamma=6)
    elif name == "33b_1b":
        c = PairConfig("33b_1b", ModelShape(62, 7168, 56, 56, 19200, 32256),
                       ModelShape(24, 2048, 16, 16, 5504, 32256), n_prompt=2048, n_generate=512, gamma=16)
    elif name == "70b_7b":
        c = PairConfig("70b_7b", ModelShape(80, 8192, 64, 8, 28672, 32000),
                       ModelShape(32, 4096, 32, 32, 11008, 32000), n_prompt=4096, n_generate=1024, gamma=8)
    else:
        raise ValueError(f"unknown config {name!r}")
    if depth is not None:
        c.target = _truncate(c.target, depth)
        if c.draft_from_target_layers:
            c.draft_from_target_layers = min(c.draft_from_target_layers, depth)
            c.draft = _truncate(c.draft, c.draft_from_target_layers)
    if draft_depth is not None:
        if c.draft_from_target_layers:
            c.draft_from_target_layers = min(draft_depth, c.target.n_layers)
            c.draft = _truncate(c.draft, c.draft_from_target_layers)
        else:
            c.draft = _truncate(c.draft, draft_depth)
    return c


# tensor ids: per-layer matrices get id = 16*layer + slot; globals sit above 1<<20
_SLOT = {"wq": 0, "wk": 1, "wv": 2, "wo": 3, "w_gate": 4, "w_up": 5, "w_down": 6, "attn_norm": 7, "ffn_norm": 8}
_GLOBAL = {"tok_embed": (1 << 20) + 0, "lm_head": (1 << 20) + 1, "final_norm": (1 << 20) + 2}
GAIN_STD = 0.3      # RMSNorm gains are 1 + GAIN_STD * N(0,1), a different vector per norm


def gain_tensor(d_model: int, seed: int, tensor_id: int, dtype: torch.dtype, device="cpu") -> torch.Tensor:
    """RMSNorm gain vector 1 + GAIN_STD * N(0,1) (distinct per tensor id), rounded to `dtype`.  Trained models have
    non-trivial gains; with all-ones gains a kernel that dropped the multiply or took the wrong vector would go
    unnoticed."""
    z = normal_tensor((d_model,), GAIN_STD, seed, tensor_id, torch.float64, device)
    return (1.0 + z).to(dtype)


def layer_matrix_shapes(s: ModelShape) -> Dict[str, tuple]:
    """All projection matrices are stored [out_features, in_features], row-major (y = x @ W^T)."""
    d, dh = s.d_model, s.head_dim
    return {"wq": (s.n_heads * dh, d), "wk": (s.n_kv_heads * dh, d), "wv": (s.n_kv_heads * dh, d),
            "wo": (d, s.n_heads * dh), "w_gate": (s.d_ffn, d), "w_up": (s.d_ffn, d), "w_down": (d, s.d_ffn)}


def make_weights(shape: ModelShape, seed: int, dtype: torch.dtype, device="cpu", std: float = 0.02) -> dict:
    """Random-init decoder weights: matrices N(0, std^2) and norm gains 1 + GAIN_STD * N(0,1), rounded to `dtype`."""
    w = {"tok_embed": normal_tensor((shape.vocab, shape.d_model), std, seed, _GLOBAL["tok_embed"], dtype, device),
         "lm_head": normal_tensor((shape.vocab, shape.d_model), std, seed, _GLOBAL["lm_head"], dtype, device),
         "final_norm": gain_tensor(shape.d_model, seed, _GLOBAL["final_norm"], dtype, device),
         "layers": []}
    mats = layer_matrix_shapes(shape)
    for l in range(shape.n_layers):
        lay = {"attn_norm": gain_tensor(shape.d_model, seed, 16 * l + _SLOT["attn_norm"], dtype, device),
               "ffn_norm": gain_tensor(shape.d_model, seed, 16 * l + _SLOT["ffn_norm"], dtype, device)}
        for name, shp in mats.items():
            lay[name] = normal_tensor(shp, std, seed, 16 * l + _SLOT[name], dtype, device)
        w["layers"].append(lay)
    return w


def make_pair(cfg: PairConfig, device="cpu") -> tuple:
    """(target weights, draft weights).  A derived draft aliases the target's tensors (same storage)."""
    dt = torch.float32 if cfg.dtype == "fp32" else torch.bfloat16
    tw = make_weights(cfg.target, cfg.seed_target, dt, device)
    if cfg.draft_from_target_layers:
        k = cfg.draft_from_target_layers
        dw = {"tok_embed": tw["tok_embed"], "lm_head": tw["lm_head"], "final_norm": tw["final_norm"],
              "layers": tw["layers"][:k]}
    else:
        dw = make_weights(cfg.draft, cfg.seed_draft, dt, device)
    return tw, dw


@dataclass
class Uniforms:
    """Per-step uniforms for the decoding loops, fixed before the loop runs.

    draft[t, i]  : draws the i-th draft token of step t
    accept[t, i] : tests the i-th verified draft token of step t
    resample[t]  : draws the corrected / bonus / autoregressive token of step t
    """
    draft: torch.Tensor
    accept: torch.Tensor
    resample: torch.Tensor


def make_uniforms(n_steps: int, gamma: int, seed: int) -> Uniforms:
    g = max(gamma, 1)
    return Uniforms(draft=uniform_array(n_steps * g, seed, 1).view(n_steps, g),
                    accept=uniform_array(n_steps * (g + 1), seed, 2).view(n_steps, g + 1),
                    resample=uniform_array(n_steps, seed, 3))
