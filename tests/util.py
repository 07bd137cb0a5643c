"""Helpers shared by the tests: glue between the input generator, the oracle and the library."""
import numpy as np
import torch

import synth
from oracle import transformer


def np_weights(w: dict, dtype=np.float32) -> dict:
    """Generator weights (torch, any float dtype) -> NumPy arrays of `dtype` (values unchanged)."""
    cv = lambda t: t.detach().to("cpu", torch.float64).numpy().astype(dtype)
    return {"tok_embed": cv(w["tok_embed"]), "lm_head": cv(w["lm_head"]), "final_norm": cv(w["final_norm"]),
            "layers": [{k: cv(v) for k, v in lay.items()} for lay in w["layers"]]}


def oracle_model(w: dict, shape: synth.ModelShape, dtype=np.float32) -> transformer.Model:
    return transformer.Model(np_weights(w, dtype), shape.n_heads, shape.n_kv_heads, shape.head_dim,
                             shape.rope_theta, shape.rms_eps, dtype=dtype)


class NpUniforms:
    """synth.Uniforms as float64 NumPy arrays (same values: every uniform is exact in fp32)."""

    def __init__(self, u: synth.Uniforms):
        self.draft = u.draft.numpy().astype(np.float64)
        self.accept = u.accept.numpy().astype(np.float64)
        self.resample = u.resample.numpy().astype(np.float64)


def gpu_available() -> bool:
    return torch.cuda.is_available()


def bf16_pair(cfg):
    """Generator weights rounded to bf16 (the values both the oracle and the library receive)."""
    tw, dw = synth.make_pair(cfg)
    rnd = lambda t: t.to(torch.bfloat16)

    def conv(w, memo):
        key = id(w)
        if key in memo:
            return memo[key]
        out = {"tok_embed": rnd(w["tok_embed"]), "lm_head": rnd(w["lm_head"]), "final_norm": rnd(w["final_norm"]),
               "layers": [{k: rnd(v) for k, v in lay.items()} for lay in w["layers"]]}
        memo[key] = out
        return out

    memo = {}
    t = conv(tw, memo)
    if cfg.draft_from_target_layers:
        k = cfg.draft_from_target_layers
        d = {"tok_embed": t["tok_embed"], "lm_head": t["lm_head"], "final_norm": t["final_norm"],
             "layers": t["layers"][:k]}
    else:
        d = conv(dw, memo)
    return t, d
