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
