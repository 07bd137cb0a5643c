"""Helpers shared by the tests: glue between the input generator, the oracle and the library."""
import numpy as np
import torch

import synth
from oracle import transformer


def np_weights(w: dict, dtype=np.float32) -> dict:
    """Generator weights (torch, any float dtype) -> NumPy arrays of `dtype` (values unchanged)."""
    if dtype == np.float32:      # bf16 / fp32 -> fp32 is exact; no fp64 detour for multi-gigabyte tensors
        cv = lambda t: np.ascontiguousarray(t.detach().to("cpu").float().numpy())
    else:
        cv = lambda t: t.detach().to("cpu", torch.float64).numpy().astype(dtype)
    return {"tok_embed": cv(w["tok_embed"]), "lm_head": cv(w["lm_head"]), "final_norm": cv(w["final_norm"]),
            "layers": [{k: cv(v) for k, v in lay.items()} for lay in w["layers"]]}


def oracle_model(w: dict, shape: synth.ModelShape, dtype=np.float32, act_bf16: bool = False) -> transformer.Model:
    return transformer.Model(np_weights(w, dtype), shape.n_heads, shape.n_kv_heads, shape.head_dim,
                             shape.rope_theta, shape.rms_eps, dtype=dtype, act_bf16=act_bf16)


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


LOGIT_TOL = 2e-2        # max |library - oracle| logit error relative to the row's logit range (bf16 path vs fp32)
EXACT_MARGIN = 2e-5     # decisions taken from the same fp32 logits may differ only this close to a flip
#                         (the kernels form exp() with the hardware's exp2 and a reciprocal: relative 1e-5)


class LockstepModel:
    """The feed / rollback / len interface of the oracle's loops, served by the library's own forward and checked
    against the oracle's forward at every call.

    `ctx` is a second context of the same weights whose *target* slot holds the model in question; feed(tokens)
    runs spec_verify on it and returns the library's fp32 logits, after comparing them row by row with the fp32
    oracle forward `ocm` on the same tokens (LOGIT_TOL of the row's range).  The oracle's loop then takes its
    decisions (fp64 sampling arithmetic, its own bookkeeping) from exactly the logits the library's loop sees, so
    the two token streams must be identical except where a decision sits within EXACT_MARGIN of flipping: the
    forward is compared within its bf16 tolerance, the decisions exactly, and neither forgives the other."""

    def __init__(self, ctx, ocm=None, tol=LOGIT_TOL):
        self.ctx, self.ocm, self.tol = ctx, ocm, tol
        self.worst, self.n_rows = 0.0, 0
        self._expect_prefix = None

    def begin(self, prompt, oracle_ready=False):
        """Prompt pass on the library side and on the oracle side (unless the oracle's cache already holds
        prompt[:-1]); the loop's own feed of prompt[:-1] is then recognised and skipped."""
        prompt = [int(t) for t in prompt]
        self.ctx.prefill(prompt)
        if self.ocm is not None and len(prompt) > 1:
            if oracle_ready:
                assert self.ocm.len == len(prompt) - 1
            else:
                self.ocm.feed(prompt[:-1])
        self._expect_prefix = prompt[:-1] if len(prompt) > 1 else None
        return self

    @property
    def len(self):
        from paper_2408_11850_amd import SPEC_TARGET
        return self.ctx.kv_len(SPEC_TARGET)

    def feed(self, tokens):
        tokens = [int(t) for t in tokens]
        if self._expect_prefix is not None:
            assert tokens == self._expect_prefix, "the loop's first feed must be the prompt without its last token"
            self._expect_prefix = None
            return None
        got = self.ctx.verify(tokens, want_logits=True)
        if self.ocm is not None:
            ref = self.ocm.feed(tokens)
            rng = ref.max(axis=-1) - ref.min(axis=-1)
            err = float((np.abs(got - ref).max(axis=-1) / rng).max())
            self.worst = max(self.worst, err)
            self.n_rows += len(tokens)
            assert err <= self.tol, f"logits off by {err:.3e} of the row's range at cache length {self.len}"
        return got

    def rollback(self, new_len):
        from paper_2408_11850_amd import SPEC_TARGET
        self.ctx.rollback_kv(SPEC_TARGET, int(new_len))
        if self.ocm is not None:
            self.ocm.rollback(int(new_len))
