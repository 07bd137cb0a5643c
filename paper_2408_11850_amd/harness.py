"""Builds synthetic model pairs on the GPU and drives the library's loops (used by bench.py and the tests)."""
from __future__ import annotations

import time
from typing import Optional, Tuple

import torch

import synth
from . import ALGO_AR, ALGO_PEARL, ALGO_SD, SPEC_DRAFT, SPEC_TARGET
from .binding import PackedModel, SpecContext, pack_from_dict, pack_model


def _generated_model(shape: synth.ModelShape, seed: int, device: str) -> PackedModel:
    """Generate each tensor on the device with the counter-based generator, pack it, drop the source."""
    mats = synth.layer_matrix_shapes(shape)
    ones = lambda: torch.ones(shape.d_model, dtype=torch.bfloat16, device=device)

    def get(layer: Optional[int], name: str) -> torch.Tensor:
        if name in ("final_norm", "attn_norm", "ffn_norm"):
            return ones()
        if layer is None:
            return synth.normal_tensor((shape.vocab, shape.d_model), 0.02, seed, synth._GLOBAL[name], torch.bfloat16,
                                       device)
        return synth.normal_tensor(mats[name], 0.02, seed, 16 * layer + synth._SLOT[name], torch.bfloat16, device)

    return pack_model(shape, get, device)


def build_pair(cfg: synth.PairConfig, device: str = "cuda", weights: Optional[Tuple[dict, dict]] = None):
    """(target PackedModel, draft PackedModel) for a workload.  With `weights` (generator dicts, e.g. the
    ones also handed to a reference implementation) those exact values are packed instead."""
    if weights is not None:
        tw, dw = weights
        target = pack_from_dict(cfg.target, tw, device)
        if cfg.draft_from_target_layers:
            draft = target.prefix(cfg.draft_from_target_layers, cfg.draft)
        else:
            draft = pack_from_dict(cfg.draft, dw, device)
        return target, draft
    target = _generated_model(cfg.target, cfg.seed_target, device)
    if cfg.draft_from_target_layers:
        draft = target.prefix(cfg.draft_from_target_layers, cfg.draft)
    else:
        draft = _generated_model(cfg.draft, cfg.seed_draft, device)
    return target, draft


def make_context(cfg: synth.PairConfig, target: PackedModel, draft: PackedModel, gamma_max: int,
                 temperature: Optional[float] = None, serial: bool = False, extra_seq: int = 0) -> SpecContext:
    max_seq = cfg.n_prompt + cfg.n_generate + 2 * gamma_max + 2 + extra_seq
    st = torch.cuda.Stream()
    sd = st if serial else torch.cuda.Stream()
    return SpecContext(target, draft, gamma_max, max_seq,
                       cfg.temperature if temperature is None else temperature, cfg.logit_scale, st, sd)


def calibrate_gamma(ctx: SpecContext, n_iter: int = 8, cap: int = 16) -> Tuple[int, float, float]:
    """Window size gamma = round(c), c = T(target forward) / T(draft forward) (paper Section 4.4.1),
    both timed alone at the current context length.  Leaves the caches as it found them."""
    lt, ld = ctx.kv_len(SPEC_TARGET), ctx.kv_len(SPEC_DRAFT)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n_iter):
        ctx.verify([0])
    torch.cuda.synchronize()
    tp = (time.perf_counter() - t0) / n_iter
    ctx.rollback_kv(SPEC_TARGET, lt)
    t0 = time.perf_counter()
    n_d = min(n_iter, 2 * ctx.gamma_max)
    for _ in range(n_d):
        ctx.draft_step(0.5)
    torch.cuda.synchronize()
    tq = (time.perf_counter() - t0) / n_d
    ctx.drop_drafts()
    ctx.rollback_kv(SPEC_DRAFT, ld)
    gamma = max(1, min(cap, int(round(tp / tq))))
    return gamma, tp, tq
