"""Builds synthetic model pairs on the GPU and drives the library's loops (used by bench.py and the tests)."""
from __future__ import annotations

import time
from typing import Optional, Tuple

import torch

import synth
from . import ALGO_AR, ALGO_PEARL, ALGO_SD, SPEC_DRAFT, SPEC_TARGET
from .binding import PackedModel, SpecContext, pack_from_dict, pack_model


def _library_generated_model(shape: synth.ModelShape, seed: int, device: str) -> PackedModel:
    """Same shapes and distributions from PyTorch's own generator (other values): for runs under the profiler's
    counter collection, which crashes on the run-time-compiled kernel behind the counter-based generator's inverse
    normal CDF.  Never used where values are compared with the oracle."""
    mats = synth.layer_matrix_shapes(shape)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)

    def get(layer: Optional[int], name: str) -> torch.Tensor:
        if name in ("final_norm", "attn_norm", "ffn_norm"):
            g = torch.empty(shape.d_model, dtype=torch.float32, device=device).normal_(0.0, synth.GAIN_STD, generator=gen)
            return (1.0 + g).to(torch.bfloat16)
        shp = (shape.vocab, shape.d_model) if layer is None else mats[name]
        return torch.empty(shp, dtype=torch.float32, device=device).normal_(0.0, 0.02, generator=gen).to(torch.bfloat16)

    return pack_model(shape, get, device)


def _generated_model(shape: synth.ModelShape, seed: int, device: str) -> PackedModel:
    """Generate each tensor on the device with the counter-based generator, pack it, drop the source."""
    mats = synth.layer_matrix_shapes(shape)

    def get(layer: Optional[int], name: str) -> torch.Tensor:
        if name == "final_norm":
            return synth.gain_tensor(shape.d_model, seed, synth._GLOBAL[name], torch.bfloat16, device)
        if name in ("attn_norm", "ffn_norm"):
            return synth.gain_tensor(shape.d_model, seed, 16 * layer + synth._SLOT[name], torch.bfloat16, device)
        if layer is None:
            return synth.normal_tensor((shape.vocab, shape.d_model), 0.02, seed, synth._GLOBAL[name], torch.bfloat16,
                                       device)
        return synth.normal_tensor(mats[name], 0.02, seed, 16 * layer + synth._SLOT[name], torch.bfloat16, device)

    return pack_model(shape, get, device)


def build_pair(cfg: synth.PairConfig, device: str = "cuda", weights: Optional[Tuple[dict, dict]] = None,
               library_generator: bool = False):
    """(target PackedModel, draft PackedModel) for a workload.  With `weights` (generator dicts, e.g. the
    ones also handed to a reference implementation) those exact values are packed instead.  library_generator:
    values from PyTorch's generator instead of the counter-based one (profiler counter runs only)."""
    if weights is not None:
        tw, dw = weights
        target = pack_from_dict(cfg.target, tw, device)
        if cfg.draft_from_target_layers:
            draft = target.prefix(cfg.draft_from_target_layers, cfg.draft)
        else:
            draft = pack_from_dict(cfg.draft, dw, device)
        return target, draft
    make = _library_generated_model if library_generator else _generated_model
    target = make(cfg.target, cfg.seed_target, device)
    if cfg.draft_from_target_layers:
        draft = target.prefix(cfg.draft_from_target_layers, cfg.draft)
    else:
        draft = make(cfg.draft, cfg.seed_draft, device)
    return target, draft


_hip = None


def _hip_lib():
    import ctypes as C
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
    return _hip


def masked_stream(first_cu: int, n_cus: int, total_cus: int = 256):
    """(torch stream, raw handle) of a HIP stream (default priority) whose kernels may only run on CUs
    first_cu .. first_cu + n_cus - 1 (hipExtStreamCreateWithCUMask).  A stream made this way owns a hardware
    queue; plain streams are dealt round-robin to a few shared ones, and two streams that land on the same queue
    take turns instead of overlapping (measured: a PEARL step of 59.8 instead of 43.5 ms).  With a mask of all CUs
    this is simply "a stream with a queue of its own"; with a partial mask it divides the GPU between the two
    models (the paper's resource-competition setting)."""
    import ctypes as C
    words = (total_cus + 31) // 32
    mask = (C.c_uint32 * words)()
    for cu in range(first_cu, first_cu + n_cus):
        mask[cu // 32] |= 1 << (cu % 32)
    stream = C.c_void_p()
    rc = _hip_lib().hipExtStreamCreateWithCUMask(C.byref(stream), C.c_uint32(words), mask)
    if rc != 0 or not stream.value:
        raise RuntimeError(f"hipExtStreamCreateWithCUMask failed with {rc}")
    return torch.cuda.ExternalStream(stream.value), stream.value


def make_context(cfg: synth.PairConfig, target: PackedModel, draft: PackedModel, gamma_max: int,
                 temperature: Optional[float] = None, serial: bool = False, extra_seq: int = 0,
                 target_cus: Optional[int] = 256) -> SpecContext:
    """serial: one stream for both models.  target_cus: 256 (default) = each model's stream owns a hardware
    queue and may use every compute unit; T < 256 = the target stream gets the first T compute units and the
    draft stream the rest; None = plain torch streams."""
    import ctypes as C
    max_seq = cfg.n_prompt + cfg.n_generate + 2 * gamma_max + 2 + extra_seq
    raw = []
    if serial or target_cus is None:
        st = torch.cuda.Stream()
        sd = st if serial else torch.cuda.Stream()
    else:
        t = 256 if target_cus >= 256 else target_cus
        st, h0 = masked_stream(0, t)
        sd, h1 = masked_stream(0, 256) if t == 256 else masked_stream(t, 256 - t)
        raw = [h0, h1]

    def destroy():
        for h in raw:
            _hip_lib().hipStreamDestroy(C.c_void_p(h))

    return SpecContext(target, draft, gamma_max, max_seq,
                       cfg.temperature if temperature is None else temperature, cfg.logit_scale, st, sd,
                       on_close=destroy if raw else None)


def calibrate_gamma(ctx: SpecContext, n_iter: int = 8, cap: int = 16, concurrent: bool = False) -> Tuple[int, float, float]:
    """Window size gamma = round(c), c = T(target forward) / T(draft forward) (paper Section 4.4.1): computed by the
    library (spec_calibrate_gamma); leaves the caches as it found them."""
    return ctx.calibrate_gamma(n_iter, cap, concurrent)
