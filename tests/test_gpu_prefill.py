"""GPU parity of the dense prompt path (matrix-core GEMMs + causal flash attention) against the oracle."""
import numpy as np
import pytest
import torch

import synth
from oracle import transformer
from tests.util import bf16_pair, gpu_available, oracle_model

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]

LOGIT_TOL = 2e-2      # max |GPU - oracle| logit error, relative to the row's logit range


def _amd():
    import paper_2408_11850_amd as amd
    amd.load_library()
    return amd


@pytest.mark.parametrize("M,N,K", [(1, 48, 96), (300, 512, 256), (257, 272, 64), (1000, 1024, 2048),
                                   (4095, 256, 128), (130, 4112, 32)])
def test_dense_projection_matches_definition(M, N, K):
    """Store and residual-add epilogues: ragged token tiles, partial panel groups, one to many K steps."""
    amd = _amd()
    print(f"dense gemm M={M} N={N} K={K}", flush=True)
    w = synth.normal_tensor((N, K), 0.05, 3, N * 7 + K, torch.bfloat16)
    x = synth.normal_tensor((M, K), 1.0, 4, M, torch.bfloat16)
    ref = x.to(torch.float64) @ w.to(torch.float64).T
    wp = amd.binding.pack_matrices([w.cuda()])
    y = amd.dense_gemm(x.cuda(), wp, N)
    scale = ref.abs().max().item()
    tol = 2e-5 * scale * max(1.0, (K / 256) ** 0.5)
    assert (y.cpu().to(torch.float64) - ref).abs().max().item() <= tol
    h0 = synth.normal_tensor((M, N), 1.0, 5, 1, torch.float32)
    h = h0.clone().cuda()
    amd.dense_gemm(x.cuda(), wp, N, epilogue=amd.EPI_RESID, y=h)
    assert (h.cpu().to(torch.float64) - (h0.to(torch.float64) + ref)).abs().max().item() <= tol + 1e-6


@pytest.mark.parametrize("M,F,K", [(70, 48, 64), (513, 1376, 512)])
def test_dense_gate_up_epilogue_matches_definition(M, F, K):
    amd = _amd()
    print(f"dense swiglu M={M} F={F} K={K}", flush=True)
    wg = synth.normal_tensor((F, K), 0.08, 3, 1, torch.bfloat16)
    wu = synth.normal_tensor((F, K), 0.08, 3, 2, torch.bfloat16)
    x = synth.normal_tensor((M, K), 1.0, 4, M, torch.bfloat16)
    g = x.to(torch.float64) @ wg.to(torch.float64).T
    u = x.to(torch.float64) @ wu.to(torch.float64).T
    ref = g / (1.0 + torch.exp(-g)) * u
    wp = amd.binding.pack_matrices([wg.cuda(), wu.cuda()], interleave=True)
    z = amd.dense_gemm(x.cuda(), wp, 2 * F, epilogue=amd.EPI_SWIGLU)
    # the result is rounded to bf16: 2^-8 relative, plus the fp32 accumulation error
    err = (z.cpu().to(torch.float64) - ref).abs()
    assert (err <= 2.0 ** -8 * ref.abs() + 1e-4 * ref.abs().max()).all()


def test_dense_projection_rejects_bad_shapes():
    amd = _amd()
    x = torch.zeros((4, 48), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(amd.SpecError):
        amd.dense_gemm(x, w, 64)               # K not a multiple of 32
    with pytest.raises(amd.SpecError):
        amd.dense_gemm(x[:, :32].contiguous(), w, 40)   # N not a multiple of 16


def _custom(shape, draft_layers, n_prompt):
    c = synth.config("tiny")
    c.name = "custom"
    c.target = shape
    c.draft = synth._truncate(shape, draft_layers)
    c.draft_from_target_layers = draft_layers
    c.n_prompt, c.n_generate = n_prompt, 64
    return c


def _setup(cfg, gamma_max=8):
    from paper_2408_11850_amd import harness
    amd = _amd()
    w = bf16_pair(cfg)
    target, draft = harness.build_pair(cfg, weights=w)
    ctx = harness.make_context(cfg, target, draft, gamma_max, temperature=1.0)
    return amd, ctx, oracle_model(w[0], cfg.target), oracle_model(w[1], cfg.draft)


def _rel_err(got, ref):
    rng = ref.max(axis=-1) - ref.min(axis=-1)
    return float((np.abs(got - ref).max(axis=-1) / rng).max())


CASES = {
    "gqa64": (synth.ModelShape(2, 512, 8, 2, 1376, 2048), 333),        # head_dim 64, group 4, ragged row tiles
    "gqa128": (synth.ModelShape(2, 1024, 8, 2, 2752, 4096), 300),      # head_dim 128, group 4
    "mha128": (synth.ModelShape(2, 512, 4, 4, 1024, 1024), 523),       # group 1: 523 rows per head, 3 row blocks
    "gqa8": (synth.ModelShape(1, 1024, 8, 1, 1024, 1024), 97),         # group 8 as in the 70B shape
}


@pytest.mark.parametrize("case", list(CASES))
def test_dense_prefill_matches_oracle(case):
    """After a dense prefill the caches must serve the decode kernels: logits of later verify passes agree
    with the oracle, for the target and (through a draft step's distribution) the draft."""
    shape, n_prompt = CASES[case]
    cfg = _custom(shape, 1, n_prompt)
    print(f"dense prefill parity case={case}", flush=True)
    amd, ctx, tm, dm = _setup(cfg)
    ctx.set_option(amd.SPEC_OPT_PREFILL, 1)
    prompt = synth.prompt_tokens(n_prompt, shape.vocab, 7).tolist()
    extra = synth.prompt_tokens(24, shape.vocab, 8).tolist()
    ctx.prefill(prompt)
    ocm = transformer.CachedModel(tm, n_prompt + 64)
    ocm.feed(prompt[:-1])
    assert ctx.kv_len(amd.SPEC_TARGET) == n_prompt - 1 == ocm.len
    assert ctx.kv_len(amd.SPEC_DRAFT) == n_prompt - 1
    pos, worst = 0, 0.0
    for m in (1, 7, 16):
        toks = ([prompt[-1]] + extra)[pos:pos + m]
        pos += m
        got = ctx.verify(toks, want_logits=True)
        worst = max(worst, _rel_err(got, ocm.feed(toks)))
    print(f"  max logit error / range = {worst:.2e}", flush=True)
    assert worst <= LOGIT_TOL
    ctx.close()


def test_dense_and_chunked_prefill_fill_the_same_cache():
    """Both prompt paths, then the same verify pass: logits agree far inside the oracle tolerance."""
    shape, n_prompt = CASES["gqa64"]
    cfg = _custom(shape, 1, n_prompt)
    amd, ctx, _, _ = _setup(cfg)
    prompt = synth.prompt_tokens(n_prompt, shape.vocab, 7).tolist()
    toks = [prompt[-1]] + synth.prompt_tokens(8, shape.vocab, 8).tolist()
    out = []
    for mode in (0, 1):
        ctx.set_option(amd.SPEC_OPT_PREFILL, mode)
        ctx.prefill(prompt)
        out.append(ctx.verify(toks, want_logits=True))
    err = _rel_err(out[1], out[0])
    print(f"  dense vs chunked: {err:.2e}", flush=True)
    assert err <= 1e-2
    ctx.close()


def test_prompt_longer_than_one_dense_block():
    """4200 tokens = one block of 4096 and a ragged second block that attends to the first through the pages."""
    shape = synth.ModelShape(2, 256, 4, 2, 512, 1024)
    n_prompt = 4200
    cfg = _custom(shape, 1, n_prompt)
    amd, ctx, tm, _ = _setup(cfg, gamma_max=4)
    ctx.set_option(amd.SPEC_OPT_PREFILL, 1)
    prompt = synth.prompt_tokens(n_prompt, shape.vocab, 11).tolist()
    ctx.prefill(prompt, which_mask=1)
    ocm = transformer.CachedModel(tm, n_prompt + 16)
    ocm.feed(prompt[:-1])
    toks = [prompt[-1], 5, 17, 900]
    err = _rel_err(ctx.verify(toks, want_logits=True), ocm.feed(toks))
    print(f"  max logit error / range = {err:.2e}", flush=True)
    assert err <= LOGIT_TOL
    ctx.close()


def test_dense_prefill_refuses_shapes_it_cannot_tile():
    shape = synth.ModelShape(1, 256, 4, 4, 688, 1024)    # d_ffn not a multiple of 32
    cfg = _custom(shape, 1, 100)
    amd, ctx, _, _ = _setup(cfg)
    prompt = synth.prompt_tokens(100, shape.vocab, 7).tolist()
    ctx.set_option(amd.SPEC_OPT_PREFILL, 1)
    with pytest.raises(amd.SpecError):
        ctx.prefill(prompt)
    ctx.set_option(amd.SPEC_OPT_PREFILL, -1)             # automatic: falls back to verify-sized forwards
    ctx.prefill(prompt)
    assert ctx.kv_len(amd.SPEC_TARGET) == 99
    ctx.close()
