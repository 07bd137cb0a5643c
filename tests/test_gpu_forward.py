"""GPU parity of the target / draft forward and of the KV cache against the oracle (run with -m gpu)."""
import numpy as np
import pytest
import torch

import synth
from oracle import transformer
from tests.util import NpUniforms, bf16_pair, gpu_available, oracle_model

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]

LOGIT_TOL = 2e-2      # max |GPU - oracle| logit error, relative to the row's logit range (bf16 path vs fp32)
DRAW_MARGIN_TOL = 5e-3  # a draw may differ from the oracle's only if u lies this close to a CDF edge


def _setup(cfg, gamma_max=8, temperature=1.0, extra_seq=0):
    import paper_2408_11850_amd as amd
    from paper_2408_11850_amd import harness
    w = bf16_pair(cfg)
    target, draft = harness.build_pair(cfg, weights=w)
    ctx = harness.make_context(cfg, target, draft, gamma_max, temperature=temperature, extra_seq=extra_seq)
    tm = oracle_model(w[0], cfg.target)
    dm = oracle_model(w[1], cfg.draft)
    return amd, ctx, tm, dm


def _rel_err(got, ref):
    rng = ref.max(axis=-1) - ref.min(axis=-1)
    return float((np.abs(got - ref).max(axis=-1) / rng).max())


CASES = {
    "tiny": lambda: synth.config("tiny"),
    "gqa64": lambda: _custom(synth.ModelShape(2, 512, 8, 2, 1376, 2048), 1),            # head_dim 64, group 4
    "gqa128": lambda: _custom(synth.ModelShape(2, 1024, 8, 2, 2752, 4096), 1),          # head_dim 128, group 4
    "mha128_ragged_ffn": lambda: _custom(synth.ModelShape(3, 512, 4, 4, 1392, 1008), 2),  # K not a multiple of 32
}


def _custom(shape, draft_layers):
    c = synth.config("tiny")
    c.name = "custom"
    c.target = shape
    c.draft = synth._truncate(shape, draft_layers)
    c.draft_from_target_layers = draft_layers
    c.n_prompt, c.n_generate = 200, 64
    return c


@pytest.mark.parametrize("case", list(CASES))
def test_verify_logits_match_oracle(case):
    cfg = CASES[case]()
    print(f"forward parity case={case}", flush=True)
    amd, ctx, tm, dm = _setup(cfg)
    n_prompt = 150 if case != "tiny" else 32
    prompt = synth.prompt_tokens(n_prompt, cfg.target.vocab, 7).tolist()
    extra = synth.prompt_tokens(40, cfg.target.vocab, 8).tolist()
    ctx.prefill(prompt)                      # chunks of 32 + a ragged tail; crosses page boundaries
    ocm = transformer.CachedModel(tm, 512)
    ocm.feed(prompt[:-1])
    assert ctx.kv_len(amd.SPEC_TARGET) == n_prompt - 1 == ocm.len
    pos = 0
    worst = 0.0
    for m in (1, 5, 17, 1, 9):               # pre-verify, post-verify, SD with gamma 16, ...
        toks = ([prompt[-1]] + extra)[pos:pos + m]
        pos += m
        got = ctx.verify(toks, want_logits=True)
        ref = ocm.feed(toks)
        worst = max(worst, _rel_err(got, ref))
    print(f"  max logit error / range = {worst:.2e}", flush=True)
    assert worst <= LOGIT_TOL
    assert ctx.kv_len(amd.SPEC_TARGET) == ocm.len
    ctx.close()


def test_multi_token_verify_equals_sequential_single_token_forwards_on_gpu():
    cfg = CASES["gqa128"]()
    amd, ctx, tm, dm = _setup(cfg)
    prompt = synth.prompt_tokens(100, cfg.target.vocab, 3).tolist()
    toks = synth.prompt_tokens(9, cfg.target.vocab, 4).tolist()
    ctx.prefill(prompt)
    base = ctx.kv_len(amd.SPEC_TARGET)
    multi = ctx.verify(toks, want_logits=True)
    ctx.rollback_kv(amd.SPEC_TARGET, base)
    seq = np.concatenate([ctx.verify([t], want_logits=True) for t in toks])
    # same weights, same bf16 rounding points; only the summation split differs
    assert _rel_err(multi, seq) < 5e-3
    ctx.close()


@pytest.mark.parametrize("case", list(CASES))
def test_single_token_forwards_with_fused_prologues_equal_the_general_chain(case):
    """Forwards over one token run seven kernels per layer (projections that form their own input) instead of ten.
    Same operations and the same order of every K-slice sum; only the sums of squares are grouped by wave instead of
    by 1024 columns.  Both chains against the oracle, and against each other far below the bf16 tolerance; the
    caches they leave are interchangeable (a multi-token forward behind either gives the same logits)."""
    cfg = CASES[case]()
    amd, ctx, tm, dm = _setup(cfg)
    prompt = synth.prompt_tokens(97, cfg.target.vocab, 7).tolist()
    toks = synth.prompt_tokens(12, cfg.target.vocab, 8).tolist()
    ocm = transformer.CachedModel(tm, 256)
    ocm.feed(prompt[:-1])
    ref = np.concatenate([ocm.feed([t]) for t in [prompt[-1]] + toks[:5]])
    ref_multi = ocm.feed(toks[5:])
    outs = {}
    for fused in (1, 0):
        ctx.set_option(amd.SPEC_OPT_FUSE_SINGLE, fused)
        assert ctx.get_option(amd.SPEC_OPT_FUSE_SINGLE) == fused
        ctx.prefill(prompt)
        single = np.concatenate([ctx.verify([t], want_logits=True) for t in [prompt[-1]] + toks[:5]])
        multi = ctx.verify(toks[5:], want_logits=True)
        assert _rel_err(single, ref) <= LOGIT_TOL and _rel_err(multi, ref_multi) <= LOGIT_TOL
        outs[fused] = (single, multi)
    e1, e2 = _rel_err(outs[1][0], outs[0][0]), _rel_err(outs[1][1], outs[0][1])
    print(f"  {case}: fused vs general single-token chain {e1:.2e}, multi-token forward behind them {e2:.2e}", flush=True)
    assert e1 < 2e-3 and e2 < 2e-3
    ctx.close()


def test_rollback_is_bit_exact_and_returns_pages():
    cfg = CASES["gqa64"]()
    amd, ctx, tm, dm = _setup(cfg, extra_seq=256)
    prompt = synth.prompt_tokens(120, cfg.target.vocab, 5).tolist()
    a = synth.prompt_tokens(6, cfg.target.vocab, 6).tolist()
    junk = synth.prompt_tokens(30, cfg.target.vocab, 9).tolist()
    ctx.prefill(prompt)
    base = ctx.kv_len(amd.SPEC_TARGET)
    free0 = ctx.free_pages(amd.SPEC_TARGET)
    first = ctx.verify(a, want_logits=True)
    ctx.verify(junk)                                    # speculate past the point, over a page boundary
    ctx.verify(junk)
    assert ctx.free_pages(amd.SPEC_TARGET) < free0
    ctx.rollback_kv(amd.SPEC_TARGET, base)
    assert ctx.free_pages(amd.SPEC_TARGET) == free0 and ctx.kv_len(amd.SPEC_TARGET) == base
    again = ctx.verify(a, want_logits=True)
    assert np.array_equal(first, again)                 # bit-exact
    with pytest.raises(amd.SpecError) as e:
        ctx.rollback_kv(amd.SPEC_TARGET, base + len(a) + 1)
    assert e.value.code == amd.SPEC_E_INVAL
    ctx.close()


def test_draft_step_distribution_matches_oracle():
    from oracle import sampling
    cfg = CASES["tiny"]()
    amd, ctx, tm, dm = _setup(cfg)
    prompt = synth.prompt_tokens(32, cfg.target.vocab, 7).tolist()
    ctx.prefill(prompt)
    ocm = transformer.CachedModel(dm, 128)
    ocm.feed(prompt[:-1])
    us = synth.uniform_array(6, 5, 5).tolist()
    inp = prompt[-1]
    agree = 0
    for i in range(6):
        q = sampling.probs(ocm.feed([inp])[0], cfg.temperature, cfg.logit_scale)
        x_ref = sampling.sample(q, us[i])
        x = ctx.draft_step(us[i], want_token=True)
        margin = sampling.sample_margin(q, us[i])
        print(f"  draft step {i}: gpu {x} oracle {x_ref} margin {margin:.4f}", flush=True)
        if x != x_ref:
            assert margin < DRAW_MARGIN_TOL     # the chains may split only on a close draw
            break
        agree += 1
        inp = x_ref
    assert agree >= 1
    ctx.close()


def test_error_paths_leave_state_intact():
    cfg = CASES["tiny"]()
    amd, ctx, tm, dm = _setup(cfg, gamma_max=4)
    with pytest.raises(amd.SpecError) as e:
        ctx.verify([1])                                 # no prefill yet
    assert e.value.code == amd.SPEC_E_STATE
    ctx.prefill(synth.prompt_tokens(16, cfg.target.vocab, 1).tolist())
    with pytest.raises(amd.SpecError) as e:
        ctx.verify([cfg.target.vocab])                  # token outside the vocabulary
    assert e.value.code == amd.SPEC_E_INVAL
    with pytest.raises(amd.SpecError) as e:
        ctx.verify(list(range(33)))
    assert e.value.code == amd.SPEC_E_INVAL
    n = ctx.kv_len(amd.SPEC_TARGET)
    # fill the cache until pages run out: the failing call must not change the length
    with pytest.raises(amd.SpecError) as e:
        for _ in range(64):
            ctx.verify(list(range(32)))
    assert e.value.code == amd.SPEC_E_NOMEM
    full = ctx.kv_len(amd.SPEC_TARGET)
    assert full > n and full % 32 == n % 32
    ctx.rollback_kv(amd.SPEC_TARGET, n)
    ctx.verify([3, 4, 5])
    assert ctx.kv_len(amd.SPEC_TARGET) == n + 3
    for _ in range(8):
        ctx.draft_step(0.5)
    with pytest.raises(amd.SpecError) as e:
        ctx.draft_step(0.5)                             # more than 2*gamma_max unverified drafts
    assert e.value.code == amd.SPEC_E_STATE
    ctx.close()


@pytest.mark.parametrize("prefill_mode", [0, 1], ids=["chunked", "dense"])
def test_prefill_that_fails_half_way_leaves_no_usable_looking_context(prefill_mode):
    """A prompt pass that gives up after some of its forwards (forced from the host, as if the KV pages had run out)
    has already reset the caches: every decoding call must then refuse with SPEC_E_STATE until a prefill succeeds.
    Errors found before anything is touched leave the context usable."""
    cfg = CASES["gqa64"]()
    amd, ctx, tm, dm = _setup(cfg, gamma_max=4)
    prompt = synth.prompt_tokens(150, cfg.target.vocab, 1).tolist()
    ctx.set_option(amd.SPEC_OPT_PREFILL, prefill_mode)
    ctx.prefill(prompt)
    ref = ctx.verify([prompt[-1], 5, 9], want_logits=True)
    ctx.rewind(len(prompt))
    # refused before anything is touched: the context stays as it was
    with pytest.raises(amd.SpecError) as e:
        ctx.prefill(list(range(1000)) * 3)                              # cannot fit max_seq
    assert e.value.code == amd.SPEC_E_NOMEM
    with pytest.raises(amd.SpecError) as e:
        ctx.prefill(prompt[:10] + [cfg.target.vocab])                   # token outside the vocabulary
    assert e.value.code == amd.SPEC_E_INVAL
    assert np.array_equal(ctx.verify([prompt[-1], 5, 9], want_logits=True), ref)
    ctx.rewind(len(prompt))
    # gives up half way
    ctx.set_option(amd.SPEC_OPT_TEST_FAIL_PREFILL, 1 if prefill_mode else 2)
    with pytest.raises(amd.SpecError) as e:
        ctx.prefill(prompt)
    assert e.value.code == amd.SPEC_E_NOMEM
    for call in (lambda: ctx.verify([1]), lambda: ctx.draft_step(0.5), lambda: ctx.rewind(1),
                 lambda: ctx.calibrate_gamma(2, 4),
                 lambda: ctx.generate(amd.ALGO_AR, 1, 2, NpUniforms(synth.make_uniforms(4, 1, 3)))):
        with pytest.raises(amd.SpecError) as e:
            call()
        assert e.value.code == amd.SPEC_E_STATE
    assert ctx.get_option(amd.SPEC_OPT_TEST_FAIL_PREFILL) == 0          # one-shot
    ctx.prefill(prompt)
    assert np.array_equal(ctx.verify([prompt[-1], 5, 9], want_logits=True), ref)
    ctx.close()


def test_graph_replays_equal_kernel_by_kernel_launches():
    """Captured forwards (HIP graphs) are replayed several times, with eager forwards, rollbacks and
    synchronisations in between; every replay must equal the kernel-by-kernel result bit for bit."""
    import torch
    cfg = CASES["gqa128"]()
    amd, ctx, tm, dm = _setup(cfg, extra_seq=256)
    prompt = synth.prompt_tokens(140, cfg.target.vocab, 21).tolist()
    toks = synth.prompt_tokens(64, cfg.target.vocab, 22).tolist()
    ctx.prefill(prompt)
    base = ctx.kv_len(amd.SPEC_TARGET)

    def run(graphs, rounds):
        ctx.set_option(amd.SPEC_OPT_GRAPHS, graphs)
        out = []
        for r in range(rounds):
            ctx.rollback_kv(amd.SPEC_TARGET, base)
            out.append(ctx.verify(toks[0:5], want_logits=True))          # M = 5
            out.append(ctx.verify(toks[5:6], want_logits=True))          # M = 1
            out.append(ctx.verify(toks[6:11], want_logits=True))         # M = 5 again, other position
            torch.cuda.synchronize()
        return out

    eager = run(0, 1)
    replays = run(1, 3)                      # first round captures, later rounds replay
    mixed = run(0, 1) + run(1, 1)            # eager work between replays
    for i, got in enumerate(replays + mixed):
        assert np.array_equal(got, eager[i % 3]), i
    # the draft chain through graphs equals the eager chain as well
    outs = []
    for graphs in (0, 1, 1):
        ctx.set_option(amd.SPEC_OPT_GRAPHS, graphs)
        ctx.rewind(len(prompt))
        outs.append([ctx.draft_step(u, want_token=True) for u in (0.11, 0.52, 0.93, 0.34)])
        ctx.drop_drafts()
    assert outs[0] == outs[1] == outs[2]
    ctx.close()


@pytest.mark.parametrize("case", ["tiny", "gqa64"])
def test_verify_at_page_and_chunk_boundaries(case):
    """Context lengths on both sides of the 32-position attention chunks and the 64-token pages, new-token blocks
    of 1, 7, 17 and 32 rows that start before a boundary and end behind it: the causal mask inside the block, the
    page-table walk and the K / V append in operand order must hold at every offset."""
    cfg = CASES[case]()
    amd, ctx, tm, dm = _setup(cfg, gamma_max=16, extra_seq=512)
    long_prompt = synth.prompt_tokens(200, cfg.target.vocab, 41).tolist()
    extra = synth.prompt_tokens(64, cfg.target.vocab, 42).tolist()
    worst = 0.0
    for n_prompt in (1, 2, 31, 32, 33, 34, 63, 64, 65, 66, 96, 127, 128, 129, 193):
        prompt = long_prompt[:n_prompt]
        ctx.prefill(prompt)
        ocm = transformer.CachedModel(tm, 512)
        ocm.feed(prompt[:-1])
        assert ctx.kv_len(amd.SPEC_TARGET) == n_prompt - 1
        pos = 0
        for m in (1, 7, 17, 32):
            toks = ([prompt[-1]] + extra)[pos:pos + m]
            pos += m
            got = ctx.verify(toks, want_logits=True)
            ref = ocm.feed(toks)
            err = _rel_err(got, ref)
            assert err <= LOGIT_TOL, (n_prompt, m, err)
            worst = max(worst, err)
    print(f"  boundary sweep {case}: max logit error / range = {worst:.2e}", flush=True)
    ctx.close()


def test_one_token_prompt_then_every_loop():
    """The shortest prompt: nothing in the caches, the prompt's only token is the frontier.  Greedy AR, SD and PEARL
    agree from there, and the first target row equals the oracle's."""
    cfg = CASES["tiny"]()
    amd, ctx, tm, dm = _setup(cfg, gamma_max=4, temperature=0.0)
    prompt = [5]
    uni = NpUniforms(synth.make_uniforms(25, 4, 2))
    outs = []
    for algo in (amd.ALGO_AR, amd.ALGO_SD, amd.ALGO_PEARL):
        ctx.prefill(prompt)
        assert ctx.kv_len(amd.SPEC_TARGET) == 0 == ctx.kv_len(amd.SPEC_DRAFT)
        out, st = ctx.generate(algo, 4, 24, uni)
        outs.append(out)
    assert outs[0] == outs[1] == outs[2] and len(outs[0]) == 24
    ctx.prefill(prompt)
    got = ctx.verify(prompt, want_logits=True)
    ref = transformer.CachedModel(tm, 8).feed(prompt)
    assert _rel_err(got, ref) <= LOGIT_TOL
    assert int(np.argmax(ref[0])) == outs[0][0] or np.sort(ref[0])[-1] - np.sort(ref[0])[-2] < 2e-2 * np.ptp(ref[0])
    ctx.close()


@pytest.mark.parametrize("prefill_mode", [1, 0], ids=["dense_prefill", "chunked_prefill"])
def test_benchmark_context_length_matches_oracle(prefill_mode):
    """The context length the benchmark runs at (4096-token prompt: 64 pages, the largest K/V split counts, one
    full block of the matrix-core prompt pass or 128 verify-sized forwards) on a narrow GQA model with head_dim 128
    that the fp64 oracle can follow: rows of 1, 7 and 8 new tokens against the oracle."""
    cfg = CASES["gqa128"]()
    cfg.n_prompt, cfg.n_generate = 4096, 64
    amd, ctx, tm, dm = _setup(cfg, gamma_max=8)
    ctx.set_option(amd.SPEC_OPT_PREFILL, prefill_mode)
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, 51).tolist()
    extra = synth.prompt_tokens(16, cfg.target.vocab, 52).tolist()
    ctx.prefill(prompt)
    assert ctx.kv_len(amd.SPEC_TARGET) == 4095
    print("oracle prompt pass over 4095 tokens", flush=True)
    ocm = transformer.CachedModel(tm, 4096 + 32)
    for b in range(0, 4095, 512):                      # blocks keep the oracle's score matrices small
        ocm.feed(prompt[b:min(b + 512, 4095)])
    worst, pos = 0.0, 0
    for m in (1, 7, 8):
        toks = ([prompt[-1]] + extra)[pos:pos + m]
        pos += m
        got = ctx.verify(toks, want_logits=True)
        ref = ocm.feed(toks)
        worst = max(worst, _rel_err(got, ref))
        print(f"  M={m}: logit error / range so far {worst:.2e}", flush=True)
    assert worst <= LOGIT_TOL
    ctx.close()
