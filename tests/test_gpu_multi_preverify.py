"""GPU parity of PEARL with pre-verify over guessed continuations (closing remark of Section 4.3) against the
oracle's reading of it (run with -m gpu).

As for the other loops: the oracle's loop runs on the library's own logits (LockstepModel), every forward is compared
with the fp32 oracle forward and every decision must be the oracle's unless it sits within EXACT_MARGIN of flipping.
"""
import numpy as np
import pytest

import synth
from oracle import loops, multi_preverify
from tests.test_gpu_loops import _pair, lockstep_run
from tests.util import EXACT_MARGIN, NpUniforms, gpu_available

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]


def guess_steps(amd, ctx, gamma, n_generate, uni, k, guess_for=None, force=None):
    """The loop of spec_generate(algo 5) driven call by call.  guess_for(committed_len, drafts) -> the caller's guesses
    for a pre-verify step (drafts = the step's x_1..x_gamma, known because the drafting is done first here); None =
    the library's own pool.  Returns per step: mode, tokens, n_accepted, rows of the target forward."""
    steps, mode, produced, t = [], amd.SPEC_MODE_PRE, 0, 0
    while produced < n_generate:
        if mode == amd.SPEC_MODE_PRE:
            xs = [ctx.draft_step(uni.draft[t, i], want_token=True) for i in range(gamma)]
            if guess_for is None:
                fed, _ = ctx.verify_guess(None, min(k, gamma - 1))
            else:
                fed, _ = ctx.verify_guess(guess_for(ctx.committed_len(), xs)[:min(k, gamma - 1)])
            kind, rows = amd.SPEC_ACCEPT_PRE_GUESS, fed + 1
        else:
            rows = ctx.pending_rows()
            assert 1 <= rows <= gamma
            ctx.verify(n_tokens=rows)
            for i in range(gamma):
                ctx.draft_step(uni.draft[t, i])
            kind = amd.SPEC_ACCEPT_POST
        fm = -1
        if force is not None:
            fm = sum(1 << i for i in range(rows) if force(t, i))
        res = ctx.accept(kind, uni.accept[t, :gamma + 1], uni.resample[t], fm)
        if res["keep_len"] >= 0:
            for w in (amd.SPEC_TARGET, amd.SPEC_DRAFT):
                if ctx.kv_len(w) > res["keep_len"]:
                    ctx.rollback_kv(w, res["keep_len"])
        assert ctx.kv_len(amd.SPEC_TARGET) == ctx.committed_len() - 1     # the target cache lacks exactly the frontier
        steps.append({"mode": mode, "tokens": res["tokens"], "n_accepted": res["n_accepted"], "rows": rows})
        produced += len(res["tokens"])
        mode = res["next_mode"]
        t += 1
    return steps


@pytest.mark.parametrize("gamma,k,temperature", [(4, 3, 0.0), (4, 3, 1.0), (2, 1, 1.0), (6, 2, 1.0)])
def test_pool_guesses_take_the_oracles_decisions(gamma, k, temperature):
    """The library's pool (the committed text as an n-gram cache) against the oracle's, through whole runs."""
    cfg = synth.config("tiny")
    amd, harness, target, draft, tm, dm = _pair(cfg)
    seen = []

    def gpu(amd_, ctx, algo, g, n, uni):
        st = guess_steps(amd_, ctx, g, n, uni, k)
        seen.extend(st)
        return st

    oracle = lambda lt, ld, prompt, n, g, uni, **kw: multi_preverify.pearl_multi_preverify(lt, ld, prompt, n, g, k, uni, **kw)
    agreed, splits, wt, wd, modes = lockstep_run(amd, harness, cfg, target, draft, tm, dm, amd.ALGO_PEARL_GUESS, gamma,
                                                 temperature, n_total=96, seed=cfg.seed_uniform + 17,
                                                 oracle_loop=oracle, gpu_steps=gpu)
    multi = sum(1 for s in seen if s["mode"] == amd.SPEC_MODE_PRE and s["n_accepted"] > 1)
    print(f"gamma={gamma} k={k} T={temperature}: {agreed} steps identical, {splits} splits; {multi} pre-verify steps "
          f"accepted more than one draft; worst logit error target {wt:.2e} draft {wd:.2e}", flush=True)
    assert splits <= 2 and agreed >= 10 * max(1, splits)
    if temperature > 0.0:     # (greedy: the tiny pair's one-layer draft model is rejected at x_1 every time)
        assert loops.PRE in modes and loops.POST in modes


def scripted_hooks(k, vocab, force=None):
    """Guesses from the caller: the step's own drafts with one of every three corrupted, so that rows get used up to
    every depth.  force(t, i): scripted accept / reject decisions for both loops (None = the pair's own).  The library's loop of a segment runs first and records what it fed (by committed length); the
    oracle's loop gets the same guesses wherever it is in the same state.  Returns (gpu_steps hook, oracle_loop hook,
    list of the library's steps)."""
    rec, seen = {}, []

    def guess_for(committed_len, xs):
        g = list(xs[:k])
        j = committed_len % 3           # which guess (if any) is wrong
        if j < len(g):
            g[j] = (g[j] + 1) % vocab
        rec[committed_len] = g
        return g

    def gpu(amd_, ctx, algo, g, n, uni):
        st = guess_steps(amd_, ctx, g, n, uni, k, guess_for=guess_for, force=force)
        seen.extend(st)
        return st

    def oracle(lt, ld, prompt, n, g, uni, **kw):
        return multi_preverify.pearl_multi_preverify(lt, ld, prompt, n, g, k, uni,
                                                     guess=lambda committed, kk: rec.get(len(committed), [])[:kk],
                                                     force=force, **kw)

    return gpu, oracle, seen


@pytest.mark.parametrize("gamma,k", [(4, 3), (5, 2)])
def test_scripted_guesses_take_the_oracles_decisions(gamma, k):
    """Rows used up to every depth - all gamma drafts verified in the pre-verify step included - and the post-verify
    forwards that follow take 1..gamma rows.  The tiny pair's one-layer draft model is seldom accepted twice in a row,
    so four of five accept / reject decisions are scripted to accept (the draws of drafts and of corrected tokens stay
    the pair's own); the full-width test below runs on the pair's own decisions."""
    cfg = synth.config("tiny")
    amd, harness, target, draft, tm, dm = _pair(cfg)
    force = lambda t, i: (7 * t + 3 * i) % 5 != 0
    gpu, oracle, seen = scripted_hooks(k, cfg.target.vocab, force=force)
    agreed, splits, wt, wd, modes = lockstep_run(amd, harness, cfg, target, draft, tm, dm, amd.ALGO_PEARL_GUESS, gamma,
                                                 1.0, n_total=96, seed=cfg.seed_uniform + 29, oracle_loop=oracle,
                                                 gpu_steps=gpu, gpu_first=True)
    rows_post = {s["rows"] for s in seen if s["mode"] == amd.SPEC_MODE_POST}
    acc_pre = {s["n_accepted"] for s in seen if s["mode"] == amd.SPEC_MODE_PRE}
    print(f"gamma={gamma} k={k}: {agreed} steps identical, {splits} splits; post-verify rows seen {sorted(rows_post)}, "
          f"pre-verify acceptances seen {sorted(acc_pre)}", flush=True)
    assert splits <= 2 and agreed >= 10 * max(1, splits)
    assert len(rows_post) >= 2 and max(acc_pre) >= 2


def test_full_width_pair_with_scripted_guesses_decodes_like_the_oracle():
    """The same on the 70B widths and the real vocabulary (depth cut to 2 layers so that the fp32 oracle can hold the
    model; the target's first layer as the draft model, which gives acceptance rates of trained pairs)."""
    import paper_2408_11850_amd as amd
    from paper_2408_11850_amd import harness
    from tests.test_gpu_fullsize import _cpu_weights
    from tests.util import oracle_model
    cfg = synth.config("70b_7b", depth=2, draft_depth=1)
    cfg.draft_from_target_layers = 1
    cfg.draft = synth._truncate(cfg.target, 1)
    tw, dw = synth.make_pair(cfg, device="cuda")
    target, draft = harness.build_pair(cfg, weights=(tw, dw))
    tm = oracle_model(_cpu_weights(tw), cfg.target)
    dm = oracle_model(_cpu_weights(dw), cfg.draft)
    del tw, dw
    cfg.n_prompt, cfg.n_generate = 100, 64
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, 9).tolist()
    gamma, k = 4, 3
    gpu, oracle, seen = scripted_hooks(k, cfg.target.vocab)
    agreed, splits, wt, wd, modes = lockstep_run(amd, harness, cfg, target, draft, tm, dm, amd.ALGO_PEARL_GUESS, gamma,
                                                 1.0, n_total=40, seed=37, prompt=prompt, first_segment=40,
                                                 oracle_loop=oracle, gpu_steps=gpu, gpu_first=True)
    acc_pre = sorted({s["n_accepted"] for s in seen if s["mode"] == amd.SPEC_MODE_PRE})
    print(f"70b widths: {agreed} steps identical, {splits} splits within {EXACT_MARGIN} of a flip; worst logit error "
          f"target {wt:.2e} draft {wd:.2e}; pre-verify acceptances seen {acc_pre}", flush=True)
    assert splits <= 2 and agreed >= 8 * max(1, splits)
    assert max(acc_pre) >= 2


def test_generate_equals_the_call_by_call_loop_and_k0_is_pearl():
    cfg = synth.config("tiny")
    amd, harness, target, draft, tm, dm = _pair(cfg)
    gamma, n_gen = 4, 64
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, 21).tolist()
    uni = NpUniforms(synth.make_uniforms(n_gen + 1, gamma, 9))
    ctx = harness.make_context(cfg, target, draft, gamma)
    assert ctx.get_option(amd.SPEC_OPT_GUESS_TOKENS) == -1
    for k in (-1, 2):
        ctx.set_option(amd.SPEC_OPT_GUESS_TOKENS, k)
        ctx.prefill(prompt)
        out, st = ctx.generate(amd.ALGO_PEARL_GUESS, gamma, n_gen, uni)
        assert st["target_forwards"] == st["steps"] and st["draft_forwards"] == gamma * st["steps"]
        ctx.prefill(prompt)
        steps = guess_steps(amd, ctx, gamma, n_gen, uni, gamma - 1 if k < 0 else k)
        assert [t for s in steps for t in s["tokens"]][:n_gen] == out
        assert len(steps) == st["steps"]
    # no guesses: exactly Algorithm 2
    ctx.set_option(amd.SPEC_OPT_GUESS_TOKENS, 0)
    ctx.prefill(prompt)
    out0, st0 = ctx.generate(amd.ALGO_PEARL_GUESS, gamma, n_gen, uni)
    ctx.prefill(prompt)
    out2, st2 = ctx.generate(amd.ALGO_PEARL, gamma, n_gen, uni)
    assert out0 == out2
    for key in ("steps", "accepted", "tested", "post_steps", "target_forwards", "draft_forwards"):
        assert st0[key] == st2[key], key
    ctx.close()


def test_greedy_output_is_the_autoregressive_one():
    """Lossless at temperature 0: the text is the target's greedy text whatever the pool guesses.  (48 tokens: further
    on this text meets a near-tie of the top two logits, which forwards over different numbers of rows - different
    orders of the same additions - may break differently.)"""
    cfg = synth.config("tiny")
    amd, harness, target, draft, tm, dm = _pair(cfg)
    gamma, n_gen = 4, 48
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, cfg.seed_prompt).tolist()
    uni = NpUniforms(synth.make_uniforms(n_gen + 1, gamma, 3))
    ctx = harness.make_context(cfg, target, draft, gamma, temperature=0.0, extra_seq=n_gen)
    outs, stats = {}, {}
    for algo in (amd.ALGO_AR, amd.ALGO_PEARL, amd.ALGO_PEARL_GUESS):
        ctx.prefill(prompt)
        outs[algo], stats[algo] = ctx.generate(algo, gamma, n_gen, uni)
    assert outs[amd.ALGO_AR] == outs[amd.ALGO_PEARL] == outs[amd.ALGO_PEARL_GUESS]
    assert stats[amd.ALGO_PEARL_GUESS]["steps"] <= stats[amd.ALGO_PEARL]["steps"]
    ctx.close()


def test_state_errors_of_the_guessed_pre_verify():
    cfg = synth.config("tiny")
    amd, harness, target, draft, tm, dm = _pair(cfg)
    gamma = 4
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, 5).tolist()
    uni = NpUniforms(synth.make_uniforms(8, gamma, 2))
    ctx = harness.make_context(cfg, target, draft, gamma)
    ctx.prefill(prompt)
    with pytest.raises(amd.SpecError):                      # more guesses than a window can use
        ctx.verify_guess([1] * gamma)
    with pytest.raises(amd.SpecError):                      # a guess outside the vocabulary
        ctx.verify_guess([cfg.target.vocab])
    for i in range(gamma):
        ctx.draft_step(uni.draft[0, i])
    ctx.verify(n_tokens=1)
    with pytest.raises(amd.SpecError):                      # a plain target forward is no guessed pre-verify
        ctx.accept(amd.SPEC_ACCEPT_PRE_GUESS, uni.accept[0], uni.resample[0])
    # the failed call changed nothing: the step can go on as an ordinary pre-verify
    res = ctx.accept(amd.SPEC_ACCEPT_PRE, uni.accept[0], uni.resample[0], force_mask=1)
    assert res["n_accepted"] == 1 and res["next_mode"] == amd.SPEC_MODE_POST
    with pytest.raises(amd.SpecError):                      # x_1 is committed: no pre-verify of any kind now
        ctx.verify_guess([1])
    # drafts of the guessed loop that another loop cannot take over
    ctx.prefill(prompt)
    force = np.ones((8, gamma + 1), dtype=np.uint8)
    ctx.set_option(amd.SPEC_OPT_GUESS_TOKENS, 0)
    ctx.generate(amd.ALGO_PEARL_GUESS, gamma, 8, uni, force_bits=force, max_steps=1)
    assert ctx.pending_rows() == gamma
    with pytest.raises(amd.SpecError):
        ctx.generate(amd.ALGO_SD, gamma, 4, uni)
    ctx.close()
