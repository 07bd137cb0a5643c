"""GPU parity of the two ablation loops (PEARL without pre-verify / without post-verify), run with -m gpu."""
import numpy as np
import pytest

import synth
from oracle import ablations, loops, transformer
from tests.test_gpu_loops import MARGIN_TOL, _pair
from tests.util import NpUniforms, gpu_available

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]


def _gpu_steps(amd, ctx, algo, gamma, n_generate, uni):
    """spec_generate's ablation loops driven call by call; returns the tokens committed by every step."""
    steps, mode, produced, t = [], amd.SPEC_MODE_PRE, 0, 0
    drafted, first_verified = 0, False          # mirror of the library's ring state (for algo 3)
    while produced < n_generate:
        if algo == amd.ALGO_PEARL_NO_PRE:
            if drafted == 0:
                for i in range(gamma):
                    ctx.draft_step(uni.draft[t, i])
                drafted = gamma
                steps.append({"tokens": []})
                t += 1
                continue
            n = gamma if first_verified else gamma + 1
            ctx.verify(n_tokens=n)
            for i in range(gamma):
                ctx.draft_step(uni.draft[t, i])
            res = ctx.accept(amd.SPEC_ACCEPT_POST, uni.accept[t, :gamma + 1], uni.resample[t])
            if res["keep_len"] >= 0:
                drafted, first_verified = 0, False
            else:
                drafted, first_verified = gamma, True
        elif mode == amd.SPEC_MODE_PRE:
            ctx.verify(n_tokens=1)
            for i in range(gamma):
                ctx.draft_step(uni.draft[t, i])
            res = ctx.accept(amd.SPEC_ACCEPT_PRE, uni.accept[t, :gamma + 1], uni.resample[t])
        else:
            ctx.verify(n_tokens=gamma)
            res = ctx.accept(amd.SPEC_ACCEPT_SD, uni.accept[t, :gamma + 1], uni.resample[t])
        if res["keep_len"] >= 0:
            for w in (amd.SPEC_TARGET, amd.SPEC_DRAFT):
                if ctx.kv_len(w) > res["keep_len"]:
                    ctx.rollback_kv(w, res["keep_len"])
        assert ctx.kv_len(amd.SPEC_TARGET) == ctx.committed_len() - 1
        steps.append({"tokens": res["tokens"]})
        produced += len(res["tokens"])
        mode = res["next_mode"]
        t += 1
    return steps


ORACLE = {3: ablations.pearl_without_pre_verify, 4: ablations.pearl_without_post_verify}


@pytest.mark.parametrize("algo", [3, 4])
def test_ablation_loops_follow_the_oracle_step_by_step(algo):
    cfg = synth.config("tiny")
    amd, harness, target, draft, tm, dm = _pair(cfg)
    gamma, seg_len, n_total = 4, 24, 72
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, cfg.seed_prompt).tolist()
    ctx = harness.make_context(cfg, target, draft, gamma, extra_seq=n_total + 64)
    done, segments, splits, agreed = 0, 0, 0, 0
    while done < n_total:
        uni = NpUniforms(synth.make_uniforms(3 * seg_len, gamma, cfg.seed_uniform + segments))
        print(f"algo={algo} segment={segments} prompt_len={len(prompt)}", flush=True)
        ref = []
        mk = lambda m: transformer.CachedModel(m, len(prompt) + seg_len + 4 * gamma + 8)
        ORACLE[algo](mk(tm), mk(dm), prompt, seg_len, gamma, uni, temperature=1.0, logit_scale=cfg.logit_scale,
                     trace=ref)
        ctx.prefill(prompt)
        got = _gpu_steps(amd, ctx, algo, gamma, seg_len, uni)
        k = 0
        while k < min(len(ref), len(got)) and ref[k]["tokens"] == got[k]["tokens"]:
            k += 1
        agreed += k
        committed = [t for s in ref[:k] for t in s["tokens"]]
        if k < min(len(ref), len(got)):
            print(f"  split at step {k}: oracle margin {ref[k]['margin']:.4f}", flush=True)
            # a draft-only step has no decision of its own: the split shows in the step that verifies its drafts
            m = min(ref[k]["margin"], ref[k - 1]["margin"] if k else 1.0)
            assert m < MARGIN_TOL, (segments, k, ref[k], got[k])
            committed += ref[k]["tokens"]
            splits += 1
        if not committed:                       # a split right after a draft-only step: restart from the same prompt
            segments += 1
            assert segments < 60
            continue
        prompt = prompt + committed
        done += len(committed)
        segments += 1
        assert segments < 60
    print(f"algo={algo}: {agreed} steps agreed, {splits} sub-margin splits", flush=True)
    assert agreed >= 2 * max(1, splits)
    ctx.close()


@pytest.mark.parametrize("algo", [3, 4])
def test_ablation_loops_take_the_oracles_decisions_on_the_librarys_own_logits(algo):
    """Every forward of the run against the fp32 oracle forward, every committed token against the oracle's ablation
    loop run on the library's own logits (see tests.util.LockstepModel)."""
    from tests.test_gpu_loops import lockstep_run
    from tests.util import EXACT_MARGIN
    cfg = synth.config("tiny")
    amd, harness, target, draft, tm, dm = _pair(cfg)
    agreed, splits, wt, wd, _ = lockstep_run(amd, harness, cfg, target, draft, tm, dm, algo, 4, 1.0, n_total=72,
                                             seed=cfg.seed_uniform, oracle_loop=ORACLE[algo], gpu_steps=_gpu_steps,
                                             uniform_rows=3)
    print(f"algo={algo}: {agreed} steps identical, {splits} splits within {EXACT_MARGIN} of a flip; worst logit "
          f"error target {wt:.2e} draft {wd:.2e}", flush=True)
    assert splits <= 2 and agreed >= 10 * max(1, splits)


@pytest.mark.parametrize("algo", [3, 4])
def test_ablation_loops_greedy_and_race_free(algo):
    cfg = synth.config("tiny")
    amd, harness, target, draft, tm, dm = _pair(cfg)
    gamma, n_gen = 4, 40
    prompt = synth.prompt_tokens(cfg.n_prompt, cfg.target.vocab, 13).tolist()
    uni = NpUniforms(synth.make_uniforms(3 * n_gen, gamma, 6))
    # greedy: same tokens as autoregressive decoding on the GPU (lossless)
    ctx = harness.make_context(cfg, target, draft, gamma, temperature=0.0)
    ctx.prefill(prompt)
    ar, _ = ctx.generate(amd.ALGO_AR, gamma, n_gen, uni)
    ctx.prefill(prompt)
    out, st = ctx.generate(algo, gamma, n_gen, uni)
    assert out == ar
    ctx.close()
    # sampled: overlapped == serialised == the call-by-call loop
    outs = []
    for serial in (True, False):
        c2 = harness.make_context(cfg, target, draft, gamma, serial=serial)
        c2.prefill(prompt)
        o, st = c2.generate(algo, gamma, n_gen, uni)
        outs.append(o)
        c2.close()
    assert outs[0] == outs[1]
    c3 = harness.make_context(cfg, target, draft, gamma)
    c3.prefill(prompt)
    steps = _gpu_steps(amd, c3, algo, gamma, n_gen, uni)
    assert [t for s in steps for t in s["tokens"]][:n_gen] == outs[0]
    c3.close()
