"""Pins for the oracle's multi-token pre-verify loop (CPU only).

The loop keeps the lossless acceptance rule (Section 2, Eq. (1); Section 3.2), so whatever the candidate pool
guesses, the joint distribution of the emitted tokens must equal the target model's (chi-square on toy table
models, where guesses match about one time in three), greedy decoding must reproduce greedy autoregressive output,
and without guesses (k = 0) the loop must be Algorithm 2 itself.
"""
import numpy as np
import pytest
from scipy import stats

import synth
from oracle import loops, multi_preverify, transformer
from tests.test_oracle_loops import RandUniforms, TableModel, _chi_square_of_loop, _tables, _tiny_pair
from tests.util import NpUniforms


def test_pool_guess_is_the_continuation_of_the_most_recent_earlier_occurrence():
    g = multi_preverify.pool_guess
    assert g([5, 1, 2, 3, 1, 7, 8, 1], 2) == [7, 8]          # the occurrence at index 4, not the one at index 1
    assert g([5, 1, 2, 3, 1], 3) == [2, 3, 1]
    assert g([5, 1, 2, 3, 1], 9) == [2, 3, 1]                # no more than the text holds
    assert g([1, 1], 2) == [1]
    assert g([4, 5, 6], 2) == [] and g([4], 2) == [] and g([4, 4], 0) == []


@pytest.mark.parametrize("gamma,k,g", [(2, 1, 3), (3, 2, 4), (4, 3, 4)])
def test_joint_output_distribution_equals_target(gamma, k, g):
    v = 3
    tp, tq = _tables(v, 21)
    prompt = [1, 2, 1]

    def run(rng):
        return multi_preverify.pearl_multi_preverify(TableModel(tp), TableModel(tq), prompt, g, gamma, k,
                                                     RandUniforms(rng, g + 2, gamma))

    chi2, df = _chi_square_of_loop(run, tp, prompt, g, 60_000, 5)
    assert chi2 < stats.chi2.ppf(1 - 1e-4, df), chi2


def test_a_row_used_without_its_guess_matching_would_fail_the_distribution_pin():
    """Planted mistake: a pool that claims to have guessed whatever the draft model then draws (so every row counts
    as valid although the target computed it behind other tokens) breaks losslessness, and the same chi-square sees
    it."""
    v, gamma, k, g = 3, 3, 2, 4
    tp, tq = _tables(v, 21)
    prompt = [1, 2, 1]

    class Liar(TableModel):                   # a target that evaluates its rows behind the guesses it was fed ...
        pass

    def run(rng):
        uni = RandUniforms(rng, g + 2, gamma)
        t, d = TableModel(tp), TableModel(tq)
        real_feed = t.feed
        # ... while the loop is told (through `guess`) that the guesses equal the coming drafts: replace the fed
        # guesses by fixed tokens after the loop has decided they "match"
        def lying_feed(tokens):
            tokens = list(tokens)
            if len(tokens) > 1 and t.len >= len(prompt) - 1:
                tokens = [tokens[0]] + [0] * (len(tokens) - 1)
            return real_feed(tokens)
        t.feed = lying_feed
        # the coming drafts: replay the draft chain with the same uniforms on a copy
        def guess(committed, kk):
            from oracle import sampling
            c = list(committed)
            out = []
            step = guess.t
            for i in range(kk):
                q = tq[c[-2] if len(c) > 1 else 0, c[-1]]
                x = sampling.sample(q, uni.draft[step, i])
                out.append(x); c.append(x)
            return out
        guess.t = 0
        tr = []
        real_guess = guess

        def counting_guess(committed, kk):
            guess.t = len(tr_steps)
            return real_guess(committed, kk)
        tr_steps = tr
        return multi_preverify.pearl_multi_preverify(t, d, prompt, g, gamma, k, uni, trace=tr, guess=counting_guess)

    chi2, df = _chi_square_of_loop(run, tp, prompt, g, 30_000, 7)
    assert chi2 > 3 * stats.chi2.ppf(1 - 1e-4, df)


@pytest.mark.parametrize("gamma", [1, 2, 4])
def test_without_guesses_it_is_algorithm_2(gamma):
    tp, tq = _tables(5, 3)
    uni = RandUniforms(np.random.default_rng(4), 60, gamma)
    a, b = [], []
    out_a = loops.pearl(TableModel(tp), TableModel(tq), [1, 2], 40, gamma, uni, trace=a)
    out_b = multi_preverify.pearl_multi_preverify(TableModel(tp), TableModel(tq), [1, 2], 40, gamma, 0, uni, trace=b)
    assert out_a == out_b
    assert [(s["mode"], s["tokens"]) for s in a] == [(s["mode"], s["tokens"]) for s in b]


def test_step_structure_when_every_guess_matches():
    """A draft model that always continues with (last + 1) mod V, a pool that guesses exactly that, every test forced to
    accept: gamma = 4, k = 2.  The pre-verify step verifies x_1..x_3 in one target forward of 3 rows; x_4 stays pending, so
    the next post-verify forward takes in 2 tokens (x_3, x_4) and verifies x_4, x_5; from then on the windows are
    gamma wide again.  One target forward and gamma draft forwards per step throughout."""
    v, gamma, k = 7, 4, 2
    tq = np.full((v, v, v), 1e-12)
    for a in range(v):
        for b in range(v):
            tq[a, b, (b + 1) % v] = 1.0
    tq /= tq.sum(-1, keepdims=True)
    tp, _ = _tables(v, 2)
    guess = lambda committed, kk: [(committed[-1] + 1 + i) % v for i in range(kk)]
    tr = []
    t, d = TableModel(tp), TableModel(tq)
    rows = []
    real_feed = t.feed
    t.feed = lambda toks: (rows.append(len(toks)), real_feed(toks))[1]
    out = multi_preverify.pearl_multi_preverify(t, d, [3], 17, gamma, k, RandUniforms(np.random.default_rng(0), 20, gamma),
                                                force=lambda s, i: True, trace=tr, guess=guess)
    assert out[:8] == [(3 + 1 + i) % v for i in range(8)]
    assert [s["mode"] for s in tr[:4]] == [loops.PRE, loops.POST, loops.POST, loops.POST]
    assert [s["n_committed"] for s in tr[:4]] == [3, 2, 4, 4]
    assert [s["guess_rows_used"] for s in tr[:2]] == [2, 0]
    assert rows[:4] == [3, 2, 4, 4]
    assert d.n_forwards == gamma * len(tr) and t.n_forwards == len(tr)
    # a rejection inside the guessed rows: x_1 accepted, x_2 rejected -> two tokens, back to pre-verify
    tr = []
    multi_preverify.pearl_multi_preverify(TableModel(tp), TableModel(tq), [3], 6, gamma, k,
                                          RandUniforms(np.random.default_rng(0), 20, gamma),
                                          force=lambda s, i: i != 1, trace=tr, guess=guess)
    assert tr[0]["mode"] == loops.PRE and tr[0]["n_accepted"] == 1 and tr[0]["n_committed"] == 2
    assert tr[0]["next_mode"] == loops.PRE and tr[1]["mode"] == loops.PRE
    # every draft of the window verified inside the pre-verify step (k = gamma - 1): nothing pending, the post-verify
    # step's target forward takes in the frontier alone
    tr = []
    multi_preverify.pearl_multi_preverify(TableModel(tp), TableModel(tq), [3], 10, gamma, gamma - 1,
                                          RandUniforms(np.random.default_rng(0), 20, gamma),
                                          force=lambda s, i: True, trace=tr, guess=guess)
    assert [(s["mode"], s["n_committed"]) for s in tr[:3]] == [(loops.PRE, gamma), (loops.POST, 1), (loops.POST, gamma)]


def test_greedy_equals_autoregressive_and_guess_rows_get_used():
    cfg, tm, dm = _tiny_pair()
    prompt = synth.prompt_tokens(8, cfg.target.vocab, 7).tolist()
    n_gen, gamma, k = 80, 4, 3
    uni = NpUniforms(synth.make_uniforms(n_gen + 1, gamma, 99))
    mk = lambda m: transformer.CachedModel(m, 256)
    ar = loops.autoregressive(mk(tm), prompt, n_gen, uni, temperature=0.0)
    # greedy decoding of a random-init network soon repeats itself, so the pool guesses right; the small draft model
    # keeps being rejected, so pre-verify steps (the only ones with guess rows) keep coming
    tr = []
    out = multi_preverify.pearl_multi_preverify(mk(tm), mk(dm), prompt, n_gen, gamma, k, uni, temperature=0.0, trace=tr)
    assert out == ar
    assert sum(s["guess_rows_used"] for s in tr) >= 1
    # the target as its own draft: never rejected, one pre-verify step at the start, the same text
    out2 = multi_preverify.pearl_multi_preverify(mk(tm), mk(tm), prompt, n_gen, gamma, k, uni, temperature=0.0)
    assert out2 == ar


def test_caches_after_a_sampled_run_equal_a_clean_pass():
    """The target's cache takes in guessed tokens that are cut off again whenever a draft leaves the guessed path,
    and both caches are rolled back on every rejection: afterwards they must hold exactly what one clean pass over the
    committed text produces (a stale guess row or a draft row that survived a rollback would differ), the target
    lacking the frontier.  Guesses: the step's own continuation under the draft's arg-max, wrong about half the
    time for a sampled run."""
    cfg, tm, dm = _tiny_pair()
    prompt = synth.prompt_tokens(8, cfg.target.vocab, 7).tolist()
    n_gen, gamma, k = 40, 4, 3
    uni = NpUniforms(synth.make_uniforms(n_gen + 1, gamma, 99))
    t, d = transformer.CachedModel(tm, 128), transformer.CachedModel(dm, 128)
    peek = transformer.CachedModel(dm, 128)

    def guess(committed, kk):            # greedy continuation of the draft model from the committed text
        peek.rollback(0)
        lg = peek.feed(committed)[-1]
        out = []
        for _ in range(kk):
            out.append(int(np.argmax(lg)))
            lg = peek.feed([out[-1]])[0]
        return out

    tr = []
    out = multi_preverify.pearl_multi_preverify(t, d, prompt, n_gen, gamma, k, uni, temperature=0.5,
                                                logit_scale=cfg.logit_scale, trace=tr, guess=guess)
    assert len(out) == n_gen
    committed_len = len(prompt) + sum(s["n_committed"] for s in tr)
    assert t.len == committed_len - 1
    assert sum(s["guess_rows_used"] for s in tr) >= 1 and any(s["mode"] == loops.POST for s in tr)
    assert t.n_forwards == len(tr) + 1 and d.n_forwards == gamma * len(tr) + 1      # + the prompt pass of each
    full = prompt + out
    for cm, model in ((t, tm), (d, dm)):
        clean = transformer.CachedModel(model, 128)
        n_check = min(cm.len, len(full) - 1)
        clean.feed(full[:n_check])
        np.testing.assert_allclose(cm.cache.k[:, :n_check], clean.cache.k[:, :n_check], rtol=0, atol=1e-10)
        np.testing.assert_allclose(cm.cache.v[:, :n_check], clean.cache.v[:, :n_check], rtol=0, atol=1e-10)
