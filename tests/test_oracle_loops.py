"""Pins for the oracle's decoding loops (CPU only).

* Figure 3 worked example and the App. B mode table (fixtures under tests/golden/).
* Losslessness (Section 3.2: same lossless verification as speculative sampling): the joint
  distribution of the emitted tokens equals the target model's, checked by chi-square on toy
  table models; greedy PEARL == greedy SD == greedy autoregressive.
* Every step costs gamma draft forwards and one target forward (App. C/E forward counts).
* Closed-form tokens per step under i.i.d. acceptance alpha (two-state Markov chain, derived below).
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch
from scipy import stats

import synth
from oracle import loops, sampling, transformer
from tests.util import NpUniforms, oracle_model

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


class TableModel:
    """Toy 'language model': the next-token distribution is a fixed table row chosen by the last two tokens."""

    def __init__(self, table):
        self.table = np.asarray(table, dtype=np.float64)      # [V, V, V]
        self.hist = []
        self.n_forwards = 0

    @property
    def len(self):
        return len(self.hist)

    def feed(self, tokens):
        self.n_forwards += 1
        rows = []
        for t in tokens:
            self.hist.append(int(t))
            prev = self.hist[-2] if len(self.hist) > 1 else 0
            rows.append(np.log(self.table[prev, self.hist[-1]]))
        return np.stack(rows)

    def rollback(self, n):
        assert 0 <= n <= len(self.hist)
        del self.hist[n:]


class RandUniforms:
    def __init__(self, rng, n_steps, gamma):
        self.draft = rng.random((n_steps, gamma))
        self.accept = rng.random((n_steps, gamma + 1))
        self.resample = rng.random(n_steps)


def _tables(v, seed):
    rng = np.random.default_rng(seed)
    return rng.dirichlet(np.ones(v) * 0.8, size=(v, v)), rng.dirichlet(np.ones(v) * 0.8, size=(v, v))


def _exact_joint(table, prompt, g):
    v = table.shape[0]
    out = {}
    for seq in itertools.product(range(v), repeat=g):
        h = list(prompt)
        pr = 1.0
        for y in seq:
            pr *= table[h[-2] if len(h) > 1 else 0, h[-1], y]
            h.append(y)
        out[seq] = pr
    return out


def _chi_square_of_loop(run, tp, prompt, g, n_runs, seed):
    exact = _exact_joint(tp, prompt, g)
    keys = sorted(exact)
    idx = {k: i for i, k in enumerate(keys)}
    counts = np.zeros(len(keys))
    rng = np.random.default_rng(seed)
    for _ in range(n_runs):
        counts[idx[tuple(run(rng))]] += 1
    e = n_runs * np.array([exact[k] for k in keys])
    return float(((counts - e) ** 2 / e).sum()), len(keys) - 1


@pytest.mark.parametrize("gamma,g", [(2, 3), (3, 4)])
def test_pearl_joint_output_distribution_equals_target(gamma, g):
    v = 3
    tp, tq = _tables(v, 21)
    prompt = [1, 2]

    def run(rng):
        return loops.pearl(TableModel(tp), TableModel(tq), prompt, g, gamma, RandUniforms(rng, g + 1, gamma))

    chi2, df = _chi_square_of_loop(run, tp, prompt, g, 60_000, 5)
    assert chi2 < stats.chi2.ppf(1 - 1e-4, df), chi2


def test_wrong_post_verify_indexing_would_fail_the_distribution_pin():
    """The same chi-square rejects a loop that pairs P_i with q_i (instead of q_{i+1}) in post-verify:
    built here by shifting the draft table the loop sees, to show the pin has teeth."""
    v, gamma, g = 3, 2, 3
    tp, tq = _tables(v, 21)
    prompt = [1, 2]

    class Misaligned(TableModel):          # reports the distribution of one position earlier
        def feed(self, tokens):
            rows = super().feed(tokens)
            return np.roll(rows, 1, axis=-1)

    def run(rng):
        # drafts are drawn from rolled rows but verified as if they came from the unrolled ones
        d = Misaligned(tq)
        out = loops.pearl(TableModel(tp), d, prompt, g, gamma, RandUniforms(rng, g + 1, gamma))
        return out

    # a consistent (if odd) draft keeps the output exact ...
    chi2, df = _chi_square_of_loop(run, tp, prompt, g, 30_000, 6)
    assert chi2 < stats.chi2.ppf(1 - 1e-4, df)

    # ... while verifying against the wrong q row does not
    real_accept = sampling.accept

    def run_bad(rng):
        def bad_accept(p_row, q_row, x, r):
            return real_accept(p_row, np.roll(q_row, 1), x, r)
        sampling.accept = bad_accept
        try:
            return loops.pearl(TableModel(tp), TableModel(tq), prompt, g, gamma, RandUniforms(rng, g + 1, gamma))
        finally:
            sampling.accept = real_accept

    chi2, df = _chi_square_of_loop(run_bad, tp, prompt, g, 30_000, 7)
    assert chi2 > 3 * stats.chi2.ppf(1 - 1e-4, df)


def test_speculative_decoding_joint_output_distribution_equals_target():
    v, gamma, g = 3, 3, 4
    tp, tq = _tables(v, 33)
    prompt = [0, 2]

    def run(rng):
        return loops.speculative(TableModel(tp), TableModel(tq), prompt, g, gamma, RandUniforms(rng, g + 1, gamma))

    chi2, df = _chi_square_of_loop(run, tp, prompt, g, 60_000, 8)
    assert chi2 < stats.chi2.ppf(1 - 1e-4, df), chi2


def test_autoregressive_distribution():
    v, g = 3, 2
    tp, _ = _tables(v, 4)
    prompt = [2]

    def run(rng):
        return loops.autoregressive(TableModel(tp), prompt, g, RandUniforms(rng, g, 1))

    chi2, df = _chi_square_of_loop(run, tp, prompt, g, 40_000, 9)
    assert chi2 < stats.chi2.ppf(1 - 1e-4, df)


# ---------------------------------------------------------------------------------------------
# Worked examples from the paper
# ---------------------------------------------------------------------------------------------
def _read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


def _scripted(decisions):
    """force(t, i) from a per-step list of decisions; unspecified positions are accepted."""
    def force(t, i):
        d = decisions[t] if t < len(decisions) else []
        return d[i] if i < len(d) else True
    return force


def test_figure3_trace():
    rows = _read_golden("fig3_trace.txt")      # step, mode, decisions, committed
    gamma = 3
    tp, tq = _tables(5, 1)
    decisions = [[c == "A" for c in r[2]] for r in rows]
    n_total = sum(int(r[3]) for r in rows)
    tr = []
    rng = np.random.default_rng(0)
    d = TableModel(tq)
    out = loops.pearl(TableModel(tp), d, [1, 2], n_total, gamma, RandUniforms(rng, 8, gamma),
                      force=_scripted(decisions), trace=tr)
    assert [s["mode"] for s in tr] == [r[1] for r in rows]
    assert [s["n_committed"] for s in tr] == [int(r[3]) for r in rows]
    assert tr[-1]["next_mode"] == loops.PRE
    assert len(out) == 7 and len(tr) == 4       # [y1, x4, x5, x6, x7, x8, y2] in four steps
    assert d.n_forwards - 1 == 4 * gamma        # (one prefill call) + gamma draft forwards per step


def test_appendix_b_mode_sequence():
    rows = _read_golden("appb_modes.txt")       # step, mode, accepted-before-reject or 'all'
    gamma = 5
    decisions = []
    for r in rows:
        k = gamma if r[2] == "all" else int(r[2])
        decisions.append([True] * k + [False])
    tp, tq = _tables(4, 2)
    tr = []
    rng = np.random.default_rng(1)
    n_total = 18
    loops.pearl(TableModel(tp), TableModel(tq), [0, 1], n_total, gamma, RandUniforms(rng, 20, gamma),
                force=_scripted(decisions), trace=tr)
    tr = tr[:len(rows)]
    assert [s["mode"] for s in tr] == [r[1] for r in rows]
    assert [s["n_committed"] for s in tr] == [int(r[3]) for r in rows]


# ---------------------------------------------------------------------------------------------
# Invariants of the loops
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("gamma", [1, 2, 4, 5])
def test_forward_count_ratio_is_gamma_to_one(gamma):
    tp, tq = _tables(4, 3)
    t, d = TableModel(tp), TableModel(tq)
    tr = []
    loops.pearl(t, d, [1, 2, 3], 40, gamma, RandUniforms(np.random.default_rng(3), 41, gamma), trace=tr)
    steps = len(tr)
    assert t.n_forwards - 1 == steps and d.n_forwards - 1 == gamma * steps


@pytest.mark.parametrize("alpha,gamma", [(0.9, 4), (0.9, 5), (0.5, 4), (0.7, 8)])
def test_tokens_per_step_closed_form(alpha, gamma):
    """i.i.d. acceptance with probability alpha.

    SD: a step commits 1 + (number accepted before the first rejection, at most gamma)
        => E = sum_{k=0..gamma} alpha^k = (1 - alpha^(gamma+1)) / (1 - alpha).
    PEARL: two-state chain.  PRE commits 1 and moves to POST w.p. alpha.  POST commits
        min(#accepted + 1, gamma), E = (1 - alpha^gamma)/(1 - alpha), and stays w.p. alpha^gamma.
        Stationary P(POST) = alpha / (1 + alpha - alpha^gamma), hence
        E[tokens/step] = (1 - alpha^gamma) / ((1 - alpha)(1 + alpha - alpha^gamma)).
    """
    n_steps = 40_000
    rng = np.random.default_rng(17)
    coin = rng.random((n_steps + 8, gamma + 1)) < alpha
    force = lambda t, i: bool(coin[t, i])
    tp, tq = _tables(3, 5)
    uni = RandUniforms(np.random.default_rng(1), n_steps + 8, gamma)

    tr = []
    loops.pearl(TableModel(tp), TableModel(tq), [1], n_steps, gamma, uni, force=force, trace=tr)
    got = sum(s["n_committed"] for s in tr) / len(tr)
    want = (1 - alpha ** gamma) / ((1 - alpha) * (1 + alpha - alpha ** gamma))
    assert abs(got - want) < 0.02 * want, (got, want)
    p_post = sum(s["mode"] == loops.POST for s in tr) / len(tr)
    assert abs(p_post - alpha / (1 + alpha - alpha ** gamma)) < 0.02

    tr = []
    loops.speculative(TableModel(tp), TableModel(tq), [1], n_steps, gamma, uni, force=force, trace=tr)
    got = sum(s["n_committed"] for s in tr) / len(tr)
    want = (1 - alpha ** (gamma + 1)) / (1 - alpha)
    assert abs(got - want) < 0.02 * want, (got, want)


def test_closed_form_values_quoted_for_the_workload_tables():
    f_sd = lambda a, g: (1 - a ** (g + 1)) / (1 - a)
    f_pl = lambda a, g: (1 - a ** g) / ((1 - a) * (1 + a - a ** g))
    assert abs(f_sd(0.9, 4) - 4.0951) < 1e-4 and abs(f_pl(0.9, 4) - 2.7647) < 1e-4
    assert abs(f_sd(0.5, 4) - 1.9375) < 1e-4 and abs(f_pl(0.5, 4) - 1.3043) < 1e-4


def _tiny_pair(dtype=np.float64):
    cfg = synth.config("tiny", depth=2)
    cfg.target.vocab = cfg.draft.vocab = 64
    tw, dw = synth.make_pair(cfg)
    return cfg, oracle_model(tw, cfg.target, dtype), oracle_model(dw, cfg.draft, dtype)


def test_greedy_pearl_equals_greedy_sd_equals_greedy_autoregressive():
    cfg, tm, dm = _tiny_pair()
    prompt = synth.prompt_tokens(8, cfg.target.vocab, 7).tolist()
    n_gen, gamma = 24, 3
    uni = NpUniforms(synth.make_uniforms(n_gen + 1, gamma, 99))
    mk = lambda m: transformer.CachedModel(m, 64)
    ar = loops.autoregressive(mk(tm), prompt, n_gen, uni, temperature=0.0)
    sd = loops.speculative(mk(tm), mk(dm), prompt, n_gen, gamma, uni, temperature=0.0)
    tr = []
    pl = loops.pearl(mk(tm), mk(dm), prompt, n_gen, gamma, uni, temperature=0.0, trace=tr)
    assert ar == sd == pl
    # and the plain definition: arg-max of the target, token by token, with no cache reuse at all
    seq = list(prompt)
    for _ in range(6):
        logits = transformer.CachedModel(tm, 64).feed(seq)[-1]
        seq.append(int(np.argmax(logits)))
    assert seq[len(prompt):] == ar[:6]


def test_sampled_pearl_leaves_caches_as_if_never_speculated():
    """After the loop the target cache holds exactly the committed tokens but the frontier, with the
    same keys/values a single clean pass over those tokens produces (rollback leaves nothing stale)."""
    cfg, tm, dm = _tiny_pair()
    prompt = synth.prompt_tokens(8, cfg.target.vocab, 7).tolist()
    n_gen, gamma = 20, 4
    uni = NpUniforms(synth.make_uniforms(n_gen + 1, gamma, 99))
    t, d = transformer.CachedModel(tm, 96), transformer.CachedModel(dm, 96)
    tr = []
    out = loops.pearl(t, d, prompt, n_gen, gamma, uni, temperature=1.0, logit_scale=cfg.logit_scale, trace=tr)
    assert len(out) == n_gen
    total = sum(s["n_committed"] for s in tr)
    committed_len = len(prompt) + total
    assert t.len == committed_len - 1                      # target lacks exactly the frontier
    modes = {s["mode"] for s in tr}
    assert loops.PRE in modes and loops.POST in modes       # the run exercises both strategies
    # rebuild the committed sequence (the output may be cut inside the last step)
    clean = transformer.CachedModel(tm, 96)
    full = prompt + out
    n_check = min(t.len, len(full) - 1)
    clean.feed(full[:n_check])
    np.testing.assert_allclose(t.cache.k[:, :n_check], clean.cache.k[:, :n_check], rtol=0, atol=1e-10)
    np.testing.assert_allclose(t.cache.v[:, :n_check], clean.cache.v[:, :n_check], rtol=0, atol=1e-10)


def test_draft_placement_beside_a_pipelined_target_matches_the_worked_example():
    """The paper's multi-GPU answer to co-location (appendix on resource-constrained scenarios), as a design aid:
    the displayed occupancy sequences for c = 5, g = 4 (fixture) and no slot with both models on one device there;
    for every window gamma = c the placement is collision-free exactly when the first half of the drafting ends
    before the target reaches the last device and not before it has left the first one."""
    from oracle import placement
    rows = {}
    for line in open(os.path.join(GOLDEN, "rc_occupancy.txt")):
        line = line.split("#")[0].split()
        if line:
            rows[line[0]] = [int(v) for v in line[1:]]
    target, draft = placement.occupancy(5, 4, 5)
    assert target == rows["target"] and draft == rows["draft"]
    assert placement.collisions(5, 4, 5) == 0
    # gamma = c (the calibrated window): collision-free when the first ceil(gamma/2) tokens (g slots each) end no
    # later than the target reaches the last device, (g-1)*c, and the target has left device 0 (c slots) by then
    for g in range(2, 9):
        for c in range(1, 17):
            first = -(-c // 2)
            free = first * g <= (g - 1) * c and first * g >= c
            assert (placement.collisions(c, g, c) == 0) == free, (c, g)
    assert placement.collisions(5, 2, 5) > 0          # two devices are too few at c = 5
    with pytest.raises(ValueError):
        placement.occupancy(5, 1, 5)
