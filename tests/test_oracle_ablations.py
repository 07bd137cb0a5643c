"""Pins for the oracle's ablation loops (PEARL without pre-verify / without post-verify), CPU only.

Both variants keep the lossless acceptance rule, so their joint output distribution must equal the target
model's (chi-square on toy table models), and greedy decoding must reproduce greedy autoregressive output.
"""
import numpy as np
import pytest
from scipy import stats

import synth
from oracle import ablations, loops, transformer
from tests.test_oracle_loops import RandUniforms, TableModel, _chi_square_of_loop, _tables, _tiny_pair
from tests.util import NpUniforms

VARIANTS = [ablations.pearl_without_pre_verify, ablations.pearl_without_post_verify]


@pytest.mark.parametrize("fn", VARIANTS)
@pytest.mark.parametrize("gamma,g", [(1, 3), (2, 3), (3, 4)])
def test_ablation_joint_output_distribution_equals_target(fn, gamma, g):
    v = 3
    tp, tq = _tables(v, 21)
    prompt = [1, 2]

    def run(rng):
        return fn(TableModel(tp), TableModel(tq), prompt, g, gamma, RandUniforms(rng, 3 * g + 3, gamma))

    chi2, df = _chi_square_of_loop(run, tp, prompt, g, 40_000, 5)
    assert chi2 < stats.chi2.ppf(1 - 1e-4, df), chi2


@pytest.mark.parametrize("fn", VARIANTS)
def test_ablation_greedy_equals_autoregressive(fn):
    cfg, tm, dm = _tiny_pair()
    prompt = synth.prompt_tokens(8, cfg.target.vocab, 7).tolist()
    n_gen, gamma = 20, 3
    uni = NpUniforms(synth.make_uniforms(3 * n_gen, gamma, 99))
    mk = lambda m: transformer.CachedModel(m, 96)
    ar = loops.autoregressive(mk(tm), prompt, n_gen, uni, temperature=0.0)
    tr = []
    out = fn(mk(tm), mk(dm), prompt, n_gen, gamma, uni, temperature=0.0, trace=tr)
    assert out == ar
    assert len({s["mode"] for s in tr}) >= 2


def test_ablation_step_structure():
    """Forced decisions: w/o pre-verify spends a step on drafting alone after every rejection; w/o post-verify
    alternates drafting (pre-verify) and verification and draws a bonus token when everything is accepted."""
    tp, tq = _tables(4, 3)
    gamma = 3
    uni = RandUniforms(np.random.default_rng(1), 40, gamma)
    tr = []
    t, d = TableModel(tp), TableModel(tq)
    ablations.pearl_without_pre_verify(t, d, [1, 2], 14, gamma, uni, force=lambda s, i: True, trace=tr)
    assert [s["n_committed"] for s in tr[:4]] == [0, gamma + 1, gamma, gamma]       # draft, first verify, post, post
    assert d.n_forwards - 1 == gamma * len(tr) and t.n_forwards - 1 == len(tr) - 1
    tr = []
    ablations.pearl_without_pre_verify(TableModel(tp), TableModel(tq), [1, 2], 6, gamma, uni,
                                       force=lambda s, i: i < 1, trace=tr)
    assert [s["mode"] for s in tr[:4]] == [ablations.DRAFT, loops.POST, ablations.DRAFT, loops.POST]
    assert [s["n_committed"] for s in tr[:4]] == [0, 2, 0, 2]
    tr = []
    t, d = TableModel(tp), TableModel(tq)
    ablations.pearl_without_post_verify(t, d, [1, 2], 12, gamma, uni, force=lambda s, i: True, trace=tr)
    assert [s["mode"] for s in tr[:4]] == [loops.PRE, ablations.VERIFY, loops.PRE, ablations.VERIFY]
    assert [s["n_committed"] for s in tr[:4]] == [1, gamma, 1, gamma]               # x_1 | x_2, x_3 + bonus
    assert d.n_forwards - 1 == gamma * (len(tr) // 2) and t.n_forwards - 1 == len(tr)
