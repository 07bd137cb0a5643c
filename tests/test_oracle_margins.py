"""Pins for the oracle's decision margins (CPU only).

The GPU loop tests forgive a GPU / oracle split only on a step whose smallest decision margin is tiny, so the
margins themselves need pins with teeth: hand-worked values, the defining property (a perturbation smaller than
the margin never flips the decision, one slightly larger across the nearest edge does), planted factor-of-10
errors that these checks must reject, and the per-step minimum of the loops recomputed by a replay written
independently of the loops (explicit token lists and index arithmetic on table models, no caches).

Decisions whose margins are defined: an inverse-CDF draw (Section 2, x_i ~ q_i; the corrected / bonus token) and
the acceptance test of Eq. (1), r <= p[x]/q[x].
"""
import numpy as np
import pytest

from oracle import loops, sampling
from tests.test_oracle_loops import RandUniforms, TableModel, _tables


# ---------------------------------------------------------------------------------------------
# hand-worked values
# ---------------------------------------------------------------------------------------------
def test_sample_margin_hand_worked():
    w = [0.1, 0.0, 0.4, 0.5]                                   # CDF edges 0.1, 0.1, 0.5, 1.0
    assert sampling.sample_margin(w, 0.45) == pytest.approx(0.05, abs=1e-15)
    assert sampling.sample_margin(w, 0.30) == pytest.approx(0.20, abs=1e-15)
    assert sampling.sample_margin(w, 0.1) == pytest.approx(0.0, abs=1e-16)     # u on an edge
    assert sampling.sample_margin(w, 0.07) == pytest.approx(0.03, abs=1e-15)   # nearest edge above
    assert sampling.sample_margin([0.2, 0.3, 0.5], 0.49) == pytest.approx(0.01, abs=1e-15)
    # unnormalised weights: the margin is relative to the total
    assert sampling.sample_margin([2.0, 3.0, 5.0], 0.49) == pytest.approx(0.01, abs=1e-15)
    assert sampling.sample_margin([20.0, 30.0, 50.0], 0.49) == pytest.approx(0.01, abs=1e-15)


def test_accept_margin_hand_worked():
    p = np.array([0.1, 0.3, 0.6]); q = np.array([0.1, 0.6, 0.3])
    # r q[x] = 0.24 against p[x] = 0.3: |0.24 - 0.3| / 0.3
    assert sampling.accept_margin(p, q, 1, 0.4) == pytest.approx(0.2, abs=1e-15)
    # r q[x] = 0.36 against 0.3 (a rejection): 0.06 / 0.36
    assert sampling.accept_margin(p, q, 1, 0.6) == pytest.approx(1.0 / 6.0, abs=1e-15)
    # p[x] == q[x], r one fp32 step below 1
    r = 1.0 - 2.0 ** -24
    assert sampling.accept_margin(p, q, 0, r) == pytest.approx(2.0 ** -24, rel=1e-9)
    # p[x] far above q[x]: nowhere near a flip
    assert sampling.accept_margin(p, q, 2, 0.5) == pytest.approx(0.75, abs=1e-15)
    # the test sits exactly on the boundary
    assert sampling.accept_margin(p, q, 1, 0.5) == pytest.approx(0.0, abs=1e-16)


# ---------------------------------------------------------------------------------------------
# the defining property, as a checker that takes the margin function
# ---------------------------------------------------------------------------------------------
def _sample_margin_property(margin_fn, n_cases=400, seed=3):
    """Returns the number of violations of: moving u by 0.999 margins never changes the draw; moving it by
    1.001 margins towards the nearest interior CDF edge does."""
    rng = np.random.default_rng(seed)
    bad = 0
    for _ in range(n_cases):
        v = int(rng.integers(2, 12))
        w = rng.dirichlet(np.ones(v) * 0.6) * rng.uniform(0.5, 20.0)
        if rng.random() < 0.3:
            w[int(rng.integers(0, v))] = 0.0
        if not w.sum() > 0:
            continue
        u = float(rng.random())
        m = margin_fn(w, u)
        k = sampling.sample(w, u)
        for du in (-0.999 * m, 0.999 * m):
            if 0.0 <= u + du < 1.0 and sampling.sample(w, u + du) != k:
                bad += 1
        cdf = np.cumsum(w) / w.sum()
        edges = cdf[:-1]                                         # the last edge (1.0) cannot be crossed
        if len(edges) == 0:
            continue
        j = int(np.argmin(np.abs(edges - u)))
        if abs(edges[j] - u) > abs(1.0 - u):                     # the nearest edge is the last one: no flip to expect
            continue
        step = 1.001 * m + 1e-15
        u2 = u + step if edges[j] > u else u - step
        if 0.0 <= u2 < 1.0 and sampling.sample(w, u2) == k:
            bad += 1
    return bad


def _accept_margin_property(margin_fn, n_cases=400, seed=4):
    """Violations of: scaling p[x] by less than the margin never flips the test, by a little more (in the
    right direction) does."""
    rng = np.random.default_rng(seed)
    bad = 0
    for _ in range(n_cases):
        v = int(rng.integers(2, 10))
        p = rng.dirichlet(np.ones(v)); q = rng.dirichlet(np.ones(v))
        x = int(rng.integers(0, v)); r = float(rng.random())
        m = margin_fn(p, q, x, r)
        acc = sampling.accept(p, q, x, r)
        lhs, rhs = r * q[x], p[x]
        # move p[x] towards the boundary r q[x] by a fraction of the gap |lhs - rhs| = m * max(lhs, rhs)
        gap = m * max(lhs, rhs)
        for f, flips in ((0.999, False), (1.001, True)):
            p2 = p.copy()
            p2[x] = rhs - f * gap - 1e-18 if acc else rhs + f * gap + 1e-18
            if (sampling.accept(p2, q, x, r) != acc) != flips:
                bad += 1
    return bad


def test_margins_have_their_defining_property():
    assert _sample_margin_property(sampling.sample_margin) == 0
    assert _accept_margin_property(sampling.accept_margin) == 0


@pytest.mark.parametrize("factor", [10.0, 0.1])
def test_a_factor_of_ten_error_in_a_margin_is_caught(factor):
    """Planted mistakes (in the oracle, on the CPU): inflated margins claim safety where a flip happens, deflated
    ones (the dangerous kind: they would let every loop test forgive a real disagreement) fail to flip."""
    assert _sample_margin_property(lambda w, u: factor * sampling.sample_margin(w, u)) > 20
    assert _accept_margin_property(lambda p, q, x, r: factor * sampling.accept_margin(p, q, x, r)) > 20


def test_wrong_normaliser_or_missing_edge_is_caught():
    # margin relative to the largest weight instead of the total; margin that ignores the edge below u
    wrong_norm = lambda w, u: float(np.min(np.abs(np.cumsum(w) / np.max(w) - u * np.sum(w) / np.max(w))))
    assert _sample_margin_property(wrong_norm) > 20

    def above_only(w, u):
        cdf = np.cumsum(w) / np.sum(w)
        return float(np.min(cdf[cdf >= u] - u))
    assert _sample_margin_property(above_only) > 20


# ---------------------------------------------------------------------------------------------
# per-step minimum of the loops, recomputed by an independent replay
# ---------------------------------------------------------------------------------------------
def _cdf_gap(w, u):
    """Distance from u to the nearest normalised CDF edge, written out with a plain loop."""
    tot = float(sum(w))
    run, best = 0.0, 2.0
    for x in w:
        run += float(x)
        best = min(best, abs(run / tot - u))
    return best


def _ratio_gap(px, qx, r):
    a, b = r * qx, px
    return abs(a - b) / max(a, b) if max(a, b) > 0 else 1.0


def _replay_pearl_margins(tp, tq, prompt, trace, gamma, uni):
    """Per-step smallest margin from the trace's tokens alone.  The table models depend on the last two tokens,
    so every distribution of a step follows from the committed sequence and the drafts."""
    P = lambda seq: tp[seq[-2] if len(seq) > 1 else 0, seq[-1]]
    Q = lambda seq: tq[seq[-2] if len(seq) > 1 else 0, seq[-1]]
    committed = list(prompt)
    pending = []            # x_2 .. x_gamma carried into a post-verify step
    pending_q = []
    out = []
    for t, s in enumerate(trace):
        ms = []
        if s["mode"] == loops.PRE:
            seq = list(committed)
            xs, qs = [], []
            for i in range(gamma):
                q = Q(seq)
                ms.append(_cdf_gap(q, uni.draft[t, i]))
                x = sampling.sample(q, uni.draft[t, i])
                xs.append(x); qs.append(q); seq.append(x)
            p = P(committed)
            ms.append(_ratio_gap(p[xs[0]], qs[0][xs[0]], uni.accept[t, 0]))
            if s["n_accepted"] == 1:
                pending, pending_q = xs[1:], qs[1:]
            else:
                res = np.maximum(p - qs[0], 0.0)
                ms.append(_cdf_gap(res if res.sum() > 0 else p, uni.resample[t]))
                pending, pending_q = [], []
        else:
            x = [committed[-1]] + pending            # x_1 .. x_gamma
            qs = [None] + pending_q
            seq = committed + pending
            for i in range(gamma):                   # x_{gamma+1} .. x_{2 gamma}
                q = Q(seq)
                ms.append(_cdf_gap(q, uni.draft[t, i]))
                xn = sampling.sample(q, uni.draft[t, i])
                x.append(xn); qs.append(q); seq.append(xn)
            n_acc = s["n_accepted"]
            n_tests = gamma if n_acc == gamma else n_acc + 1
            for i in range(1, n_tests + 1):          # P_i tests x_{i+1}
                Pi = P(committed[:-1] + x[:i])
                ms.append(_ratio_gap(Pi[x[i]], qs[i][x[i]], uni.accept[t, i - 1]))
            if n_acc == gamma:
                pending, pending_q = x[gamma + 1:], qs[gamma + 1:]
            else:
                j = n_acc + 1
                Pj = P(committed[:-1] + x[:j])
                res = np.maximum(Pj - qs[j], 0.0)
                ms.append(_cdf_gap(res if res.sum() > 0 else Pj, uni.resample[t]))
                pending, pending_q = [], []
        committed += s["tokens"]
        out.append(min(ms))
    return out


@pytest.mark.parametrize("gamma,seed", [(3, 5), (2, 6), (5, 7)])
def test_pearl_step_margin_is_the_minimum_over_every_decision_of_the_step(gamma, seed):
    tp, tq0 = _tables(6, seed)
    tq = 0.7 * tp + 0.3 * tq0                        # a draft close to the target: pre- and post-verify steps, full accepts
    prompt = [1, 2, 3]
    n_gen = 60
    uni = RandUniforms(np.random.default_rng(seed), n_gen + 2, gamma)
    tr = []
    loops.pearl(TableModel(tp), TableModel(tq), prompt, n_gen, gamma, uni, trace=tr)
    modes = {s["mode"] for s in tr}
    assert modes == {loops.PRE, loops.POST}
    assert any(s["mode"] == loops.POST and s["n_accepted"] == gamma for s in tr)
    assert any(s["mode"] == loops.POST and s["n_accepted"] < gamma for s in tr)
    want = _replay_pearl_margins(tp, tq, prompt, tr, gamma, uni)
    got = [s["margin"] for s in tr]
    np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-15)


def test_sd_and_ar_step_margins():
    gamma, seed = 3, 9
    tp, tq0 = _tables(5, seed)
    tq = 0.6 * tp + 0.4 * tq0
    prompt = [0, 4]
    uni = RandUniforms(np.random.default_rng(seed), 50, gamma)
    P = lambda seq: tp[seq[-2] if len(seq) > 1 else 0, seq[-1]]
    Q = lambda seq: tq[seq[-2] if len(seq) > 1 else 0, seq[-1]]
    tr = []
    loops.speculative(TableModel(tp), TableModel(tq), prompt, 40, gamma, uni, trace=tr)
    committed = list(prompt)
    for t, s in enumerate(tr):
        ms, seq, xs, qs = [], list(committed), [], []
        for i in range(gamma):
            q = Q(seq)
            ms.append(_cdf_gap(q, uni.draft[t, i]))
            xs.append(sampling.sample(q, uni.draft[t, i])); qs.append(q); seq.append(xs[-1])
        n_acc = s["n_accepted"]
        for i in range(min(n_acc + 1, gamma)):       # row i tests x_{i+1}
            Pi = P(committed + xs[:i])
            ms.append(_ratio_gap(Pi[xs[i]], qs[i][xs[i]], uni.accept[t, i]))
        Pn = P(committed + xs[:n_acc])
        if n_acc == gamma:
            ms.append(_cdf_gap(Pn, uni.resample[t]))                 # bonus token
        else:
            res = np.maximum(Pn - qs[n_acc], 0.0)
            ms.append(_cdf_gap(res if res.sum() > 0 else Pn, uni.resample[t]))
        assert s["margin"] == pytest.approx(min(ms), rel=1e-9, abs=1e-15), (t, s)
        committed += s["tokens"]
    assert any(s["n_accepted"] == gamma for s in tr) and any(s["n_accepted"] < gamma for s in tr)
    tr = []
    out = loops.autoregressive(TableModel(tp), prompt, 20, uni, trace=tr)
    committed = list(prompt)
    for t, s in enumerate(tr):
        assert s["margin"] == pytest.approx(_cdf_gap(P(committed), uni.resample[t]), rel=1e-9, abs=1e-15)
        committed.append(out[t])
