"""Oracle: the two ablations of Section 4.3 (test infrastructure only).

The paper names "PEARL w/o pre-verify" and "PEARL w/o post-verify" and reports their speed-ups (ablation table)
but gives no listing for them.  Readings used here (both keep the lossless acceptance rule of Eq. (1)):

w/o pre-verify   The drafting phase runs alone: gamma draft forwards, no target forward, nothing committed.
                 The verification phase that follows keeps the post-verify strategy: the target takes in the last
                 committed token and x_1..x_gamma (gamma + 1 rows) while the draft goes on to x_{gamma+1}..x_{2 gamma};
                 rows P_1..P_{gamma+1} test x_1..x_{gamma+1} (the last row verifies x_{gamma+1}, as Section 3.3 says of
                 the last logit).  All accepted: carry on with ordinary post-verify steps.  A rejection commits the
                 accepted prefix plus the resampled token and returns to the drafting phase.

w/o post-verify  The drafting phase keeps the pre-verify strategy (gamma draft forwards beside M_p(x), x_1 tested
                 early).  If x_1 is rejected, the corrected token is committed and drafting starts over.  If it is
                 accepted, the verification phase runs with the draft model idle: the target takes in x_1..x_gamma;
                 row P_i tests x_{i+1} (i < gamma); all accepted -> a bonus token is drawn from P_gamma as in vanilla
                 speculative decoding; then back to the drafting phase.

Same conventions as oracle.loops (committed tokens, frontier, uniforms indexed by step).
"""
from __future__ import annotations

from . import sampling
from .loops import PRE, POST, _decide, _draw, _prefill, _redraw

DRAFT, VERIFY = "draft-only", "verify-only"


def pearl_without_pre_verify(target, draft, prompt, n_generate, gamma, uni, temperature=1.0, logit_scale=1.0,
                             force=None, trace=None):
    P = lambda logits: sampling.probs(logits, temperature, logit_scale)
    committed = [int(t) for t in prompt]
    n0 = len(committed)
    _prefill([target, draft], committed)
    mode = DRAFT
    xs, qs = [], []                      # drafts after the last committed token, and their distributions
    first_verified = False               # xs[0] is already committed (it is the frontier)
    t = 0
    while len(committed) - n0 < n_generate:
        mg = [] if trace is not None else None
        n_before = len(committed)
        n_acc = 0
        # every step drafts gamma more tokens
        inp = [xs[-1]] if xs else committed[draft.len:]
        for i in range(gamma):
            q = P(draft.feed(inp)[-1])
            x = _draw(q, uni.draft[t, i], mg)
            xs.append(x); qs.append(q)
            inp = [x]
        if mode == DRAFT:
            mode_next = POST             # the next step verifies (and keeps drafting)
        else:
            # xs held gamma tokens before this step's drafting; the target takes in gamma (+1) tokens
            if first_verified:
                fed = xs[:gamma]                       # x_1 (frontier) .. x_gamma ; row i tests xs[i + 1]
                tests = list(range(1, gamma + 1))
            else:
                fed = [committed[-1]] + xs[:gamma]     # frontier, x_1 .. x_gamma ; row i tests xs[i]
                tests = list(range(0, gamma + 1))
            Pm = P(target.feed(fed))
            rej = None
            for row, k in enumerate(tests):
                if _decide(force, t, row, Pm[row], qs[k], xs[k], uni.accept[t, row], mg):
                    n_acc += 1
                else:
                    rej = (row, k)
                    break
            start = 1 if first_verified else 0
            if rej is None:
                last = tests[-1]
                committed += xs[start:last + 1]
                xs, qs = xs[last:], qs[last:]          # the last accepted draft is the new frontier
                first_verified = True
                mode_next = POST
            else:
                row, k = rej
                committed += xs[start:k] + [_redraw(Pm[row], qs[k], uni.resample[t], mg)]
                keep = len(committed) - 1
                target.rollback(keep)
                draft.rollback(keep)
                xs, qs, first_verified = [], [], False
                mode_next = DRAFT
        if trace is not None:
            trace.append({"mode": mode, "n_accepted": n_acc, "n_committed": len(committed) - n_before,
                          "next_mode": mode_next, "margin": min(mg), "tokens": committed[n_before:]})
        mode = mode_next
        t += 1
    return committed[n0:n0 + n_generate]


def pearl_without_post_verify(target, draft, prompt, n_generate, gamma, uni, temperature=1.0, logit_scale=1.0,
                              force=None, trace=None):
    P = lambda logits: sampling.probs(logits, temperature, logit_scale)
    committed = [int(t) for t in prompt]
    n0 = len(committed)
    _prefill([target, draft], committed)
    mode = PRE
    xs, qs = [], []
    t = 0
    while len(committed) - n0 < n_generate:
        mg = [] if trace is not None else None
        n_before = len(committed)
        frontier = committed[-1]
        if mode == PRE:
            base = len(committed) - 1
            xs, qs = [], []
            inp = committed[draft.len:]                # the frontier, preceded by x_gamma after an all-accept
            for i in range(gamma):
                q = P(draft.feed(inp)[-1])
                x = _draw(q, uni.draft[t, i], mg)
                xs.append(x); qs.append(q)
                inp = [x]
            p = P(target.feed([frontier])[0])
            if _decide(force, t, 0, p, qs[0], xs[0], uni.accept[t, 0], mg):
                committed.append(xs[0])
                n_acc, mode_next = 1, VERIFY
            else:
                committed.append(_redraw(p, qs[0], uni.resample[t], mg))
                draft.rollback(base + 1)
                n_acc, mode_next = 0, PRE
        else:
            Pm = P(target.feed(xs[:gamma]))            # P_i = distribution after x_i
            n_acc = 0
            for i in range(1, gamma):                  # P_i tests x_{i+1}
                if _decide(force, t, i - 1, Pm[i - 1], qs[i], xs[i], uni.accept[t, i - 1], mg):
                    n_acc += 1
                else:
                    break
            if n_acc == gamma - 1:
                y = _draw(Pm[gamma - 1], uni.resample[t], mg)       # bonus token
            else:
                y = _redraw(Pm[n_acc], qs[n_acc + 1], uni.resample[t], mg)
            committed += xs[1:1 + n_acc] + [y]
            keep = len(committed) - 1
            target.rollback(min(target.len, keep))
            draft.rollback(min(draft.len, keep))
            mode_next = PRE
        if trace is not None:
            trace.append({"mode": mode, "n_accepted": n_acc, "n_committed": len(committed) - n_before,
                          "next_mode": mode_next, "margin": min(mg), "tokens": committed[n_before:]})
        mode = mode_next
        t += 1
    return committed[n0:n0 + n_generate]
