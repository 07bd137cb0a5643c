"""Oracle: decoding loops (test infrastructure only).

autoregressive : K tokens = K serial target forwards (Section 1).
speculative    : vanilla speculative decoding with a fixed window gamma (Section 2):
                 gamma draft forwards, one target forward over the last committed token
                 plus the gamma drafts giving p_1..p_{gamma+1}, sequential acceptance,
                 residual resampling at the first rejection or a bonus token from p_{gamma+1}.
pearl          : Algorithms 1 and 2 with explicit caches.  One step always runs gamma draft
                 forwards and one target forward (side by side in the real system).

Vocabulary used below: *committed* = verified tokens (prompt included); the *frontier* is the
last committed token.  At every step boundary the target's cache holds all committed tokens
except the frontier.

Readings of Algorithm 2 that the listing leaves open or gets inconsistent:
  * Post-verify indexing.  The target takes in the gamma tokens x_1..x_gamma and returns
    P_1..P_gamma with P_i the distribution of the token *after* x_i.  x_1 was already
    verified (by the preceding pre-verify, or by the last row of the preceding post-verify:
    Section 3.3 says that last logit verifies x_{gamma+1}), so P_i tests x_{i+1} against
    q_{i+1}, i = 1..gamma; x_1 is never tested twice.  This matches the Figure 3 narrative
    (target takes in x7,x8,x9; x8 accepted, x9 rejected) and keeps the output lossless.
  * The loop stops on the number of *committed* tokens and the output is cut to exactly
    n_generate tokens; drafted-but-unverified tokens are never output.
  * All-accept in post-verify commits gamma tokens and draws no bonus token (Section 3.3).
  * Uniforms are fixed arrays indexed by (step, purpose, position), so a draw does not depend
    on the path taken so far; a post-verify step owns gamma acceptance uniforms even if an
    early rejection leaves some unused (Algorithm 2 draws r_1..r_gamma up front).

`models` expose feed(tokens) -> logits [len(tokens), V], rollback(new_len) and .len.
`uni` exposes arrays draft[t, i], accept[t, i], resample[t].
`force(t, i)` (optional) overrides the i-th acceptance decision of step t - used only by the
closed-form throughput pins and the Figure 3 trace.
"""
from __future__ import annotations

import numpy as np

from . import sampling

PRE, POST = "pre-verify", "post-verify"


def _decide(force, t, i, p_row, q_row, x, r, margins=None):
    if force is not None:
        f = force(t, i)
        if f is not None:
            return bool(f)
    if margins is not None:
        margins.append(sampling.accept_margin(p_row, q_row, x, r))
    return sampling.accept(p_row, q_row, x, r)


def _draw(weights, u, margins=None):
    if margins is not None:
        margins.append(sampling.sample_margin(weights, u))
    return sampling.sample(weights, u)


def _redraw(p_row, q_row, u, margins=None):
    if margins is not None:
        res = sampling.residual(p_row, q_row)
        margins.append(sampling.sample_margin(res if res.sum() > 0.0 else p_row, u))
    return sampling.resample(p_row, q_row, u)


def _prefill(models, prompt):
    if len(prompt) < 1:
        raise ValueError("prompt must hold at least one token")
    if len(prompt) > 1:
        for m in models:
            m.feed(prompt[:-1])


def autoregressive(target, prompt, n_generate, uni, temperature=1.0, logit_scale=1.0, trace=None):
    committed = [int(t) for t in prompt]
    _prefill([target], committed)
    for t in range(n_generate):
        mg = [] if trace is not None else None
        p = sampling.probs(target.feed([committed[-1]])[0], temperature, logit_scale)
        committed.append(_draw(p, uni.resample[t], mg))
        if trace is not None:
            trace.append({"mode": "ar", "n_accepted": 0, "n_committed": 1, "margin": min(mg)})
    return committed[len(prompt):]


def speculative(target, draft, prompt, n_generate, gamma, uni, temperature=1.0, logit_scale=1.0,
                force=None, trace=None):
    P = lambda logits: sampling.probs(logits, temperature, logit_scale)
    committed = [int(t) for t in prompt]
    n0 = len(committed)
    _prefill([target, draft], committed)
    t = 0
    while len(committed) - n0 < n_generate:
        frontier = committed[-1]
        mg = [] if trace is not None else None
        inp = committed[draft.len:]           # the frontier, preceded by the last draft after an all-accept
        xs, qs = [], []
        for i in range(gamma):                # drafting phase: x_i ~ q_i
            q = P(draft.feed(inp)[-1])
            x = _draw(q, uni.draft[t, i], mg)
            xs.append(x); qs.append(q)
            inp = [x]
        Pm = P(target.feed([frontier] + xs))  # p_1 .. p_{gamma+1}
        n_acc = 0
        for i in range(gamma):                # p_{i+1} (row i) tests x_{i+1}
            if _decide(force, t, i, Pm[i], qs[i], xs[i], uni.accept[t, i], mg):
                n_acc += 1
            else:
                break
        if n_acc == gamma:
            y = _draw(Pm[gamma], uni.resample[t], mg)
        else:
            y = _redraw(Pm[n_acc], qs[n_acc], uni.resample[t], mg)
        committed += xs[:n_acc] + [y]
        keep = len(committed) - 1
        target.rollback(min(target.len, keep))
        draft.rollback(min(draft.len, keep))
        if trace is not None:
            trace.append({"mode": "sd", "n_accepted": n_acc, "n_committed": n_acc + 1, "margin": min(mg),
                          "tokens": xs[:n_acc] + [y]})
        t += 1
    return committed[n0:n0 + n_generate]


def pearl(target, draft, prompt, n_generate, gamma, uni, temperature=1.0, logit_scale=1.0,
          force=None, trace=None):
    P = lambda logits: sampling.probs(logits, temperature, logit_scale)
    committed = [int(t) for t in prompt]
    n0 = len(committed)
    _prefill([target, draft], committed)
    mode = PRE
    pending, pending_q = [], []               # x_2..x_gamma and q_2..q_gamma carried into a post-verify step
    t = 0
    while len(committed) - n0 < n_generate:
        frontier = committed[-1]
        mg = [] if trace is not None else None
        n_before = len(committed)
        if mode == PRE:
            base = draft.len
            xs, qs = [], []
            inp = frontier
            for i in range(gamma):            # q_i = M_q(x + [x_1..x_{i-1}]), x_i ~ q_i
                q = P(draft.feed([inp])[0])
                x = _draw(q, uni.draft[t, i], mg)
                xs.append(x); qs.append(q)
                inp = x
            p = P(target.feed([frontier])[0])  # p = M_p(x), side by side with the drafting
            if _decide(force, t, 0, p, qs[0], xs[0], uni.accept[t, 0], mg):
                committed.append(xs[0])
                pending, pending_q = xs[1:], qs[1:]
                n_acc, n_com, mode_next = 1, 1, POST
            else:
                committed.append(_redraw(p, qs[0], uni.resample[t], mg))
                draft.rollback(base + 1)      # keep the old frontier only
                pending, pending_q = [], []
                n_acc, n_com, mode_next = 0, 1, PRE
        else:
            x = [frontier] + pending          # x[i-1] = x_i, i = 1..gamma (x_1 is the frontier)
            qs = [None] + pending_q           # qs[i-1] = q_i (q_1 no longer needed)
            inp = x[-1]
            for i in range(gamma):            # keep drafting x_{gamma+1}..x_{2 gamma}
                q = P(draft.feed([inp])[0])
                xn = _draw(q, uni.draft[t, i], mg)
                x.append(xn); qs.append(q)
                inp = xn
            Pm = P(target.feed(x[:gamma]))    # P_i = M_p(x + [x_1..x_i]), i = 1..gamma
            n_acc = 0
            for i in range(1, gamma + 1):     # P_i tests x_{i+1} against q_{i+1}
                if _decide(force, t, i - 1, Pm[i - 1], qs[i], x[i], uni.accept[t, i - 1], mg):
                    n_acc += 1
                else:
                    break
            if n_acc == gamma:
                committed += x[1:gamma + 1]
                pending, pending_q = x[gamma + 1:], qs[gamma + 1:]
                n_com, mode_next = gamma, POST
            else:
                j = n_acc + 1                 # P_j rejected x_{j+1}
                y = _redraw(Pm[j - 1], qs[j], uni.resample[t], mg)
                committed += x[1:j] + [y]
                keep = len(committed) - 1
                target.rollback(keep)
                draft.rollback(keep)
                pending, pending_q = [], []
                n_com, mode_next = n_acc + 1, PRE
        if trace is not None:
            trace.append({"mode": mode, "n_accepted": n_acc, "n_committed": n_com, "next_mode": mode_next,
                          "margin": min(mg), "tokens": committed[n_before:]})
        mode = mode_next
        t += 1
    return committed[n0:n0 + n_generate]
