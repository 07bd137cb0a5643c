"""Oracle: PEARL with multi-token pre-verify (test infrastructure only).

Section 4.3 closes with the remark that pre-verify could be improved by pre-verifying several draft tokens, in the
manner of the candidate pools that lookahead-style decoders keep; the paper gives no algorithm.  The reading used here
keeps the lossless acceptance rule of Eq. (1) untouched and only changes which target rows exist when drafting ends:

  * A candidate pool guesses how the text goes on after the last committed token x (the frontier): g_1..g_m, m <= k.
    The pool here is the committed text itself, as an n-gram cache: the tokens that followed the most recent earlier
    occurrence of the frontier token (possibly none).
  * In a pre-verify step the target takes in x, g_1..g_m in ONE forward, side by side with the gamma draft forwards,
    giving P_0 = M_p(x), P_i = M_p(x + [g_1..g_i]).  Row P_0 tests x_1 exactly as in pre-verify (Section 3.2).  If x_1
    is accepted and x_1 == g_1, then P_1 is the target's distribution after x_1 and tests x_2 (against q_2) at once;
    and so on while the accepted drafts keep matching the guesses and drafts are left.
  * A rejection at x_j commits x_1..x_{j-1} and a token from norm(max(0, P_{j-1} - q_j)); both caches drop everything
    behind the committed text; the next step is a pre-verify step again.
  * Otherwise the n >= 1 accepted drafts are committed, the target's cache is cut back to the committed text but the
    frontier (guess rows beyond it are dropped), and the drafts x_{n+1}..x_gamma stay pending: the next step is a
    post-verify step (Section 3.3) whose target forward takes in x_n and the pending drafts - fewer than gamma rows
    this once, x_n alone if all gamma drafts were verified - while the draft model drafts gamma more.

Every committed token is an accepted draft tested against the target's exact distribution for its actual prefix, or
a residual / plain draw from it: the output distribution is the target's (pinned by the chi-square test), whatever
the pool guesses; guesses only decide how many rows of the forward are usable.  With k = 0 this is Algorithm 2.

Same conventions as oracle.loops (committed tokens, frontier, uniforms indexed by step: accept[t, i] is the i-th test
of step t).
"""
from __future__ import annotations

from . import sampling
from .loops import PRE, POST, _decide, _draw, _prefill, _redraw


def pool_guess(committed, k: int):
    """Up to k tokens that followed the most recent earlier occurrence of the last committed token."""
    if k <= 0 or len(committed) < 2:
        return []
    last = committed[-1]
    for j in range(len(committed) - 2, -1, -1):
        if committed[j] == last:
            return [int(t) for t in committed[j + 1:j + 1 + k]]
    return []


def pearl_multi_preverify(target, draft, prompt, n_generate, gamma, k, uni, temperature=1.0, logit_scale=1.0,
                          force=None, trace=None, guess=pool_guess):
    P = lambda logits: sampling.probs(logits, temperature, logit_scale)
    committed = [int(t) for t in prompt]
    n0 = len(committed)
    _prefill([target, draft], committed)
    mode = PRE
    pending, pending_q = [], []               # unverified drafts behind the frontier and their distributions
    t = 0
    while len(committed) - n0 < n_generate:
        frontier = committed[-1]
        mg = [] if trace is not None else None
        n_before = len(committed)
        n_guess_used = 0
        if mode == PRE:
            g = list(guess(committed, min(k, gamma - 1)))
            xs, qs = [], []
            inp = committed[draft.len:]       # the frontier (after a fully verified window: preceded by x_gamma)
            for i in range(gamma):            # q_i = M_q(x + [x_1..x_{i-1}]), x_i ~ q_i
                q = P(draft.feed(inp)[-1])
                x = _draw(q, uni.draft[t, i], mg)
                xs.append(x); qs.append(q)
                inp = [x]
            Pm = P(target.feed([frontier] + g))       # P_0 = M_p(x), P_i = M_p(x + [g_1..g_i])
            n_acc, rejected = 0, False
            for i in range(gamma):            # row i tests x_{i+1}; it exists if x_1..x_i are the guesses g_1..g_i
                if i > len(g) or (i >= 1 and xs[i - 1] != g[i - 1]):
                    break
                if _decide(force, t, i, Pm[i], qs[i], xs[i], uni.accept[t, i], mg):
                    n_acc += 1
                else:
                    rejected = True
                    break
            n_guess_used = max(n_acc - 1, 0) if not rejected else n_acc
            if rejected:
                y = _redraw(Pm[n_acc], qs[n_acc], uni.resample[t], mg)
                committed += xs[:n_acc] + [y]
                keep = len(committed) - 1
                target.rollback(keep)
                draft.rollback(min(draft.len, keep))
                pending, pending_q = [], []
                mode_next = PRE
            else:
                committed += xs[:n_acc]
                target.rollback(len(committed) - 1)   # the guess rows behind the new frontier go
                pending, pending_q = xs[n_acc:], qs[n_acc:]
                mode_next = POST              # also when nothing is pending: the target then takes in the frontier alone
        else:
            x = [frontier] + pending          # x[i-1] = x_i, i = 1..m (x_1 is the frontier), m <= gamma
            qs = [None] + pending_q
            m = len(x)
            inp = x[-1]
            for i in range(gamma):            # the draft goes on: gamma more tokens
                q = P(draft.feed([inp])[0])
                xn = _draw(q, uni.draft[t, i], mg)
                x.append(xn); qs.append(q)
                inp = xn
            Pm = P(target.feed(x[:m]))        # P_i = M_p(.. x_1..x_i), i = 1..m
            n_acc = 0
            for i in range(1, m + 1):         # P_i tests x_{i+1} against q_{i+1}
                if _decide(force, t, i - 1, Pm[i - 1], qs[i], x[i], uni.accept[t, i - 1], mg):
                    n_acc += 1
                else:
                    break
            if n_acc == m:
                committed += x[1:m + 1]
                pending, pending_q = x[m + 1:], qs[m + 1:]
                mode_next = POST
            else:
                j = n_acc + 1                 # P_j rejected x_{j+1}
                y = _redraw(Pm[j - 1], qs[j], uni.resample[t], mg)
                committed += x[1:j] + [y]
                keep = len(committed) - 1
                target.rollback(keep)
                draft.rollback(keep)
                pending, pending_q = [], []
                mode_next = PRE
        if trace is not None:
            trace.append({"mode": mode, "n_accepted": n_acc, "n_committed": len(committed) - n_before,
                          "next_mode": mode_next, "margin": min(mg), "tokens": committed[n_before:],
                          "guess_rows_used": n_guess_used})
        mode = mode_next
        t += 1
    return committed[n0:n0 + n_generate]
