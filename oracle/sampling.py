"""Oracle: speculative sampling primitives (test infrastructure only).

Section 2 of the paper: draft tokens x_i ~ q_i, acceptance probability
alpha_i = min(1, p_i[x_i] / q_i[x_i]) (Eq. 1), and on rejection a token drawn from
norm(max(0, p_i - q_i)); Algorithm 2 draws r ~ U(0,1) and accepts iff r <= p[x]/q[x].

Readings the paper leaves open:
  * a draw from a distribution is an inverse-CDF walk in ascending token id with one
    uniform u: the smallest k with sum_{j<=k} w_j > u * sum_j w_j (sums in float64);
  * the test is done without dividing: accept iff r * q[x] <= p[x];
  * temperature 0 (greedy) replaces a distribution by the one-hot at its arg-max
    (lowest id on ties), which turns the rule into "accept iff x == argmax p";
  * if the residual has no mass in floating point, the draw falls back to p.
"""
from __future__ import annotations

import numpy as np


def probs(logits, temperature: float, logit_scale: float = 1.0) -> np.ndarray:
    """softmax(logit_scale * logits / temperature) over the last axis; one-hot arg-max if temperature == 0."""
    x = np.asarray(logits)
    if temperature == 0.0:
        out = np.zeros_like(x)
        idx = np.argmax(x, axis=-1)                     # first maximum = lowest id
        np.put_along_axis(out, np.expand_dims(idx, -1), 1.0, axis=-1)
        return out
    z = x * x.dtype.type(logit_scale / temperature)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def sample(weights, u: float) -> int:
    """Inverse-CDF draw from unnormalised non-negative weights with one uniform u in [0,1)."""
    w = np.asarray(weights, dtype=np.float64)
    cdf = np.cumsum(w)
    total = cdf[-1]
    if not total > 0.0:
        raise ValueError("cannot sample from zero mass")
    k = int(np.searchsorted(cdf, np.float64(u) * total, side="right"))   # first k with cdf[k] > u*total
    last = int(np.nonzero(w > 0.0)[0][-1])
    return min(k, last)


def accept(p_row, q_row, x: int, r: float) -> bool:
    """Acceptance test of Eq. (1): keep draft token x iff r <= p[x]/q[x], evaluated as r*q[x] <= p[x]."""
    return bool(np.float64(r) * np.float64(q_row[x]) <= np.float64(p_row[x]))


def residual(p_row, q_row) -> np.ndarray:
    """Unnormalised max(0, p - q)."""
    return np.maximum(np.asarray(p_row, dtype=np.float64) - np.asarray(q_row, dtype=np.float64), 0.0)


def resample(p_row, q_row, u: float) -> int:
    """Draw the replacement token from norm(max(0, p - q)); from p itself if that has no mass."""
    res = residual(p_row, q_row)
    if res.sum() > 0.0:
        return sample(res, u)
    return sample(p_row, u)


def sample_margin(weights, u: float) -> float:
    """How far u is from flipping an inverse-CDF draw: distance of u*total to the nearest CDF edge, over total."""
    cdf = np.cumsum(np.asarray(weights, dtype=np.float64))
    return float(np.min(np.abs(cdf / cdf[-1] - np.float64(u))))


def accept_margin(p_row, q_row, x: int, r: float) -> float:
    """How far an acceptance test is from flipping: |r q[x] - p[x]| / max(r q[x], p[x])."""
    lhs, rhs = np.float64(r) * np.float64(q_row[x]), np.float64(p_row[x])
    top = max(lhs, rhs)
    return float(abs(lhs - rhs) / top) if top > 0 else 1.0
