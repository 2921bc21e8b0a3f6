"""Pure-Python brute force for tiny attention-variant problems.  TEST INFRASTRUCTURE ONLY.

Written separately from attention_oracle.py (nested loops over scalars, math.exp,
math.fsum, no NumPy arithmetic) so that an indexing, sign or ordering mistake in the
vectorised oracle shows up as a disagreement.  The softmax here is the *online*
recurrence of Alg. 2 (running max m_j and rescaled running sum d_j), while the NumPy
oracle uses the two-loop stable form of Alg. 1: their agreement is the post-condition
both algorithms assert (m_N = max x, d_N = sum e^{x_j - max x}) and the ds[N] = do[N]
statement of Sec. 3.3.
"""
from __future__ import annotations

import math


def online_softmax_state(xs):
    """Alg. 2: returns (m_N, d_N) for a sequence of scores; -inf entries allowed."""
    m = -math.inf
    d = 0.0
    for x in xs:
        m_new = x if x > m else m
        if m_new == -math.inf:
            continue                       # nothing visible yet: (m, d) stays (-inf, 0)
        d = d * math.exp(m - m_new) + math.exp(x - m_new)
        m = m_new
    return m, d


def attention_row(q_row, keys, values, *, scale, i, causal=False, window=None, prefix=None,
                  cap=None, slope=None, bias_row=None, q_doc=None, kv_doc=None):
    """One query row against all keys.  q_row [D], keys [Sk][D], values [Sk][Dv].

    Returns (out_row [Dv], lse, probs [Sk]).
    """
    Sk = len(keys)
    scores = []
    for j in range(Sk):
        s = scale * math.fsum(q_row[d] * keys[j][d] for d in range(len(q_row)))
        if cap is not None:
            s = cap * math.tanh(s / cap)
        if slope is not None:
            s = s - slope * abs(i - j)
        if bias_row is not None:
            s = s + bias_row[j]
        hidden = False
        if prefix is not None:
            hidden = hidden or (j > i and j >= prefix)
        elif causal or window is not None:
            hidden = hidden or j > i
        if window is not None:
            hidden = hidden or (i - j) > window
        if q_doc is not None:
            hidden = hidden or (q_doc != kv_doc[j])
        scores.append(-math.inf if hidden else s)
    m, d = online_softmax_state(scores)
    Dv = len(values[0])
    if m == -math.inf:
        return [0.0] * Dv, -math.inf, [0.0] * Sk
    probs = [math.exp(s - m) / d for s in scores]
    out = [math.fsum(probs[j] * values[j][c] for j in range(Sk)) for c in range(Dv)]
    return out, m + math.log(d), probs


def rmsnorm_row(x, eps, weight=None):
    ms = math.fsum(t * t for t in x) / len(x)
    r = 1.0 / math.sqrt(ms + eps)
    return [x[c] * r * (1.0 if weight is None else weight[c]) for c in range(len(x))]


def sigmoid(x):
    return 1.0 / (1.0 + math.exp(-x))
