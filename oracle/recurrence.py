"""Per-row fp64 evaluation of the recurrences, from a score vector
(TEST INFRASTRUCTURE ONLY).

Every function takes the scores s[0..N) of ONE query against its visible keys
(and, where an output is formed, the value rows V[N, d]) and walks the keys in
order with Python loops, so each step can be read against the paper.  All
intermediate quantities are returned, not just the last.
"""
from __future__ import annotations

import math

import numpy as np


def sigmoid(x: float) -> float:
    """sigma(x) = 1/(1+e^{-x}) (Sec. III-B), evaluated on the side where the
    exponential is at most 1."""
    if x >= 0.0:
        return 1.0 / (1.0 + math.exp(-x))
    e = math.exp(x)
    return e / (1.0 + e)


def log_sigmoid(x: float) -> float:
    """ln sigma(x) without forming sigma(x) first (the logarithm of a weight
    that has rounded to 0 or 1 would lose the information the next step needs)."""
    if x >= 0.0:
        return -math.log1p(math.exp(-x))
    return x - math.log1p(math.exp(x))


def weights_sigmoid(s):
    """Boxed weight equation of Sec. III-B: w_1 = 1,
    w_i = sigma(s_i - s_{i-1} + ln w_{i-1}).  Returns (w, ln w)."""
    s = np.asarray(s, dtype=np.float64)
    w = np.empty_like(s)
    lnw = np.empty_like(s)
    for i in range(len(s)):
        if i == 0:
            w[i], lnw[i] = 1.0, 0.0
        else:
            x = s[i] - s[i - 1] + lnw[i - 1]
            w[i], lnw[i] = sigmoid(x), log_sigmoid(x)
    return w, lnw


def weights_rational(s):
    """Rational form of Sec. III-B: w_i = w_{i-1} / (w_{i-1} + e^{s_{i-1}-s_i}).
    Has an explicit division and overflows for large score drops; kept as a
    cross-check at moderate scores only."""
    s = np.asarray(s, dtype=np.float64)
    w = np.empty_like(s)
    for i in range(len(s)):
        if i == 0:
            w[i] = 1.0
        else:
            w[i] = w[i - 1] / (w[i - 1] + math.exp(s[i - 1] - s[i]))
    return w


def flashd_row(s, V):
    """Alg. 3 with the blend in the form of Sec. IV-A:
    o_i = o_{i-1} + (v_i - o_{i-1}) w_i.  Returns (o[N, d], w[N])."""
    V = np.asarray(V, dtype=np.float64)
    w, _ = weights_sigmoid(s)
    o = np.zeros_like(V)
    cur = np.zeros(V.shape[1])
    for i in range(len(w)):
        cur = cur + (V[i] - cur) * w[i]
        o[i] = cur
    return o, w


def flashd_row_two_products(s, V):
    """Alg. 3 with the blend as printed in the algorithm box:
    o_i = o_{i-1}(1 - w_i) + v_i w_i."""
    V = np.asarray(V, dtype=np.float64)
    w, _ = weights_sigmoid(s)
    o = np.zeros_like(V)
    cur = np.zeros(V.shape[1])
    for i in range(len(w)):
        cur = cur * (1.0 - w[i]) + V[i] * w[i]
        o[i] = cur
    return o


def fa1_row(s, V):
    """Alg. 1: m_i = max(m_{i-1}, s_i), l_i = l_{i-1}e^{m_{i-1}-m_i} + e^{s_i-m_i},
    o_i = o_{i-1} (l_{i-1}e^{m_{i-1}-m_i}/l_i) + v_i (e^{s_i-m_i}/l_i).
    Returns every o_i, plus the weight e^{s_i-m_i}/l_i of Sec. III-A."""
    s = np.asarray(s, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    m, l = -math.inf, 0.0
    cur = np.zeros(V.shape[1])
    o = np.zeros_like(V)
    w = np.empty_like(s)
    for i in range(len(s)):
        mn = max(m, s[i])
        carry = l * math.exp(m - mn)
        fresh = math.exp(s[i] - mn)
        ln = carry + fresh
        cur = cur * (carry / ln) + V[i] * (fresh / ln)
        w[i] = fresh / ln
        o[i] = cur
        m, l = mn, ln
    return o, w


def fa2_row(s, V):
    """Alg. 2: unnormalised accumulation, Attn = o_N / l_N."""
    s = np.asarray(s, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    m, l = -math.inf, 0.0
    cur = np.zeros(V.shape[1])
    for i in range(len(s)):
        mn = max(m, s[i])
        resc = math.exp(m - mn)
        fresh = math.exp(s[i] - mn)
        l = l * resc + fresh
        cur = cur * resc + V[i] * fresh
        m = mn
    return cur / l


# ---------------------------------------------------------------------------
# Group-lifted recurrence and the merge of two partial states.
#
# The paper gives no block form of Alg. 3.  The state after a run of keys is
# (o, s_last, ln w_last); only Lambda = s_last - ln w_last enters later steps
# (the weight equation uses s_i - (s_{i-1} - ln w_{i-1})), and from the first
# recursive relation of Sec. III-B, e^{s_i}/w_i = e^{s_{i-1}}/w_{i-1} + e^{s_i},
# Lambda_i = ln sum_{j<=i} e^{s_j}.  A group G of keys therefore acts as one
# key with score S_G = ln sum_{j in G} e^{s_j} and value
# v_G = sum_{j in G} e^{s_j - S_G} v_j, which is itself the result of running
# Alg. 3 over the group alone.  A state is the pair (o, Lambda); the empty
# state is (0, -inf).
# ---------------------------------------------------------------------------

EMPTY_LAMBDA = -math.inf


def state_of_run(s, V):
    """State (o, Lambda) after Alg. 3 over the keys of one run, carried as
    (s_last, ln w_last) exactly as the algorithm does."""
    s = np.asarray(s, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    if len(s) == 0:
        return np.zeros(V.shape[1]), EMPTY_LAMBDA
    o, _ = flashd_row(s, V)
    _, lnw = weights_sigmoid(s)
    return o[-1], s[-1] - lnw[-1]


def merge(state_a, state_b):
    """Append run B after run A: B acts as one key of score Lambda_B and value
    o_B, so W = sigma(Lambda_B - Lambda_A) (weight equation with
    s_{i-1} - ln w_{i-1} = Lambda_A), o = o_A + (o_B - o_A) W, and the new
    Lambda = Lambda_B - ln W."""
    oa, la = state_a
    ob, lb = state_b
    if lb == EMPTY_LAMBDA:
        return oa, la
    if la == EMPTY_LAMBDA:
        return ob, lb
    x = lb - la
    W = sigmoid(x)
    return oa + (ob - oa) * W, lb - log_sigmoid(x)


def grouped_row(s, V, bounds):
    """Alg. 3 lifted to groups: bounds = [0, b1, b2, ..., N] cuts the keys into
    consecutive groups; each group is reduced on its own and the group states
    are merged left to right."""
    V = np.asarray(V, dtype=np.float64)
    st = (np.zeros(V.shape[1]), EMPTY_LAMBDA)
    for a, b in zip(bounds[:-1], bounds[1:]):
        st = merge(st, state_of_run(s[a:b], V[a:b]))
    return st


# ---------------------------------------------------------------------------
# Static skip rule of Sec. III-C (an approximation, reported as statistics
# only): outside [-6, 11] the weight is not computed.
# ---------------------------------------------------------------------------

SKIP_LOW, SKIP_HIGH = -6.0, 11.0


def skip_counts(s):
    """(#steps with s_i - s_{i-1} <= -6, #steps with s_i - s_{i-1} >= 11,
    #steps), over i = 2..N."""
    s = np.asarray(s, dtype=np.float64)
    dlt = np.diff(s)
    return int(np.sum(dlt <= SKIP_LOW)), int(np.sum(dlt >= SKIP_HIGH)), int(len(dlt))
