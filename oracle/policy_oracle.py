"""CPU oracle for learning a sharing policy from attention weights (Sec. 3.3).

TEST INFRASTRUCTURE ONLY (same rules as san_oracle.py: plain numpy fp64, no code
shared with the HIP library, never imported by the product path).

  * JS divergence between the attention distributions of two layers, computed
    per head and averaged (Sec. 3.1);
  * similarity mu(i,j) = ln 2 - JS(i,j) (Sec. 3.3);
  * block similarity sim(m,n): the mean of mu over all ordered pairs i != j of
    the block b(m,n) (Eq. 6);
  * greedy search: starting from layer 1 take the biggest block whose similarity
    is at least theta, continue after it, until every layer is covered (Sec. 3.3).

Readings: natural logarithms (so JS <= ln 2 and mu >= 0, as "ln(2) - JS" needs;
two entries of the paper's Fig. 2(b) exceed ln 2, so that figure was not produced
with exactly this definition); 0 log 0 = 0; "biggest block that satisfies the
criterion" = the largest n >= m with sim(m,n) >= theta, a single layer always
qualifying.  Pins: tests/test_policy_oracle.py.
"""
from __future__ import annotations

import numpy as np

LN2 = float(np.log(2.0))


def kl(p, q):
    """sum_x p log(p/q) along the last axis, with 0 log 0 = 0."""
    p = np.asarray(p, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = np.where(p > 0, p * (np.log(p) - np.log(q)), 0.0)
    return t.sum(axis=-1)


def js_divergence(p, q):
    """Jensen-Shannon divergence of distributions along the last axis."""
    p = np.asarray(p, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    m = 0.5 * (p + q)
    return 0.5 * kl(p, m) + 0.5 * kl(q, m)


def layer_js_matrix(S_layers):
    """S_layers: list over layers of weights [rows, heads, keys] (each [row, head]
    slice a distribution).  Returns the [L, L] matrix of JS divergences, each the
    mean over rows and heads of the per-head divergence."""
    L = len(S_layers)
    out = np.zeros((L, L))
    for a in range(L):
        for b in range(a + 1, L):
            out[a, b] = out[b, a] = js_divergence(S_layers[a], S_layers[b]).mean()
    return out


def block_similarity(js, m, n):
    """Eq. 6 for the block of layers m..n (0-based, inclusive), n > m."""
    size = n - m + 1
    total = 0.0
    for i in range(m, n + 1):
        for j in range(m, n + 1):
            if i != j:
                total += LN2 - js[i][j]
    return total / (size * (size - 1))


def greedy_policy(js, theta):
    """Block sizes {pi_i}, bottom-up."""
    L = len(js)
    pi, m = [], 0
    while m < L:
        best = m
        for n in range(m + 1, L):
            if block_similarity(js, m, n) >= theta:
                best = n
        pi.append(best - m + 1)
        m = best + 1
    return pi
