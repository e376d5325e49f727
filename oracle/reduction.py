"""CPU oracle for the reduction schedule template (the second of the two templates the paper builds:
sum-like reductions along the last axis; end of Section 5) and for the row softmax that joins the two
attention products of the transformer workloads into attention.

TEST INFRASTRUCTURE ONLY, like the rest of this package.  Plain definitions in float64:

* ``reduce_rows``: y[i] = sum_j x[i][j] (``math.fsum``: the correctly rounded exact sum), max_j, or the mean.
* ``softmax_rows``: y[i][j] = exp(x[i][j] - m_i) / sum_j exp(x[i][j] - m_i), m_i = max_j x[i][j]; the
  subtraction of m_i is part of the definition used by every framework (it changes nothing
  mathematically and keeps exp in range).
* ``attention``: softmax(alpha * Q.K^T) . V per batch entry, composed from the definitions above and
  numpy's matmul.
"""
import math

import numpy as np

SUM, MAX, MEAN = 0, 1, 2


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def reduce_rows(x, op=SUM):
    x = _f64(x)
    rows, cols = x.shape
    out = np.empty(rows, dtype=np.float64)
    for i in range(rows):
        if op == MAX:
            out[i] = x[i].max() if cols else -np.inf
        else:
            s = math.fsum(x[i].tolist())
            out[i] = s if op == SUM else (s / cols if cols else np.nan)
    return out


def softmax_rows(x):
    x = _f64(x)
    out = np.empty_like(x)
    for i in range(x.shape[0]):
        if x.shape[1] == 0:
            continue
        m = x[i].max()
        e = np.exp(x[i] - m)
        out[i] = e / math.fsum(e.tolist())
    return out


def attention(Q, K, V, alpha):
    """Q, K, V: [batch, seq, d] -> softmax(alpha * Q K^T) V, [batch, seq, d]."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    out = np.empty_like(Q)
    for b in range(Q.shape[0]):
        out[b] = softmax_rows(alpha * (Q[b] @ K[b].T)) @ V[b]
    return out
