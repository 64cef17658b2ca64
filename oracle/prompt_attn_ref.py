"""Dense causal attention over a prompt, in fp64 -- TEST INFRASTRUCTURE ONLY.

What the model's own attention pass over the prompt computes (Eq.1 applied to every prompt position, with the
convention that a token attends to itself), written as its textbook definition: logits, causal mask, softmax,
weighted sum of values.  Also returns the natural-log sum of exponentials of every row, the quantity from which
the window rows' weights (Eq.4) are recovered without a second normalisation pass.

Only tests and the benchmark's checks may import this; it imports nothing from the product package.
"""
from __future__ import annotations

import numpy as np


def prompt_attention(Q, K, V, N: int, scale: float | None = None):
    """Q [M, >=N, d]; K, V [M', >=N, d] (query head h reads KV head h // (M / M')); first N rows are the prompt.

    Returns (O [M, N, d], lse [M, N]) as float64:
      l[h, i, k] = scale * Q[h, i] . K[h // G, k]        for k <= i      (causal, self included)
      lse[h, i]  = log sum_k exp l[h, i, k]
      O[h, i]    = sum_k exp(l[h, i, k] - lse[h, i]) V[h // G, k]
    """
    Q = np.asarray(Q, dtype=np.float64)[:, :N]
    K = np.asarray(K, dtype=np.float64)[:, :N]
    V = np.asarray(V, dtype=np.float64)[:, :N]
    M, _, d = Q.shape
    G = M // K.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    O = np.empty((M, N, d))
    lse = np.empty((M, N))
    future = np.arange(N)[None, :] > np.arange(N)[:, None]       # [query i, key k]: k > i
    for h in range(M):
        l = (Q[h] @ K[h // G].T) * scale
        l[future] = -np.inf
        m = l.max(axis=1, keepdims=True)
        e = np.exp(l - m)
        z = e.sum(axis=1, keepdims=True)
        O[h] = (e / z) @ V[h // G]
        lse[h] = (m + np.log(z))[:, 0]
    return O, lse
