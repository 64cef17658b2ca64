"""Definitional brute force used to pin the oracle's bookkeeping on tiny inputs.

It keeps the whole K/V history, a dict ``W[(query_pos, key_pos)]`` of every
group-summed attention weight ever computed, and a plain Python set of the
older tokens that are resident.  There are no slots, no ring, no column moves:
every step it looks the R window queries' weights up in the dict, fuses them
(Eq.5 / Eq.6) and keeps the top-C older tokens (Eq.7), ties keeping the lower
position.  numpy fp64; one instance per unit.
"""
from __future__ import annotations

import numpy as np


def _softmax_weights(qs: np.ndarray, keys: np.ndarray, scale: float) -> np.ndarray:
    """qs [G,d], keys [n,d] -> weights [G,n] (Eq.1)."""
    lg = (qs @ keys.T) * scale
    lg = lg - lg.max(axis=1, keepdims=True)
    e = np.exp(lg)
    return e / e.sum(axis=1, keepdims=True)


class BruteForceUnit:
    def __init__(self, C: int, R: int, fusion: str, scale: float, evict_every: int = 1):
        self.C, self.R, self.fusion, self.scale, self.T = C, R, fusion, scale, evict_every
        self.K = []            # every key ever seen, by position
        self.V = []
        self.W = {}            # (query position, key position) -> group-summed weight
        self.old = set()       # resident older tokens
        self.last_scores = {}  # candidate position -> fused score, of the last selection

    def _fuse(self, vals):
        return float(max(vals)) if self.fusion == "max" else float(sum(vals))

    def _select(self, cands, queries):
        if self.fusion == "cumsum":  # comparison policy: every weight later queries gave the token, no window
            queries = None
        F = {k: (self._fuse([self.W[(t, k)] for t in queries]) if queries is not None else
                 float(sum(w for (t, kk), w in self.W.items() if kk == k and t > k))) for k in cands}
        self.last_scores = F
        order = sorted(cands, key=lambda k: (-F[k], k))
        return set(order[: self.C])

    def prefill(self, Qw: np.ndarray, K: np.ndarray, V: np.ndarray):
        """Qw [G,R,d] (row j = query of position N-min(R,N)+j), K,V [N,d]."""
        N = K.shape[0]
        self.N = N
        self.K = [K[i].astype(np.float64) for i in range(N)]
        self.V = [V[i].astype(np.float64) for i in range(N)]
        Rw = min(self.R, N)
        queries = list(range(N - Rw, N))
        for j, pj in enumerate(queries):
            w = _softmax_weights(Qw[:, j, :].astype(np.float64), np.stack(self.K[: pj + 1]), self.scale)
            for k in range(pj + 1):
                self.W[(pj, k)] = float(w[:, k].sum())
        cands = list(range(N - Rw))
        self.old = self._select(cands, queries) if len(cands) > self.C else set(cands)
        if len(cands) <= self.C:
            self.last_scores = {k: self._fuse([self.W[(t, k)] for t in queries]) for k in cands}

    def resident(self):
        p = len(self.K)
        return sorted(self.old | set(range(max(0, p - self.R), p)))

    def decode(self, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray) -> np.ndarray:
        """q [G,d]; returns out [G,d]."""
        p = len(self.K)
        res = self.resident()
        keys = np.stack([self.K[i] for i in res] + [k_new.astype(np.float64)])
        vals = np.stack([self.V[i] for i in res] + [v_new.astype(np.float64)])
        w = _softmax_weights(q.astype(np.float64), keys, self.scale)
        out = w @ vals
        for i, k in enumerate(res):
            self.W[(p, k)] = float(w[:, i].sum())
        self.K.append(k_new.astype(np.float64))
        self.V.append(v_new.astype(np.float64))
        if p - self.R >= 0:
            cands = sorted(self.old | {p - self.R})
            if self.T >= 1 and (p - self.N + 1) % self.T == 0 and len(cands) > self.C:   # T == 0: selection at the prompt only
                self.old = self._select(cands, list(range(p - self.R + 1, p + 1)))
            else:
                self.old = set(cands)
        return out
