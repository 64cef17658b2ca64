"""The incremental score state of the decode step, emulated in numpy and checked against naive re-fusion (Eq.4-6).

The kernels never re-read the R recorded rows: every cache slot is a column with an old part (one stored row of
suffix aggregates, rebuilt when the column's turn comes, once in R steps) and a new part (a running aggregate since
that turn), and no token ever changes its slot -- a new token is written into the slot an eviction has freed, whose
column still holds the former occupant's numbers.  Three rules make those harmless: rows of queries up to a token's
own position count as zero where a column is rebuilt; the stored new part of a column born at the previous step is
ignored; the stored old part of a column whose last turn was before its birth is ignored.  This file restates that
scheme (it shares no code with the library or with the oracle) and shows, for sum and max fusion, random weights,
random evictions, every-step and coarse schedules, that the score it gives for EVERY held token at EVERY step is the
aggregate over the window's rows recorded since the token's birth."""
import numpy as np
import pytest


def fuse(f, a, b):
    return a + b if f == "sum" else max(a, b)


class Scheme:
    def __init__(self, C, R, T, fusion, N, rng):
        self.C, self.R, self.T, self.f, self.rng = C, R, T, fusion, rng
        self.Cs = C + T - 1
        self.n = self.Cs + R
        self.cps = -(-self.n // R)                     # columns rebuilt per step: every column once in R steps
        self.pos = np.full(self.n, -1)
        self.ring = np.zeros((R, self.n))              # recorded rows, row = query position mod R
        self.sfx = rng.random((R, self.n))             # garbage where nothing was ever stored: must never be read
        self.nw = rng.random(self.n)
        self.holes = []
        self.hist = {}                                 # (slot, query position) -> weight of the slot's PRESENT token
        # the prompt: the last min(R, N) tokens and up to C older ones, packed into the first slots
        Rw = min(R, N)
        older = sorted(rng.choice(N - Rw, size=min(C, N - Rw), replace=False)) if N > Rw else []
        held = list(older) + list(range(N - Rw, N))
        self.n_used = len(held)
        self.pos[:self.n_used] = held
        for t in range(N - Rw, N):                     # rows of the window's queries: later tokens get nothing
            for j in range(self.n_used):
                if self.pos[j] < t:                    # a token's rows are those of LATER queries
                    self.ring[t % R, j] = self.hist[(j, t)] = rng.random()
        self.p = self.N0 = N
        for c in range(self.n_used):                   # state as of the end of step N-1
            self.scan(c, N - 1, self.last_turn_before(N - 1, c))

    def phase(self, c):
        return c // self.cps

    def last_turn_before(self, p, c):                  # most recent step p0 < p with p0 mod R == phase(c)
        return p - 1 - ((p - 1 - self.phase(c)) % self.R)

    def value(self, c, t):                             # row of query t in column c, zero up to the token's own position
        if t < 0 or self.pos[c] < 0 or t <= self.pos[c]:
            return 0.0
        return self.ring[t % self.R, c]

    def scan(self, c, p_end, p0):
        """old part for every future step that still needs rows <= p0, new part = rows p0+1 .. p_end"""
        nw = 0.0
        for t in range(p0 + 1, p_end + 1):
            nw = fuse(self.f, nw, self.value(c, t))
        acc = 0.0
        for t in range(p0, p_end - self.R + 1, -1):    # t = p0 .. p_end-R+2
            acc = fuse(self.f, acc, self.value(c, t))
            self.sfx[(t - 1) % self.R, c] = acc
        self.sfx[p0 % self.R, c] = 0.0
        self.nw[c] = nw

    def step(self):
        R, p, f = self.R, self.p, self.f
        w, wm1 = p % R, (p - 1) % R
        for c in range(wm1 * self.cps, min((wm1 + 1) * self.cps, self.n_used)):   # this step's turn columns
            self.scan(c, p - 1, p - 1)
        S = np.where(self.pos >= 0, self.rng.random(self.n), 0.0)                 # the new query's group-summed weights
        self.ring[w, :] = S
        F = {}
        for j in range(self.n_used):
            if self.pos[j] < 0:
                continue
            self.hist[(j, p)] = S[j]
            d = (wm1 - self.phase(j)) % R              # steps since the column's last turn
            age = p - 1 - self.pos[j]                  # rows recorded since the token's birth, before this one
            old = 0.0 if d > age else self.sfx[w, j]
            new_before = 0.0 if self.pos[j] == p - 1 else self.nw[j]
            self.nw[j] = fuse(f, new_before, S[j])
            F[j] = fuse(f, old, self.nw[j])
            naive = 0.0
            for t in range(max(p - R + 1, self.pos[j] + 1), p + 1):
                naive = fuse(f, naive, self.hist[(j, t)])
            if f == "max":
                assert F[j] == naive, (p, j)
            else:
                assert abs(F[j] - naive) <= 1e-12 * max(1.0, naive), (p, j, F[j], naive)
        # who goes: any candidate will do for this check (the scheme must be right whoever is evicted)
        tokens = self.n_used - len(self.holes)
        older = tokens + 1 - min(R, p + 1)
        cand = [j for j in range(self.n_used) if 0 <= self.pos[j] <= p - R]
        assert len(cand) == max(older, 0)
        gen_step = p - self.N0 + 1
        if self.T > 1:
            if gen_step % self.T == 0 and older > self.C:
                out = list(self.rng.choice(cand, size=older - self.C, replace=False))
                for j in out:
                    self.drop(j)
                dest, self.holes = out[0], self.holes + out[1:]
            elif self.holes:
                dest = self.holes.pop()
            else:
                dest, self.n_used = self.n_used, self.n_used + 1
        elif older > self.Cs:
            dest = int(self.rng.choice(cand))
            self.drop(dest)
        else:
            dest, self.n_used = self.n_used, self.n_used + 1
        assert dest < self.n and self.pos[dest] < 0
        self.pos[dest] = p                             # nothing else is written for the new token
        self.p += 1

    def drop(self, j):
        self.pos[j] = -1
        for key in [k for k in self.hist if k[0] == j]:
            del self.hist[key]


CASES = [(8, 4, 1, 20), (5, 3, 1, 4), (16, 8, 1, 40), (7, 5, 1, 5), (3, 8, 1, 30), (9, 1, 1, 12), (1, 5, 1, 9),
         (16, 4, 1, 5), (6, 4, 3, 25), (10, 8, 8, 30), (4, 3, 2, 2), (12, 16, 4, 7)]


@pytest.mark.parametrize("fusion", ["sum", "max"])
@pytest.mark.parametrize("case", CASES, ids=["C%d_R%d_T%d_N%d" % c for c in CASES])
def test_incremental_state_equals_naive_fusion(case, fusion):
    C, R, T, N = case
    rng = np.random.default_rng(1000 * C + 10 * R + T)
    s = Scheme(C, R, T, fusion, N, rng)
    steps = 6 * R + 3 * C + 20
    for _ in range(steps):
        s.step()
    assert s.p == N + steps and s.n_used <= s.n
