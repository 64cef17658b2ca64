"""Lock-step GPU-vs-oracle driver used by the GPU parity tests, the smoke check and nothing else.

Selection is chaotic after one divergent eviction, so both sides run the same steps on the same
seeded inputs and are compared every step:
  * attention output: max abs error within tolerance (2e-3 for bf16 inputs, 1e-5 for fp32);
  * evicted position: identical, or -- the only exemption -- a near-tie at the top-C boundary,
    where the oracle's own fp64 scores of the two choices differ by less than 1e-5 relative (and
    do differ); the oracle then adopts the GPU's choice (so the runs stay comparable) and the
    event is counted.  Where the oracle's two scores are EQUAL the choice is fixed by the tie
    rule (the lower position is kept) and any other choice fails the step;
  * retained sets: compared in full every `check_every` steps and at the end.
The oracle may cover only a sample of the sequences (batch_index) when the full batch is too slow
for the host; the GPU always runs the full configuration.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

from oracle import ref as oref
from paper_2503_00979_amd import binding

NEAR_TIE_REL = 1e-5
OUT_TOL = {"bf16": 2e-3, "f32": 1e-5}


@dataclass
class Report:
    steps: int = 0
    near_ties_prefill: int = 0
    near_ties_decode: int = 0
    exact_ties_prefill: int = 0   # units whose C-th largest prompt score is shared by several candidates
    exact_ties_decode: int = 0    # selections whose boundary score is shared by several candidates (the tie rule decided)
    max_out_err: float = 0.0
    max_score_rel_err: float = 0.0
    evictions: int = 0
    notes: List[str] = field(default_factory=list)


def _unit_map(wl, batch_index):
    """oracle unit -> GPU unit"""
    m = []
    for l in range(wl.n_layers):
        for b in batch_index:
            for h in range(wl.n_kv_heads):
                m.append((l * wl.batch + b) * wl.n_kv_heads + h)
    return np.array(m)


def _gpu_sets(gpu, wl, umap):
    """Per unit: the sorted positions of the older tokens and of the window's, from the exported slot positions.  A
    token is in the window if it is among the R most recent positions of its sequence; slots are in no particular
    order and -1 where free."""
    pos, n_snap = gpu.export_positions()
    pos = pos.cpu().numpy()[umap]
    n_snap = n_snap.cpu().numpy()[umap]
    snaps, wins = [], []
    for i in range(len(umap)):
        held = pos[i][pos[i] >= 0]
        assert len(np.unique(held)) == len(held), "a position is held twice"
        held = np.sort(held)
        last = held[-1]
        w = held[held > last - wl.R]
        assert len(w) == min(wl.R, last + 1) and w[0] == last - len(w) + 1, "the window must hold the R most recent positions"
        s = held[held <= last - wl.R]
        assert len(s) == n_snap[i], "exported count of older tokens"
        snaps.append(s)
        wins.append(w)
    return snaps, wins, pos


def window_lse(wl, Qw, K):
    """Natural-log sum of exp of the window rows' causal logits, [L, B, M, R] fp32, with torch in fp64: what the
    caller's own attention pass over the prompt would hand over."""
    L, B, M, R, d = Qw.shape
    G = wl.n_q_heads // wl.n_kv_heads
    out = torch.zeros(L, B, M, R, dtype=torch.float64)
    for b in range(B):
        N = wl.prompt_lens[b]
        Rw = min(R, N)
        q = Qw[:, b, :, :Rw].double().cpu()                               # [L, M, Rw, d]
        k = K[:, b, :, :N].double().cpu().repeat_interleave(G, dim=1)     # [L, M, N, d]
        logits = torch.einsum("lmjd,lmnd->lmjn", q, k) / d ** 0.5
        pj = torch.arange(N - Rw, N)[:, None]
        logits = logits.masked_fill(torch.arange(N)[None, :] > pj, float("-inf"))
        out[:, b, :, :Rw] = torch.logsumexp(logits, -1)
    return out.float()


class LockStep:
    def __init__(self, wl, device="cuda:0", batch_index: Optional[List[int]] = None, gen_device=None,
                 capture_scores=False, per_layer=False, use_lse=False, use_attend=False):
        self.wl = wl
        self.device = device
        self.bidx = list(range(wl.batch)) if batch_index is None else list(batch_index)
        self.wl_o = wl.with_batch_subset(self.bidx)
        self.umap = _unit_map(wl, self.bidx)
        self.gen_device = gen_device or "cpu"
        self.gpu = binding.MorphKV.from_workload(wl, device)
        self.oracle = oref.RefMorphKV.from_workload(self.wl_o)
        self.rep = Report()
        self.tol = OUT_TOL[wl.dtype]
        self.scoreF = self.gpu.capture_scores(True) if capture_scores else None
        self.t = 0
        self.use_lse = use_lse       # prefill through the variant that takes the rows' log-sum-exp from the caller
        self.use_attend = use_attend  # prefill through the entry that also runs the prompt's attention pass
        self.attn_out = None          # (Q, O, lse) of that pass, for the caller to check
        self.per_layer = per_layer   # one call per layer (reverse order, to show the calls are independent)

    # ---- prefill --------------------------------------------------------
    def prefill(self):
        wl, rep = self.wl, self.rep
        Qw, K, V = wl.prompt(self.gen_device)
        plen = wl.prompt_len_tensor().numpy()
        lse = window_lse(wl, Qw, K).to(self.device) if self.use_lse else None
        if self.use_attend:
            Q = wl.prompt_queries(self.gen_device).to(self.device)
            lse_all = torch.full(Q.shape[:-1], float("nan"), dtype=torch.float32, device=self.device)
            O = torch.full_like(Q, float("nan"))
            self.gpu.prefill_attend_select(Q, K.to(self.device), V.to(self.device), plen, O=O, lse=lse_all)
            self.attn_out = (Q, O, lse_all)
        else:
            self.gpu.prefill_select(Qw.to(self.device), K.to(self.device), V.to(self.device), plen, lse_window=lse)
        ix = torch.tensor(self.bidx, device=Qw.device)
        Qo, Ko, Vo = (t.index_select(1, ix).cpu().contiguous() for t in (Qw, K, V))
        del Qw, K, V
        plo = self.wl_o.prompt_len_tensor().numpy()
        self.oracle.prefill_select(Qo, Ko, Vo, plo)
        gs, gw, _ = _gpu_sets(self.gpu, wl, self.umap)
        os_, ow = self.oracle.export_positions()
        forced = None
        for i in range(len(self.umap)):
            assert list(gw[i]) == list(ow[i]), f"window differs after prefill, unit {i}"
            F = self.oracle.prefill_scores(i)
            kth = None
            if len(F) > wl.C:
                kth = np.sort(F)[::-1][wl.C - 1]
                rep.exact_ties_prefill += int(np.count_nonzero(F == kth) > 1)
            if list(gs[i]) == list(os_[i]):
                continue
            assert kth is not None, f"prefill unit {i}: retained sets differ although every older token fits"
            # near-tie exemption: every element of the symmetric difference scores within 1e-5 relative
            # of the C-th largest oracle score -- and not exactly at it: equal scores are decided by position
            diff = set(gs[i]) ^ set(os_[i])
            assert len(gs[i]) == len(os_[i])
            for k in diff:
                assert abs(F[k] - kth) <= NEAR_TIE_REL * abs(kth), (
                    f"prefill selection differs beyond a near-tie: unit {i} pos {k} F={F[k]!r} C-th={kth!r}")
            lost, won = sorted(set(os_[i]) - set(gs[i])), sorted(set(gs[i]) - set(os_[i]))
            for a in lost:
                for b_ in won:
                    assert F[a] != F[b_], (
                        f"prefill unit {i}: positions {a} and {b_} have EQUAL scores {F[a]!r}; the tie rule keeps the "
                        f"lower position, the GPU kept {b_}")
            rep.near_ties_prefill += len(diff) // 2
            if forced is None:
                forced = np.full((len(self.umap), wl.C), -1, np.int32)
                for x in range(len(self.umap)):
                    forced[x, :len(os_[x])] = os_[x]
            forced[i, :] = -1
            forced[i, :len(gs[i])] = gs[i]
        if forced is not None:
            self.oracle.prefill_select(Qo, Ko, Vo, plo, forced_pos=forced)
            os_, _ = self.oracle.export_positions()
            for i in range(len(self.umap)):
                assert list(gs[i]) == list(os_[i])
        return self

    # ---- one decode step ------------------------------------------------
    def step(self, check_sets=False):
        wl, rep, t = self.wl, self.rep, self.t
        q, k, v = wl.decode_inputs(t, self.gen_device)
        pos_before = None
        if self.scoreF is not None:
            pos_before = self.gpu.export_positions()[0].cpu().numpy()[self.umap]
        qd, kd, vd = q.to(self.device), k.to(self.device), v.to(self.device)
        if self.per_layer:
            out = torch.full(self.gpu.out_shape, float("nan"), dtype=torch.float32, device=self.device)
            for l in reversed(range(wl.n_layers)):
                self.gpu.decode_step_layer(l, qd[l], kd[l], vd[l], out[l])
        else:
            out = self.gpu.decode_step(qd, kd, vd)
        T = wl.evict_every
        if T > 1:
            return self._finish_step_multi(q, k, v, out, check_sets)
        ev = self.gpu.export_evicted().cpu().numpy()[self.umap]
        ix = torch.tensor(self.bidx, device=q.device)
        qo, ko, vo = (x.index_select(1, ix).cpu().contiguous() for x in (q, k, v))
        oout = self.oracle.decode_begin(qo, ko, vo)
        n_cand, cand_pos, cand_F, n_evict, choice = self.oracle.candidates()
        gout = out.index_select(1, torch.tensor(self.bidx, device=out.device)).cpu().numpy().astype(np.float64)
        err = float(np.max(np.abs(gout - oout)))
        rep.max_out_err = max(rep.max_out_err, err)
        assert err <= self.tol, f"step {t}: attention output off by {err:.3e} (> {self.tol})"
        decided = np.full(len(self.umap), -1, np.int32)
        Fg_all = self.scoreF.cpu().numpy() if self.scoreF is not None else None
        for i in range(len(self.umap)):
            if n_evict[i] == 0:
                assert ev[i] == -1, f"step {t} unit {i}: GPU evicted {ev[i]} where nothing may be evicted"
                continue
            rep.evictions += 1
            nc = int(n_cand[i])
            cp, cF = cand_pos[i, :nc], cand_F[i, :nc]
            e_or, e_gpu = int(choice[i, 0]), int(ev[i])
            F_or = cF[np.nonzero(cp == e_or)[0][0]]
            rep.exact_ties_decode += int(np.count_nonzero(cF == F_or) > 1)
            if e_gpu != e_or:
                hit = np.nonzero(cp == e_gpu)[0]
                assert len(hit) == 1, f"step {t} unit {i}: GPU evicted {e_gpu}, not a candidate"
                F_gpu = cF[hit[0]]
                gap = F_gpu - F_or
                assert gap != 0, (
                    f"step {t} unit {i}: positions {e_gpu} and {e_or} have EQUAL scores {F_or!r}; the tie rule evicts "
                    f"the higher position ({e_or}), the GPU evicted {e_gpu}")
                assert gap <= NEAR_TIE_REL * abs(F_or), (
                    f"step {t} unit {i}: GPU evicted {e_gpu} (F={F_gpu!r}), oracle {e_or} (F={F_or!r}): "
                    f"not a near-tie")
                rep.near_ties_decode += 1
            decided[i] = e_gpu
            if Fg_all is not None:
                # captured GPU scores are in slot order: look each candidate slot's position up among the oracle's
                Fg = Fg_all[self.umap[i]]
                pb = pos_before[i]
                slots = np.nonzero((pb >= 0) & (pb <= cp.max()))[0]
                assert np.array_equal(np.sort(pb[slots]), np.sort(cp)), "candidates differ"
                order = np.argsort(cp)
                at = order[np.searchsorted(cp[order], pb[slots])]
                rel = np.abs(Fg[slots] - cF[at]) / np.maximum(np.abs(cF[at]), 1e-30)
                rep.max_score_rel_err = max(rep.max_score_rel_err, float(rel.max()))
        self.oracle.decode_commit(decided)
        self.t += 1
        rep.steps += 1
        if check_sets:
            self.check_sets()

    def _finish_step_multi(self, q, k, v, out, check_sets):
        """Coarse schedule (several evictions at once): the evicted SETS must agree; where they differ every
        element of the symmetric difference must score within 1e-5 relative of the boundary (the largest
        score the oracle evicts), and the oracle then adopts the GPU's set."""
        wl, rep, t, T = self.wl, self.rep, self.t, self.wl.evict_every
        evl = self.gpu.export_evicted_list().cpu().numpy()[self.umap]
        ix = torch.tensor(self.bidx, device=q.device)
        qo, ko, vo = (x.index_select(1, ix).cpu().contiguous() for x in (q, k, v))
        oout = self.oracle.decode_begin(qo, ko, vo)
        n_cand, cand_pos, cand_F, n_evict, choice = self.oracle.candidates()
        gout = out.index_select(1, torch.tensor(self.bidx, device=out.device)).cpu().numpy().astype(np.float64)
        err = float(np.max(np.abs(gout - oout)))
        rep.max_out_err = max(rep.max_out_err, err)
        assert err <= self.tol, f"step {t}: attention output off by {err:.3e} (> {self.tol})"
        decided = np.full((len(self.umap), T), -1, np.int32)
        for i in range(len(self.umap)):
            g_set = set(int(x) for x in evl[i] if x >= 0)
            if n_evict[i] == 0:
                assert not g_set, f"step {t} unit {i}: GPU evicted {g_set} where nothing may be evicted"
                continue
            rep.evictions += int(n_evict[i])
            o_set = set(int(x) for x in choice[i, :n_evict[i]])
            assert len(g_set) == n_evict[i], f"step {t} unit {i}: GPU evicted {len(g_set)} tokens, {n_evict[i]} are due"
            F = {int(cand_pos[i, x]): cand_F[i, x] for x in range(n_cand[i])}
            bound = max(F[e] for e in o_set)
            rep.exact_ties_decode += int(sum(1 for f in F.values() if f == bound) > sum(1 for e in o_set if F[e] == bound))
            if g_set != o_set:
                for e in g_set ^ o_set:
                    assert e in F, f"step {t} unit {i}: {e} is not a candidate"
                    assert abs(F[e] - bound) <= NEAR_TIE_REL * abs(bound), (
                        f"step {t} unit {i}: evicted sets differ beyond a near-tie at {e}: F={F[e]!r} boundary={bound!r}")
                for a in g_set - o_set:
                    for b_ in o_set - g_set:
                        assert F[a] != F[b_], (
                            f"step {t} unit {i}: positions {a} and {b_} have EQUAL scores {F[a]!r}; the tie rule evicts "
                            f"the higher position ({b_}), the GPU evicted {a}")
                rep.near_ties_decode += len(g_set - o_set)
            decided[i, :len(g_set)] = sorted(g_set)
        self.oracle.decode_commit(decided)
        self.t += 1
        rep.steps += 1
        if check_sets:
            self.check_sets()

    def check_sets(self):
        gs, gw, _ = _gpu_sets(self.gpu, self.wl, self.umap)
        os_, ow = self.oracle.export_positions()
        for i in range(len(self.umap)):
            assert list(gw[i]) == list(ow[i]), f"step {self.t}: window differs, unit {i}"
            assert list(gs[i]) == list(os_[i]), f"step {self.t}: retained older tokens differ, unit {i}"

    def run(self, steps, check_every=16):
        for s in range(steps):
            self.step(check_sets=((s + 1) % check_every == 0) or s == steps - 1)
        return self.rep
