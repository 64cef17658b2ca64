"""Lock-step GPU-vs-oracle driver used by the GPU parity tests, the smoke check and nothing else.

Selection is chaotic after one divergent eviction, so both sides run the same steps on the same
seeded inputs and are compared every step:
  * attention output: max abs error within tolerance (2e-3 for bf16 inputs, 1e-5 for fp32);
  * evicted position: identical, or -- the only exemption -- a near-tie at the top-C boundary,
    where the oracle's own fp64 scores of the two choices differ by less than 1e-5 relative; the
    oracle then adopts the GPU's choice (so the runs stay comparable) and the event is counted;
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
    pos, n_snap = gpu.export_positions()
    pos = pos.cpu().numpy()[umap]
    n_snap = n_snap.cpu().numpy()[umap]
    # older-token slots: more than C are held between coarse selections, or for good when selection is at the prompt only
    C = wl.C + (wl.evict_every - 1 if wl.evict_every >= 1 else wl.max_new_tokens)
    snaps, wins = [], []
    for i in range(len(umap)):
        s = pos[i, :C]
        assert np.all(s[n_snap[i]:] == -1), "unused older-token slots must be empty"
        assert np.all(s[:n_snap[i]] >= 0)
        snaps.append(np.sort(s[:n_snap[i]]))
        wv = pos[i, C:]
        for x, pv in enumerate(wv):
            assert pv == -1 or pv % wl.R == x, "window slot must be position mod R"
        wins.append(np.sort(wv[wv >= 0]))
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
            if list(gs[i]) == list(os_[i]):
                continue
            # near-tie exemption: every element of the symmetric difference scores within 1e-5 relative
            # of the C-th largest oracle score
            F = self.oracle.prefill_scores(i)
            kth = np.sort(F)[::-1][wl.C - 1]
            diff = set(gs[i]) ^ set(os_[i])
            assert len(gs[i]) == len(os_[i])
            for k in diff:
                assert abs(F[k] - kth) <= NEAR_TIE_REL * abs(kth), (
                    f"prefill selection differs beyond a near-tie: unit {i} pos {k} F={F[k]!r} C-th={kth!r}")
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
        for i in range(len(self.umap)):
            if n_evict[i] == 0:
                assert ev[i] == -1, f"step {t} unit {i}: GPU evicted {ev[i]} where nothing may be evicted"
                continue
            rep.evictions += 1
            e_or, e_gpu = int(choice[i, 0]), int(ev[i])
            F = {int(cand_pos[i, x]): cand_F[i, x] for x in range(n_cand[i])}
            if e_gpu != e_or:
                assert e_gpu in F, f"step {t} unit {i}: GPU evicted {e_gpu}, not a candidate"
                gap = F[e_gpu] - F[e_or]
                assert gap <= NEAR_TIE_REL * abs(F[e_or]), (
                    f"step {t} unit {i}: GPU evicted {e_gpu} (F={F[e_gpu]!r}), oracle {e_or} (F={F[e_or]!r}): "
                    f"not a near-tie")
                rep.near_ties_decode += 1
            decided[i] = e_gpu
            if self.scoreF is not None:
                Fg = self.scoreF.cpu().numpy()[self.umap[i]]
                for slot in range(wl.C):
                    pk = int(pos_before[i, slot])
                    rel = abs(Fg[slot] - F[pk]) / max(abs(F[pk]), 1e-30)
                    rep.max_score_rel_err = max(rep.max_score_rel_err, rel)
                dem = [kk for kk in F if kk not in set(pos_before[i, :wl.C].tolist())]
                assert len(dem) == 1
                rel = abs(Fg[wl.C] - F[dem[0]]) / max(abs(F[dem[0]]), 1e-30)
                rep.max_score_rel_err = max(rep.max_score_rel_err, rel)
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
            if g_set != o_set:
                F = {int(cand_pos[i, x]): cand_F[i, x] for x in range(n_cand[i])}
                bound = max(F[e] for e in o_set)
                for e in g_set ^ o_set:
                    assert e in F, f"step {t} unit {i}: {e} is not a candidate"
                    assert abs(F[e] - bound) <= NEAR_TIE_REL * abs(bound), (
                        f"step {t} unit {i}: evicted sets differ beyond a near-tie at {e}: F={F[e]!r} boundary={bound!r}")
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
