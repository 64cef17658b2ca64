"""ctypes access to the CPU oracle (oracle/morphkv_ref.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this.  It imports nothing from the product package.  Tensors are torch CPU
tensors (fp32 or bf16) or numpy arrays; all pointers handed over are host
pointers.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmorphkv_ref.so")


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (plain C, OpenMP across units)."""
    src = os.path.join(_HERE, "morphkv_ref.c")
    if force or not os.path.exists(LIB_PATH) or os.path.getmtime(LIB_PATH) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", LIB_PATH, src, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return LIB_PATH


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "batch", "n_q_heads", "n_kv_heads", "head_dim", "C", "R",
                 "fusion", "dtype", "evict_every", "max_prompt_len")] + [("softmax_scale", C.c_float),
                                                                         ("max_new_tokens", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            build(force=True)
        L = C.CDLL(LIB_PATH)
        vp, i32p, f64p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_double)
        L.morphkv_ref_create.argtypes = [C.POINTER(vp), C.POINTER(_Cfg)]
        L.morphkv_ref_destroy.argtypes = [vp]
        L.morphkv_ref_prefill_select.argtypes = [vp, vp, vp, vp, vp, C.c_int32, vp]
        L.morphkv_ref_prefill_scores.argtypes = [vp, C.c_int32, vp, C.c_int32]
        L.morphkv_ref_decode_begin.argtypes = [vp, vp, vp, vp, vp]
        L.morphkv_ref_decode_commit.argtypes = [vp, vp]
        L.morphkv_ref_decode_commit_multi.argtypes = [vp, vp]
        L.morphkv_ref_decode_step.argtypes = [vp, vp, vp, vp, vp]
        L.morphkv_ref_candidates.argtypes = [vp, vp, vp, vp, vp, vp]
        L.morphkv_ref_export_positions.argtypes = [vp, vp, vp, vp]
        L.morphkv_ref_row_stride.argtypes = [vp]
        L.morphkv_ref_num_threads.argtypes = []
        for f in ("create", "destroy", "prefill_select", "prefill_scores", "decode_begin", "decode_commit",
                  "decode_commit_multi", "decode_step", "candidates", "export_positions", "row_stride",
                  "num_threads"):
            getattr(L, "morphkv_ref_" + f).restype = C.c_int
        _lib = L
    return _lib


def num_threads() -> int:
    return lib().morphkv_ref_num_threads()


def _host_ptr(t):
    if isinstance(t, torch.Tensor):
        assert t.device.type == "cpu" and t.is_contiguous()
        return C.c_void_p(t.data_ptr())
    assert isinstance(t, np.ndarray) and t.flags["C_CONTIGUOUS"]
    return C.c_void_p(t.ctypes.data)


_FUSION = {"sum": 0, "max": 1, "cumsum": 2}
_DTYPE = {"f32": 0, "bf16": 1}


class RefMorphKV:
    """The oracle, one instance per configuration (state lives in the C handle)."""

    def __init__(self, *, n_layers, batch, n_q_heads, n_kv_heads, head_dim, C_, R, fusion, dtype,
                 evict_every=1, softmax_scale=0.0, max_new_tokens=0):
        self.cfg = _Cfg(n_layers, batch, n_q_heads, n_kv_heads, head_dim, C_, R,
                        _FUSION[fusion], _DTYPE[dtype], evict_every, 0, softmax_scale, max_new_tokens)
        self.dtype = dtype
        self.U = n_layers * batch * n_kv_heads
        self.C, self.R, self.T = C_, R, evict_every
        self.Cs = C_ + (evict_every - 1 if evict_every >= 1 else max_new_tokens)
        self.out_shape = (n_layers, batch, n_q_heads, head_dim)
        self._h = C.c_void_p()
        rc = lib().morphkv_ref_create(C.byref(self._h), C.byref(self.cfg))
        if rc != 0:
            raise ValueError(f"morphkv_ref_create failed: {rc}")

    @classmethod
    def from_workload(cls, wl, **kw):
        if getattr(wl, "n_keep_all_layers", 0):
            return RefMorphKVLayered(wl, **kw)
        return cls(n_layers=wl.n_layers, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                   head_dim=wl.head_dim, C_=wl.C, R=wl.R, fusion=wl.fusion, dtype=wl.dtype,
                   evict_every=wl.evict_every, max_new_tokens=wl.max_new_tokens, **kw)

    def close(self):
        if self._h:
            lib().morphkv_ref_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, t):
        want = torch.float32 if self.dtype == "f32" else torch.bfloat16
        assert isinstance(t, torch.Tensor) and t.dtype == want, (t.dtype, want)

    def prefill_select(self, Qw, K, V, prompt_len, forced_pos: Optional[np.ndarray] = None) -> None:
        for t in (Qw, K, V):
            self._check(t)
        Nmax = K.shape[3]
        pl = np.ascontiguousarray(np.asarray(prompt_len, dtype=np.int32))
        fp = None
        if forced_pos is not None:
            fp = np.ascontiguousarray(forced_pos, dtype=np.int32)
            assert fp.shape == (self.U, self.C)
        rc = lib().morphkv_ref_prefill_select(self._h, _host_ptr(Qw), _host_ptr(K), _host_ptr(V), _host_ptr(pl),
                                              Nmax, _host_ptr(fp) if fp is not None else None)
        if rc != 0:
            raise RuntimeError(f"morphkv_ref_prefill_select failed: {rc}")

    def prefill_scores(self, unit: int) -> np.ndarray:
        n = lib().morphkv_ref_prefill_scores(self._h, unit, None, 0)
        if n < 0:
            raise RuntimeError(f"morphkv_ref_prefill_scores failed: {n}")
        F = np.zeros(max(n, 1), dtype=np.float64)
        lib().morphkv_ref_prefill_scores(self._h, unit, _host_ptr(F), n)
        return F[:n]

    def decode_begin(self, q, k_new, v_new) -> np.ndarray:
        for t in (q, k_new, v_new):
            self._check(t)
        out = np.zeros(self.out_shape, dtype=np.float64)
        rc = lib().morphkv_ref_decode_begin(self._h, _host_ptr(q), _host_ptr(k_new), _host_ptr(v_new), _host_ptr(out))
        if rc != 0:
            raise RuntimeError(f"morphkv_ref_decode_begin failed: {rc}")
        return out

    def candidates(self):
        """(n_cand [U], cand_pos [U][Cs+1], cand_F [U][Cs+1], n_evict [U], choice [U][T])"""
        n_cand = np.zeros(self.U, np.int32)
        n_evict = np.zeros(self.U, np.int32)
        cand_pos = np.full((self.U, self.Cs + 1), -1, np.int32)
        cand_F = np.zeros((self.U, self.Cs + 1), np.float64)
        choice = np.full((self.U, max(self.T, 1)), -1, np.int32)
        rc = lib().morphkv_ref_candidates(self._h, _host_ptr(n_cand), _host_ptr(cand_pos), _host_ptr(cand_F),
                                          _host_ptr(n_evict), _host_ptr(choice))
        if rc != 0:
            raise RuntimeError(f"morphkv_ref_candidates failed: {rc}")
        return n_cand, cand_pos, cand_F, n_evict, choice

    def decode_commit(self, evict_pos: Optional[np.ndarray] = None) -> None:
        ep = None
        if evict_pos is not None:
            ep = np.ascontiguousarray(evict_pos, dtype=np.int32).reshape(self.U, max(self.T, 1))
        rc = lib().morphkv_ref_decode_commit_multi(self._h, _host_ptr(ep) if ep is not None else None)
        if rc != 0:
            raise RuntimeError(f"morphkv_ref_decode_commit failed: {rc}")

    def decode_step(self, q, k_new, v_new) -> np.ndarray:
        out = self.decode_begin(q, k_new, v_new)
        self.decode_commit(None)
        return out

    def export_positions(self):
        """(snapshot positions list per unit (ascending), window positions list per unit (ascending))"""
        W = lib().morphkv_ref_row_stride(self._h)
        pos = np.full((self.U, W), -1, np.int32)
        n_snap = np.zeros(self.U, np.int32)
        n_win = np.zeros(self.U, np.int32)
        rc = lib().morphkv_ref_export_positions(self._h, _host_ptr(pos), _host_ptr(n_snap), _host_ptr(n_win))
        if rc != 0:
            raise RuntimeError(f"morphkv_ref_export_positions failed: {rc}")
        snaps = [pos[u, :n_snap[u]].copy() for u in range(self.U)]
        wins = [pos[u, n_snap[u]:n_snap[u] + n_win[u]].copy() for u in range(self.U)]
        return snaps, wins


class RefMorphKVLayered:
    """Selective layer retention (Appendix A.6): the method is switched off in the first k layers, which keep every
    token.  No new arithmetic: those layers are the same oracle with room for every token (nothing is ever evicted
    there, so each step is plain attention over the whole history), the other layers are the oracle as configured;
    this class only splits the tensors by layer and joins the results (units of the first k layers come first).
    """

    def __init__(self, wl, **kw):
        k = wl.n_keep_all_layers
        assert 0 < k <= wl.n_layers
        common = dict(batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim, R=wl.R,
                      fusion=wl.fusion, dtype=wl.dtype, **kw)
        self.k = k
        self.keep = RefMorphKV(n_layers=k, C_=wl.Nmax, evict_every=0, max_new_tokens=wl.max_new_tokens, **common)
        self.sel = (RefMorphKV(n_layers=wl.n_layers - k, C_=wl.C, evict_every=wl.evict_every,
                               max_new_tokens=wl.max_new_tokens, **common) if k < wl.n_layers else None)
        self.parts = [p for p in (self.keep, self.sel) if p is not None]
        self.dtype = wl.dtype
        self.U = sum(p.U for p in self.parts)
        self.C, self.R, self.T = wl.C, wl.R, wl.evict_every
        self.Cs = self.sel.Cs if self.sel else self.keep.Cs
        self.out_shape = (wl.n_layers, wl.batch, wl.n_q_heads, wl.head_dim)

    def _split(self, t):
        return [t[: self.k].contiguous(), t[self.k:].contiguous()][: len(self.parts)]

    def close(self):
        for p in self.parts:
            p.close()

    def prefill_select(self, Qw, K, V, prompt_len, forced_pos: Optional[np.ndarray] = None) -> None:
        for i, (p, q, k, v) in enumerate(zip(self.parts, self._split(Qw), self._split(K), self._split(V))):
            fp = None
            if forced_pos is not None and p is self.sel:
                fp = np.ascontiguousarray(forced_pos[self.keep.U:])
            p.prefill_select(q, k, v, prompt_len, forced_pos=fp)

    def prefill_scores(self, unit: int) -> np.ndarray:
        return self.keep.prefill_scores(unit) if unit < self.keep.U else self.sel.prefill_scores(unit - self.keep.U)

    def decode_begin(self, q, k_new, v_new) -> np.ndarray:
        outs = [p.decode_begin(a, b, c) for p, a, b, c in
                zip(self.parts, self._split(q), self._split(k_new), self._split(v_new))]
        return np.concatenate(outs, axis=0)

    def candidates(self):
        T = max(self.T, 1)
        n_cand = np.zeros(self.U, np.int32)
        n_evict = np.zeros(self.U, np.int32)
        cand_pos = np.full((self.U, self.Cs + 1), -1, np.int32)
        cand_F = np.zeros((self.U, self.Cs + 1), np.float64)
        choice = np.full((self.U, T), -1, np.int32)
        if self.sel is not None:
            a, b, c, d, e = self.sel.candidates()
            u0 = self.keep.U
            n_cand[u0:], cand_pos[u0:], cand_F[u0:], n_evict[u0:], choice[u0:] = a, b, c, d, e
        ka = self.keep.candidates()
        assert not ka[0].any() and not ka[3].any(), "a layer that keeps every token never has candidates"
        return n_cand, cand_pos, cand_F, n_evict, choice

    def decode_commit(self, evict_pos: Optional[np.ndarray] = None) -> None:
        self.keep.decode_commit(None)
        if self.sel is not None:
            ep = None
            if evict_pos is not None:
                ep = np.asarray(evict_pos).reshape(self.U, -1)[self.keep.U:]
            self.sel.decode_commit(ep)

    def decode_step(self, q, k_new, v_new) -> np.ndarray:
        out = self.decode_begin(q, k_new, v_new)
        self.decode_commit(None)
        return out

    def export_positions(self):
        snaps, wins = [], []
        for p in self.parts:
            a, b = p.export_positions()
            snaps += a
            wins += b
        return snaps, wins
