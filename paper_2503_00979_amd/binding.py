"""Thin ctypes binding over libmorphkv.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; torch is used here for
device memory and the current stream.  There is no CPU fallback: if the shared
library is missing or the tensors are not on a GPU this raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MORPHKV_LIB") or os.path.join(_HERE, "libmorphkv.so")  # MORPHKV_LIB: another build

OK, EINVAL, ESTATE, EHIP = 0, -1, -2, -3
FUSION = {"sum": 0, "max": 1, "cumsum": 2}
DTYPE = {"f32": 0, "bf16": 1}
_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}

EXPORTS = ("morphkv_sizes", "morphkv_create", "morphkv_destroy", "morphkv_prefill_select", "morphkv_prefill_select_lse",
           "morphkv_prefill_select_noalloc",
           "morphkv_prefill_attend_select", "morphkv_decode_step",
           "morphkv_decode_step_layer",
           "morphkv_export_positions", "morphkv_export_evicted", "morphkv_export_evicted_list", "morphkv_capture_scores",
           "morphkv_capture_phase_clocks", "morphkv_calib_copy", "morphkv_calib_read", "morphkv_decode_plan",
           "morphkv_last_error")


class MorphKVError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libmorphkv error {code}: {text}")
        self.code = code


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "batch", "n_q_heads", "n_kv_heads", "head_dim", "C", "R", "fusion", "dtype",
                 "evict_every", "max_prompt_len")] + [("softmax_scale", C.c_float), ("max_new_tokens", C.c_int32),
                                                      ("n_keep_all_layers", C.c_int32)]


_lib = None


def load_library():
    """Load the built library; build it first only if no built library is there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build(force=True)
    L = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    szp = C.POINTER(C.c_size_t)
    L.morphkv_sizes.argtypes = [C.POINTER(Config), szp, szp, szp]
    L.morphkv_create.argtypes = [C.POINTER(vp), C.POINTER(Config), vp, vp, vp]
    L.morphkv_destroy.argtypes = [vp]
    L.morphkv_prefill_select.argtypes = [vp, vp, vp, vp, C.POINTER(C.c_int32), C.c_int32, vp]
    L.morphkv_prefill_select_noalloc.argtypes = [vp, vp, vp, vp, C.POINTER(C.c_int32), C.c_int32, vp]
    L.morphkv_prefill_select_lse.argtypes = [vp, vp, vp, vp, vp, C.POINTER(C.c_int32), C.c_int32, vp]
    L.morphkv_prefill_attend_select.argtypes = [vp, vp, vp, vp, vp, vp, C.POINTER(C.c_int32), C.c_int32, vp]
    L.morphkv_decode_step.argtypes = [vp, vp, vp, vp, vp, vp]
    L.morphkv_decode_step_layer.argtypes = [vp, C.c_int32, vp, vp, vp, vp, vp]
    L.morphkv_export_positions.argtypes = [vp, vp, vp, vp]
    L.morphkv_export_evicted.argtypes = [vp, vp, vp]
    L.morphkv_export_evicted_list.argtypes = [vp, vp, vp]
    L.morphkv_capture_scores.argtypes = [vp, vp]
    L.morphkv_capture_phase_clocks.argtypes = [vp, vp]
    L.morphkv_decode_plan.argtypes = [vp, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    L.morphkv_calib_copy.argtypes = [vp, vp, C.c_size_t, vp]
    L.morphkv_calib_read.argtypes = [vp, vp, C.c_size_t, vp]
    L.morphkv_last_error.argtypes = []
    L.morphkv_last_error.restype = C.c_char_p
    for f in EXPORTS[:-1]:
        getattr(L, f).restype = C.c_int
    _lib = L
    return L


def _check(rc: int):
    if rc != OK:
        raise MorphKVError(rc, load_library().morphkv_last_error().decode())


def _dev_ptr(t: torch.Tensor):
    if not t.is_cuda:
        raise ValueError("libmorphkv works on device memory only: tensor is on " + str(t.device))
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return C.c_void_p(t.data_ptr())


def make_config(*, n_layers, batch, n_q_heads, n_kv_heads, head_dim, C_, R, fusion, dtype, max_prompt_len,
                evict_every=1, softmax_scale=0.0, max_new_tokens=0, n_keep_all_layers=0) -> Config:
    return Config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, C_, R, FUSION[fusion], DTYPE[dtype],
                  evict_every, max_prompt_len, softmax_scale, max_new_tokens, n_keep_all_layers)


def morphkv_sizes(cfg: Config):
    a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(load_library().morphkv_sizes(C.byref(cfg), C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def calib_copy(dst: torch.Tensor, src: torch.Tensor):
    """Plain device copy through the library's yardstick kernel (same byte count read and written)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    stream = C.c_void_p(torch.cuda.current_stream(src.device).cuda_stream)
    _check(load_library().morphkv_calib_copy(_dev_ptr(dst), _dev_ptr(src), nbytes, stream))


def calib_read(src: torch.Tensor, sink: torch.Tensor):
    """Plain streaming read of `src` through the library's yardstick kernel; sink: uint32/int32 [256] device tensor."""
    assert sink.numel() >= 256 and sink.element_size() == 4
    stream = C.c_void_p(torch.cuda.current_stream(src.device).cuda_stream)
    _check(load_library().morphkv_calib_read(_dev_ptr(sink), _dev_ptr(src), src.numel() * src.element_size(), stream))


class MorphKV:
    """One handle over caller-owned device buffers (allocated here as torch tensors)."""

    def __init__(self, cfg: Config, device="cuda:0"):
        self.lib = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        if self.device.type != "cuda":
            raise ValueError("libmorphkv needs a GPU device")
        self.U = cfg.n_layers * cfg.batch * cfg.n_kv_heads
        # older-token slots of a selecting layer and of a layer that keeps every token; rows of export_positions
        self.Cs = cfg.C + (cfg.evict_every - 1 if cfg.evict_every >= 1 else cfg.max_new_tokens)
        self.Cs_keep = cfg.max_prompt_len + cfg.max_new_tokens
        k = cfg.n_keep_all_layers
        self.n = (max(self.Cs, self.Cs_keep) if 0 < k < cfg.n_layers else self.Cs_keep if k else self.Cs) + cfg.R
        self.dtype = _TORCH_DTYPE["f32" if cfg.dtype == 0 else "bf16"]
        cb, rb, sb = morphkv_sizes(cfg)
        self.bytes = (cb, rb, sb)
        self.cache = torch.empty(cb, dtype=torch.uint8, device=self.device)
        self.scores_ring = torch.empty(rb, dtype=torch.uint8, device=self.device)
        self.scratch = torch.empty(sb, dtype=torch.uint8, device=self.device)
        self._h = C.c_void_p()
        _check(self.lib.morphkv_create(C.byref(self._h), C.byref(cfg), _dev_ptr(self.cache),
                                       _dev_ptr(self.scores_ring), _dev_ptr(self.scratch)))
        self.out_shape = (cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.head_dim)
        self._scoreF = None

    @classmethod
    def from_workload(cls, wl, device="cuda:0", **kw):
        cfg = make_config(n_layers=wl.n_layers, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                          head_dim=wl.head_dim, C_=wl.C, R=wl.R, fusion=wl.fusion, dtype=wl.dtype,
                          max_prompt_len=wl.Nmax, evict_every=wl.evict_every,
                          max_new_tokens=wl.max_new_tokens, n_keep_all_layers=wl.n_keep_all_layers, **kw)
        return cls(cfg, device)

    def close(self):
        if self._h:
            self.lib.morphkv_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _stream(self):
        return C.c_void_p(torch.cuda.current_stream(self.device).cuda_stream)

    def _want(self, t, shape):
        if t.dtype != self.dtype or tuple(t.shape) != tuple(shape):
            raise ValueError(f"expected {self.dtype} {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")

    def prefill_select(self, Q_window, K, V, prompt_len, lse_window=None):
        """lse_window: optional fp32 [L, B, M, R] log-sum-exp of the window rows from the caller's attention pass."""
        c = self.cfg
        Nmax = K.shape[3]
        self._want(Q_window, (c.n_layers, c.batch, c.n_q_heads, c.R, c.head_dim))
        self._want(K, (c.n_layers, c.batch, c.n_kv_heads, Nmax, c.head_dim))
        self._want(V, (c.n_layers, c.batch, c.n_kv_heads, Nmax, c.head_dim))
        pl = (C.c_int32 * c.batch)(*[int(x) for x in prompt_len])
        if lse_window is not None:
            if lse_window.dtype != torch.float32 or tuple(lse_window.shape) != (c.n_layers, c.batch, c.n_q_heads, c.R):
                raise ValueError("lse_window must be fp32 [L, B, M, R]")
            _check(self.lib.morphkv_prefill_select_lse(self._h, _dev_ptr(Q_window), _dev_ptr(K), _dev_ptr(V),
                                                       _dev_ptr(lse_window), pl, Nmax, self._stream()))
            return
        _check(self.lib.morphkv_prefill_select(self._h, _dev_ptr(Q_window), _dev_ptr(K), _dev_ptr(V), pl, Nmax,
                                               self._stream()))

    def prefill_select_noalloc(self, Q_window, K, V, prompt_len):
        """prefill_select on the library's own static workspace (for callers that cannot allocate)."""
        c = self.cfg
        Nmax = K.shape[3]
        self._want(Q_window, (c.n_layers, c.batch, c.n_q_heads, c.R, c.head_dim))
        self._want(K, (c.n_layers, c.batch, c.n_kv_heads, Nmax, c.head_dim))
        self._want(V, (c.n_layers, c.batch, c.n_kv_heads, Nmax, c.head_dim))
        pl = (C.c_int32 * c.batch)(*[int(x) for x in prompt_len])
        _check(self.lib.morphkv_prefill_select_noalloc(self._h, _dev_ptr(Q_window), _dev_ptr(K), _dev_ptr(V), pl, Nmax,
                                                       self._stream()))

    def prefill_attend_select(self, Q, K, V, prompt_len, O=None, lse=None):
        """Causal attention over the whole prompt (O, optionally lse, are written) and the selection over it.

        Q [L, B, M, Nmax, d], K/V [L, B, M', Nmax, d] bf16; O like Q (allocated if None); lse fp32 [L, B, M, Nmax] or None.
        """
        c = self.cfg
        Nmax = K.shape[3]
        self._want(Q, (c.n_layers, c.batch, c.n_q_heads, Nmax, c.head_dim))
        self._want(K, (c.n_layers, c.batch, c.n_kv_heads, Nmax, c.head_dim))
        self._want(V, (c.n_layers, c.batch, c.n_kv_heads, Nmax, c.head_dim))
        if O is None:
            O = torch.zeros_like(Q)
        self._want(O, Q.shape)
        if lse is not None and (lse.dtype != torch.float32 or tuple(lse.shape) != tuple(Q.shape[:-1])):
            raise ValueError("lse must be fp32 [L, B, M, Nmax]")
        pl = (C.c_int32 * c.batch)(*[int(x) for x in prompt_len])
        _check(self.lib.morphkv_prefill_attend_select(self._h, _dev_ptr(Q), _dev_ptr(K), _dev_ptr(V), _dev_ptr(O),
                                                      _dev_ptr(lse) if lse is not None else None, pl, Nmax,
                                                      self._stream()))
        return O

    def decode_step(self, q, k_new, v_new, out=None):
        c = self.cfg
        self._want(q, (c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        self._want(k_new, (c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._want(v_new, (c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        if out is None:
            out = torch.empty(self.out_shape, dtype=torch.float32, device=self.device)
        _check(self.lib.morphkv_decode_step(self._h, _dev_ptr(q), _dev_ptr(k_new), _dev_ptr(v_new), _dev_ptr(out),
                                            self._stream()))
        return out

    def decode_step_layer(self, layer: int, q, k_new, v_new, out):
        """One layer's units only; the tensors are that layer's [B, M, d] / [B, M', d] / [B, M, d] fp32."""
        c = self.cfg
        self._want(q, (c.batch, c.n_q_heads, c.head_dim))
        self._want(k_new, (c.batch, c.n_kv_heads, c.head_dim))
        self._want(v_new, (c.batch, c.n_kv_heads, c.head_dim))
        if tuple(out.shape) != (c.batch, c.n_q_heads, c.head_dim) or out.dtype != torch.float32 or not out.is_contiguous():
            raise ValueError("out must be a contiguous fp32 [B, M, d] tensor")
        _check(self.lib.morphkv_decode_step_layer(self._h, int(layer), _dev_ptr(q), _dev_ptr(k_new), _dev_ptr(v_new),
                                                  _dev_ptr(out), self._stream()))
        return out

    def decode_step_layer_ptrs(self, layer: int, q_ptr: int, k_ptr: int, v_ptr: int, out_ptr: int, stream_ptr: int):
        rc = self.lib.morphkv_decode_step_layer(self._h, layer, q_ptr, k_ptr, v_ptr, out_ptr, stream_ptr)
        if rc != OK:
            _check(rc)

    def decode_step_ptrs(self, q_ptr: int, k_ptr: int, v_ptr: int, out_ptr: int, stream_ptr: int):
        """Same call with raw device addresses (no shape checks): for tight loops over pre-checked tensors."""
        rc = self.lib.morphkv_decode_step(self._h, q_ptr, k_ptr, v_ptr, out_ptr, stream_ptr)
        if rc != OK:
            _check(rc)

    def export_positions(self):
        """(pos [U, C+R] int32: the position each cache slot holds, in the cache's own order, -1 = free; n_snap [U] int32:
        how many of a unit's tokens are older than its R most recent) device tensors."""
        pos = torch.empty(self.U, self.n, dtype=torch.int32, device=self.device)
        n_snap = torch.empty(self.U, dtype=torch.int32, device=self.device)
        _check(self.lib.morphkv_export_positions(self._h, _dev_ptr(pos), _dev_ptr(n_snap), self._stream()))
        return pos, n_snap

    def export_evicted(self):
        ev = torch.empty(self.U, dtype=torch.int32, device=self.device)
        _check(self.lib.morphkv_export_evicted(self._h, _dev_ptr(ev), self._stream()))
        return ev

    def export_evicted_list(self):
        """[U, evict_every] int32: every position the last step evicted, -1 padded."""
        ev = torch.empty(self.U, max(self.cfg.evict_every, 1), dtype=torch.int32, device=self.device)
        _check(self.lib.morphkv_export_evicted_list(self._h, _dev_ptr(ev), self._stream()))
        return ev

    def decode_plan(self, n_units=None):
        """(workgroups per unit, 32-slot blocks per workgroup) of a decode launch over n_units units (default: all)."""
        a, b = C.c_int32(), C.c_int32()
        _check(self.lib.morphkv_decode_plan(self._h, self.U if n_units is None else int(n_units), C.byref(a), C.byref(b)))
        return a.value, b.value

    def capture_scores(self, enable=True):
        """Returns the [U, n_pad] fp32 device tensor the next decode steps write their fused scores to: one per cache
        slot (the order of export_positions; n_pad = C + R slots rounded up to 32) that holds an eviction candidate."""
        if enable:
            self._scoreF = torch.zeros(self.U, (self.Cs + self.cfg.R + 31) // 32 * 32, dtype=torch.float32, device=self.device)
            _check(self.lib.morphkv_capture_scores(self._h, _dev_ptr(self._scoreF)))
        else:
            _check(self.lib.morphkv_capture_scores(self._h, None))
            self._scoreF = None
        return self._scoreF

    def capture_phase_clocks(self, enable=True):
        """[U, 8] int64 device tensor of per-unit phase time stamps of the next decode steps (100 MHz clock)."""
        if enable:
            self._clocks = torch.zeros(self.U, 8, dtype=torch.int64, device=self.device)
            _check(self.lib.morphkv_capture_phase_clocks(self._h, _dev_ptr(self._clocks)))
        else:
            _check(self.lib.morphkv_capture_phase_clocks(self._h, None))
            self._clocks = None
        return self._clocks
