"""Seeded synthetic inputs for the MorphKV decode hot path.

This module only draws numbers and shapes them: it holds none of the method's
arithmetic (no attention, no softmax, no fusion, no selection), so both the HIP
path and the CPU oracle may be fed from it without sharing any logic.

Generator: a counter-based stream.  Element ``i`` of stream ``(seed, stream)``
is ``mix64(key + (i + 1) * GOLDEN)`` with the splitmix64 finaliser, turned into
one N(0,1) draw by Box-Muller from two 24-bit uniforms.  Any slice of any
tensor is therefore reproducible on its own, on the CPU or on the GPU (torch
ops only), and the same bytes can be handed to both sides of a parity test.

The five workloads are the synthetic stand-ins for the paper's long-response
and long-context runs (Section 4, "Benchmarks"): only their shapes are used
(prompt length, retained capacity C, recent window R, fusion, head layout of
Llama-3.1-8B / Mistral-7B, Section 4 "Models").
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import torch

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB

# tensor ids (upper bits of the stream number)
T_PROMPT_K, T_PROMPT_V, T_PROMPT_Q, T_DEC_Q, T_DEC_K, T_DEC_V, T_LEN, T_OUTLIER = range(1, 9)
T_PROMPT_QALL = 9
T_CODEBOOK, T_CODE_PROMPT, T_CODE_DEC = 10, 11, 12


def _s64(x: int) -> int:
    """Python int (mod 2^64) -> the signed value torch.int64 holds for it."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix64_int(x: int) -> int:
    x &= _M64
    x ^= x >> 30
    x = (x * _C1) & _M64
    x ^= x >> 27
    x = (x * _C2) & _M64
    x ^= x >> 31
    return x


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    return (x >> k) & ((1 << (64 - k)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    x = x ^ _lsr(x, 30)
    x = x * _s64(_C1)
    x = x ^ _lsr(x, 27)
    x = x * _s64(_C2)
    x = x ^ _lsr(x, 31)
    return x


def _key(seed: int, stream: int) -> int:
    return _mix64_int(seed ^ _mix64_int(stream + _GOLDEN))


def raw_bits(seed: int, stream: int, n: int, device="cpu", offset: int = 0) -> torch.Tensor:
    """n 64-bit words (as int64) of stream (seed, stream), starting at element ``offset``."""
    idx = torch.arange(offset + 1, offset + n + 1, dtype=torch.int64, device=device)
    return _mix64(idx * _s64(_GOLDEN) + _s64(_key(seed, stream)))


def normal(seed: int, stream: int, shape, device="cpu", offset: int = 0) -> torch.Tensor:
    """fp32 tensor of N(0,1) draws, element i from word i of the stream."""
    n = 1
    for s in shape:
        n *= int(s)
    z = raw_bits(seed, stream, n, device, offset)
    u1 = (_lsr(z, 40) + 1).to(torch.float32) * (1.0 / (1 << 24))          # (0, 1]
    u2 = (_lsr(z, 16) & 0xFFFFFF).to(torch.float32) * (1.0 / (1 << 24))   # [0, 1)
    r = torch.sqrt(-2.0 * torch.log(u1))
    return (r * torch.cos((2.0 * math.pi) * u2)).reshape(tuple(shape))


def integers(seed: int, stream: int, lo: int, hi: int, n: int) -> List[int]:
    """n integers uniform in [lo, hi] (host list)."""
    z = raw_bits(seed, stream, n, "cpu")
    return [lo + int(v) % (hi - lo + 1) for v in _lsr(z, 11).tolist()]


_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


@dataclass(frozen=True)
class Workload:
    """Shape of one synthetic run; field names follow the paper's notation
    (M query heads, M' KV heads, capacity C, window R; Algorithm 1 inputs)."""
    name: str
    n_layers: int
    batch: int
    n_q_heads: int          # M
    n_kv_heads: int         # M'
    head_dim: int           # d_h
    dtype: str              # "f32" | "bf16"
    C: int
    R: int
    fusion: str             # "sum" | "max"
    prompt_lens: Tuple[int, ...]
    steps: int
    seed: int
    n_outlier_channels: int = 0     # per KV head, key channels scaled by outlier_scale
    outlier_scale: float = 5.0
    evict_every: int = 1
    max_new_tokens: int = 0   # only with evict_every == 0 (selection at the prompt only): room for decode steps
    n_keep_all_layers: int = 0  # the first layers keep every token (selective layer retention); needs max_new_tokens
    key_codes: int = 0        # > 0: every key is one of this many seeded vectors per (layer, KV head), so that
                              # many tokens hold bit-identical keys (inputs with exact ties); 1 = all keys identical

    # ---- derived sizes -------------------------------------------------
    @property
    def G(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_units(self) -> int:
        return self.n_layers * self.batch * self.n_kv_heads

    @property
    def Nmax(self) -> int:
        return max(self.prompt_lens)

    @property
    def torch_dtype(self):
        return _TORCH_DTYPE[self.dtype]

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    # ---- tensors -------------------------------------------------------
    def key_channel_scale(self, device="cpu") -> torch.Tensor:
        """[L, 1, M', 1, d] multiplier for keys: outlier_scale on a few seeded channels."""
        sc = torch.ones(self.n_layers, 1, self.n_kv_heads, 1, self.head_dim, dtype=torch.float32)
        if self.n_outlier_channels:
            for l in range(self.n_layers):
                for h in range(self.n_kv_heads):
                    ch = integers(self.seed, (T_OUTLIER << 40) + l * self.n_kv_heads + h,
                                  0, self.head_dim - 1, self.n_outlier_channels)
                    for c in ch:
                        sc[l, 0, h, 0, c] = self.outlier_scale
        return sc.to(device)

    def _slab(self, tid: int, l: int, b: int, heads: int, rows: int, device) -> torch.Tensor:
        return normal(self.seed, (tid << 40) + l * self.batch + b, (heads, rows, self.head_dim), device)

    def _coded_keys(self, l: int, tid: int, stream: int, rows: int, device) -> torch.Tensor:
        """[M', rows, d] fp32: row r of head h is code word code[h, r] of that head's seeded codebook."""
        book = normal(self.seed, (T_CODEBOOK << 40) + l, (self.n_kv_heads, self.key_codes, self.head_dim), device)
        z = _lsr(raw_bits(self.seed, (tid << 40) + stream, self.n_kv_heads * rows, device), 11) % self.key_codes
        idx = z.reshape(self.n_kv_heads, rows, 1).expand(-1, -1, self.head_dim)
        return torch.gather(book, 1, idx)

    def prompt(self, device="cpu", batch_index: Optional[List[int]] = None):
        """(Q_window [L,B,M,R,d], K [L,B,M',Nmax,d], V [L,B,M',Nmax,d]) in the workload dtype.

        Row j of Q_window is the query of prompt position N_b - min(R, N_b) + j.
        K/V rows at or beyond a sequence's prompt length are padding (still seeded).
        """
        bs = list(range(self.batch)) if batch_index is None else list(batch_index)
        L, Mq, Mk, d, Nm, R = self.n_layers, self.n_q_heads, self.n_kv_heads, self.head_dim, self.Nmax, self.R
        dt = self.torch_dtype
        Q = torch.empty(L, len(bs), Mq, R, d, dtype=dt, device=device)
        K = torch.empty(L, len(bs), Mk, Nm, d, dtype=dt, device=device)
        V = torch.empty(L, len(bs), Mk, Nm, d, dtype=dt, device=device)
        ksc = self.key_channel_scale(device)
        for l in range(L):
            for i, b in enumerate(bs):
                Q[l, i] = self._slab(T_PROMPT_Q, l, b, Mq, R, device).to(dt)
                K[l, i] = (self._slab(T_PROMPT_K, l, b, Mk, Nm, device) * ksc[l, 0]).to(dt)
                if self.key_codes:
                    K[l, i] = self._coded_keys(l, T_CODE_PROMPT, l * self.batch + b, Nm, device).to(dt)
                V[l, i] = self._slab(T_PROMPT_V, l, b, Mk, Nm, device).to(dt)
        return Q, K, V

    def prompt_queries(self, device="cpu", batch_index: Optional[List[int]] = None) -> torch.Tensor:
        """Queries of every prompt position, [L,B,M,Nmax,d] in the workload dtype, ~N(0,1).

        The last min(R, N_b) rows before N_b are the rows of prompt()'s Q_window, so that a pass over the whole
        prompt and the window-only entry see the same window queries; rows at or beyond N_b are padding.
        """
        bs = list(range(self.batch)) if batch_index is None else list(batch_index)
        L, Mq, d, Nm, R = self.n_layers, self.n_q_heads, self.head_dim, self.Nmax, self.R
        dt = self.torch_dtype
        Q = torch.empty(L, len(bs), Mq, Nm, d, dtype=dt, device=device)
        for l in range(L):
            for i, b in enumerate(bs):
                Q[l, i] = self._slab(T_PROMPT_QALL, l, b, Mq, Nm, device).to(dt)
                N = self.prompt_lens[b]
                Rw = min(R, N)
                Q[l, i, :, N - Rw:N] = self._slab(T_PROMPT_Q, l, b, Mq, R, device).to(dt)[:, :Rw]
        return Q

    def decode_inputs(self, step: int, device="cpu", batch_index: Optional[List[int]] = None):
        """(q [L,B,M,d], k_new [L,B,M',d], v_new [L,B,M',d]) of decode step ``step`` (0-based)."""
        L, B, Mq, Mk, d = self.n_layers, self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim
        dt = self.torch_dtype
        q = normal(self.seed, (T_DEC_Q << 40) + step, (L, B, Mq, d), device)
        k = normal(self.seed, (T_DEC_K << 40) + step, (L, B, Mk, d), device)
        v = normal(self.seed, (T_DEC_V << 40) + step, (L, B, Mk, d), device)
        k = k * self.key_channel_scale(device)[:, :, :, 0, :]
        if self.key_codes:
            for l in range(L):
                for b in range(B):
                    k[l, b] = self._coded_keys(l, T_CODE_DEC, (step * L + l) * B + b, 1, device)[:, 0]
        q, k, v = q.to(dt), k.to(dt), v.to(dt)
        if batch_index is not None:
            ix = torch.tensor(list(batch_index), device=device)
            q, k, v = q.index_select(1, ix), k.index_select(1, ix), v.index_select(1, ix)
        return q.contiguous(), k.contiguous(), v.contiguous()

    def prompt_len_tensor(self, batch_index: Optional[List[int]] = None) -> torch.Tensor:
        bs = list(range(self.batch)) if batch_index is None else list(batch_index)
        return torch.tensor([self.prompt_lens[b] for b in bs], dtype=torch.int32)

    def with_batch_subset(self, batch_index: List[int]) -> "Workload":
        """Same workload restricted to some sequences (shape bookkeeping only:
        tensors for it come from prompt()/decode_inputs() with the same batch_index)."""
        return replace(self, batch=len(batch_index),
                       prompt_lens=tuple(self.prompt_lens[b] for b in batch_index))


def _uniform_lens(seed: int, batch: int, lo: int, hi: int) -> Tuple[int, ...]:
    return tuple(integers(seed, T_LEN << 40, lo, hi, batch))


def workload(name: str) -> Workload:
    """The five named synthetic configurations (c1..c5)."""
    base = 0x5EED0000
    if name == "c1":   # toy single layer, fp32
        return Workload("c1", 1, 1, 8, 2, 64, "f32", 32, 16, "sum", (256,), 64, base + 1)
    if name == "c2":   # Llama-3.1-8B-shaped layer, batch 1, outlier key channels, max fusion
        return Workload("c2", 1, 1, 32, 8, 128, "bf16", 1024, 64, "max", (4096,), 2048, base + 2,
                        n_outlier_channels=3)
    if name == "c3":   # same layer, batch 32, ragged prompts 1k-8k, long responses, sum fusion
        return Workload("c3", 1, 32, 32, 8, 128, "bf16", 2048, 128, "sum",
                        _uniform_lens(base + 3, 32, 1024, 8192), 4096, base + 3, n_outlier_channels=3)
    if name == "c4":   # Mistral-7B-shaped full stack, per-layer independent selection
        return Workload("c4", 32, 8, 32, 8, 128, "bf16", 512, 32, "sum", (2048,) * 8, 8192, base + 4)
    if name == "c5":   # wide-GQA stress
        return Workload("c5", 1, 64, 28, 4, 128, "bf16", 4096, 256, "max", (16384,) * 64, 1024, base + 5)
    raise KeyError(name)


def small_workload(seed: int, *, L=1, B=1, M=4, Mkv=2, d=64, dtype="f32", C=6, R=4, fusion="sum",
                   prompt_lens=(20,), steps=30, n_outlier_channels=0, evict_every=1, max_new_tokens=0,
                   key_codes=0, n_keep_all_layers=0) -> Workload:
    """Free-form small case for tests."""
    return Workload(f"small{seed}", L, B, M, Mkv, d, dtype, C, R, fusion, tuple(prompt_lens), steps, seed,
                    n_outlier_channels=n_outlier_channels, evict_every=evict_every, max_new_tokens=max_new_tokens,
                    key_codes=key_codes, n_keep_all_layers=n_keep_all_layers)
