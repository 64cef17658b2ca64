"""CPU-only checks: the C-ABI library loads and exports every symbol the header declares; host-side
validation; the seeded generators are reproducible and slice-consistent."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

from paper_2503_00979_amd import binding, inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    declared = set()
    for name in ("morphkv.h", "morphkv_diag.h"):     # the product interface and the diagnostics beside it
        hdr = open(os.path.join(ROOT, "include", name)).read()
        declared |= set(re.findall(r"\b(morphkv_[a-z_]+)\s*\(", hdr))
    assert declared == set(binding.EXPORTS)
    product = open(os.path.join(ROOT, "include", "morphkv.h")).read()
    for diag in ("morphkv_capture_scores", "morphkv_capture_phase_clocks", "morphkv_calib_copy", "morphkv_calib_read"):
        assert diag not in product
    lib = binding.load_library()
    for name in declared:
        assert hasattr(lib, name), name


def test_oracle_exports(oracle_lib):
    hdr = open(os.path.join(ROOT, "oracle", "morphkv_ref.h")).read()
    declared = set(re.findall(r"\b(morphkv_ref_[a-z_]+)\s*\(", hdr))
    lib = oracle_lib.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_sizes_and_validation_on_host():
    cfg = binding.make_config(n_layers=1, batch=32, n_q_heads=32, n_kv_heads=8, head_dim=128, C_=2048, R=128,
                              fusion="sum", dtype="bf16", max_prompt_len=8192)
    cb, rb, sb = binding.morphkv_sizes(cfg)
    U, n = 256, 2176
    assert cb >= 2 * U * n * 128 * 2 + U * n * 4
    assert rb >= U * 128 * n * 4
    assert cb % 256 == 0 and rb % 256 == 0 and sb % 256 == 0
    bad = [dict(n_q_heads=33), dict(head_dim=96), dict(C_=0), dict(R=0), dict(R=2000), dict(fusion_="x"),
           dict(evict_every=0), dict(max_prompt_len=0), dict(n_q_heads=72, n_kv_heads=8)]
    base = dict(n_layers=1, batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, C_=16, R=4, fusion="sum",
                dtype="bf16", max_prompt_len=64)
    for b in bad:
        kw = dict(base)
        if "fusion_" in b:
            c = binding.make_config(**kw)
            c.fusion = 7
        else:
            kw.update(b)
            c = binding.make_config(**kw)
        with pytest.raises(binding.MorphKVError) as e:
            binding.morphkv_sizes(c)
        assert e.value.code == binding.EINVAL
        assert binding.load_library().morphkv_last_error()


def test_generator_is_counter_based():
    a = inputs.normal(5, 3, (1000,))
    b = inputs.normal(5, 3, (400,), offset=600)
    assert torch.equal(a[600:], b)
    assert not torch.equal(a, inputs.normal(6, 3, (1000,)))
    big = inputs.normal(1, 1, (200000,))
    assert abs(float(big.mean())) < 0.01 and abs(float(big.std()) - 1.0) < 0.01


def test_workload_shapes_and_subsets():
    wl = inputs.workload("c3")
    assert wl.n_units == 256 and wl.G == 4 and len(wl.prompt_lens) == 32
    assert all(1024 <= x <= 8192 for x in wl.prompt_lens)
    assert inputs.workload("c5").G == 7 and inputs.workload("c4").n_units == 2048
    s = inputs.small_workload(9, L=2, B=3, M=4, Mkv=2, d=16, dtype="bf16", C=4, R=3, prompt_lens=(5, 9, 7), steps=2,
                              n_outlier_channels=2)
    Q, K, V = s.prompt()
    Qs, Ks, Vs = s.prompt(batch_index=[2, 0])
    assert torch.equal(Ks[:, 0], K[:, 2]) and torch.equal(Qs[:, 1], Q[:, 0]) and torch.equal(Vs[:, 0], V[:, 2])
    q, k, v = s.decode_inputs(1)
    qs, ks, vs = s.decode_inputs(1, batch_index=[2, 0])
    assert torch.equal(qs[:, 0], q[:, 2]) and torch.equal(ks[:, 1], k[:, 0])
    sc = s.key_channel_scale()
    assert int((sc == 5.0).sum()) <= 2 * 2 * 2 and int((sc == 5.0).sum()) >= 2 * 2


def test_prompt_queries_hold_the_window_rows():
    """The whole-prompt queries carry prompt()'s window queries in the last min(R, N_b) rows before N_b, so the
    fused entry and the window-only entry are given the same window."""
    wl = inputs.small_workload(5, L=2, B=3, M=4, Mkv=2, d=64, dtype="bf16", C=6, R=8, prompt_lens=(20, 3, 8), steps=1)
    Qw, _, _ = wl.prompt()
    Q = wl.prompt_queries()
    assert tuple(Q.shape) == (2, 3, 4, wl.Nmax, 64)
    for b, N in enumerate(wl.prompt_lens):
        Rw = min(wl.R, N)
        assert torch.equal(Q[:, b, :, N - Rw:N], Qw[:, b, :, :Rw])
    sub = wl.prompt_queries(batch_index=[2])
    assert torch.equal(sub[:, 0], Q[:, 2])


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_keep_all_layers_sizes_and_validation_on_host():
    """Layers that keep every token (n_keep_all_layers): their K/V for max_prompt_len + max_new_tokens + R slots are
    added to the cache, next to nothing to the recorded rows; bad combinations are refused with the reason."""
    base = dict(n_layers=4, batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, C_=256, R=32, fusion="sum", dtype="bf16",
                max_prompt_len=4096, max_new_tokens=512)
    c0, r0, _ = binding.morphkv_sizes(binding.make_config(**base))
    c2, r2, _ = binding.morphkv_sizes(binding.make_config(**base, n_keep_all_layers=2))
    sel2 = dict(base, n_layers=2)
    cs, rs, _ = binding.morphkv_sizes(binding.make_config(**sel2))
    n_keep = 4096 + 512 + 32
    units = 2 * 2 * 2                                   # 2 layers x batch 2 x 2 KV heads
    assert c2 - cs >= units * n_keep * 128 * 2 * 2      # K and V, bf16
    assert c2 - cs <= units * (n_keep + 64) * (128 * 2 * 2 + 4) + (1 << 16)
    assert r2 - rs < 1 << 20 and r0 > rs
    for bad, word in ((dict(n_keep_all_layers=5), "n_keep_all_layers"), (dict(n_keep_all_layers=1, max_new_tokens=0), "max_new_tokens"),
                      (dict(n_keep_all_layers=1, dtype="f32"), "bf16"), (dict(n_keep_all_layers=-1), "n_keep_all_layers"),
                      (dict(n_keep_all_layers=1, max_prompt_len=1 << 20), "1048576")):
        with pytest.raises(binding.MorphKVError) as e:
            binding.morphkv_sizes(binding.make_config(**dict(base, **bad)))
        assert e.value.code == binding.EINVAL and word in str(e.value)
