"""The entry point for callers that cannot allocate: morphkv_prefill_select_noalloc (the library's own static
workspace) against morphkv_prefill_select (caller-provided scratch), through the C-ABI.

Bar: the two run the same kernels on the same inputs, so everything they leave behind must be bit-identical:
retained positions, and the outputs and evictions of the decode steps that follow (index work: bit-exact; the
attention output is the same arithmetic in the same order).  Two calls in a row share the static workspace, the
second with a smaller input (fewer, shorter prompts), so that nothing may depend on what the first left in it.
"""
import pytest
import torch

from paper_2503_00979_amd import binding, inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _compare(wl, steps):
    Qw, K, V = (t.to(DEV) for t in wl.prompt())
    plen = wl.prompt_len_tensor().numpy()
    a = binding.MorphKV.from_workload(wl, DEV)
    b = binding.MorphKV.from_workload(wl, DEV)
    b.scratch.fill_(0xFF)           # the variant must not touch (or need) the handle's scratch buffer
    a.prefill_select(Qw, K, V, plen)
    b.prefill_select_noalloc(Qw, K, V, plen)
    pa, na = a.export_positions()
    pb, nb = b.export_positions()
    assert torch.equal(pa, pb) and torch.equal(na, nb)
    assert int(na.max()) > 0
    for t in range(steps):
        q, k, v = (x.to(DEV) for x in wl.decode_inputs(t))
        assert torch.equal(a.decode_step(q, k, v), b.decode_step(q, k, v)), f"decode step {t} differs"
        assert torch.equal(a.export_evicted(), b.export_evicted())
    pa, na = a.export_positions()
    pb, nb = b.export_positions()
    assert torch.equal(pa, pb) and torch.equal(na, nb)
    assert bool((b.scratch == 0xFF).all()), "the handle's scratch buffer was written"


def test_noalloc_prefill_matches_prefill_select_twice_in_a_row():
    big = inputs.small_workload(41000, L=2, B=3, M=8, Mkv=2, d=128, dtype="bf16", C=200, R=24, fusion="sum",
                                prompt_lens=(1500, 900, 40), steps=40)
    small = inputs.small_workload(41001, L=1, B=2, M=8, Mkv=2, d=128, dtype="bf16", C=48, R=8, fusion="max",
                                  prompt_lens=(130, 9), steps=30)
    _compare(big, big.steps)
    _compare(small, small.steps)      # second call: smaller input, the workspace still holds the first call's data
    f32 = inputs.small_workload(41002, L=1, B=2, M=4, Mkv=2, d=64, dtype="f32", C=20, R=6, fusion="sum",
                                prompt_lens=(70, 33), steps=20)
    _compare(f32, f32.steps)          # the fp32 kernels keep whole rows of weights in the workspace


def test_noalloc_prefill_rejects_sizes_beyond_the_static_workspace():
    # c3's prompt-time workspace is 45 MB: beyond the library's 16 MiB array
    wl = inputs.workload("c3")
    need = binding.morphkv_sizes(binding.make_config(
        n_layers=wl.n_layers, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
        C_=wl.C, R=wl.R, fusion=wl.fusion, dtype=wl.dtype, max_prompt_len=wl.Nmax))[2]
    assert need > 16 << 20
    g = binding.MorphKV.from_workload(wl, DEV)
    L, B, M, Mk, d, R, Nm = wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.R, wl.Nmax
    Qw = torch.zeros(L, B, M, R, d, dtype=torch.bfloat16, device=DEV)
    K = torch.zeros(L, B, Mk, Nm, d, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(binding.MorphKVError) as e:
        g.prefill_select_noalloc(Qw, K, K, wl.prompt_len_tensor().numpy())
    assert e.value.code == binding.EINVAL and "workspace" in str(e.value)
    q, k, v = (x.to(DEV) for x in wl.decode_inputs(0))
    with pytest.raises(binding.MorphKVError) as e:      # the refused call left the handle untouched
        g.decode_step(q, k, v)
    assert e.value.code == binding.ESTATE
