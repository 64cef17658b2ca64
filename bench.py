#!/usr/bin/env python3
"""Benchmark of the MorphKV decode hot path on one MI355X.

A "step" is one morphkv_decode_step call over all units of the workload: attention of the new token
over the C+R resident tokens, recording the row, score fusion, top-C selection and K/V compaction.
Default workload: c3 (Llama-3.1-8B-shaped layer, batch 32, C=2048, R=128, sum fusion, bf16), measured
in steady state (every cache full), inputs resident in HBM before the timed region.

Prints ONE JSON line (see the keys below).  `roofline` prices the fused decode kernel against the HBM
peak using the algorithmic bytes per step; `cpu_baseline` is the CPU oracle timed on a bounded sample
of the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, vendor figure


def algorithmic_bytes_per_step(wl, keep_tokens: float = 0.0) -> int:
    """Bytes the method must move per decode step in steady state (per unit, times U):
    K and V of the C+R resident tokens read once; the new row of recorded weights written;
    the score state (one aggregate row read, the running aggregate read and written);
    q, k_new, v_new in, the new token's K/V written, fp32 output; one K/V row moved and one
    column of the R rows moved on compaction.  Units of layers that keep every token (Appendix A.6) read the K
    and V of the `keep_tokens` tokens they hold and write the new token's; they have no score state."""
    d, s, G, R = wl.head_dim, wl.elem_bytes, wl.G, wl.R
    C = wl.C + (wl.evict_every - 1) / 2.0   # older tokens held, averaged over the T steps between selections
    n = C + R
    per_unit = (2 * n * d * s) + 4 * n + 12 * (C + 1) + (G + 4) * d * s + 4 * G * d + 4 * d * s + 8 * R
    upl = wl.batch * wl.n_kv_heads
    k = getattr(wl, "n_keep_all_layers", 0)
    per_keep_unit = 2 * keep_tokens * d * s + (G + 4) * d * s + 4 * G * d + 2 * d * s
    return int(per_unit * (wl.n_layers - k) * upl + per_keep_unit * k * upl)


def read_traffic(name: str):
    """(bytes, source): HBM-side bytes per launch of the decode kernel from the STORED rocprofv3 counter runs under
    profiles/ (FETCH_SIZE and WRITE_SIZE, scaled by a plain copy of known size).  Not measured in this run: hardware
    counters need the profiler around the process."""
    path = os.path.join(ROOT, "profiles", f"decode_fused_{name}_hbm_traffic.json")
    if os.path.exists(path):
        with open(path) as f:
            return (json.load(f).get("traffic_bytes_per_launch"),
                    f"stored profile profiles/decode_fused_{name}_hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE / "
                    f"WRITE_SIZE runs of this benchmark; not measured in this run)")
    return None, None


def phase_clocks(g, run_steps, n_units, launches=5, steps_per_launch_sample=8, dump=None, groups=1):
    """Phase time stamps of the fused decode kernel (diagnostics build, bf16 head_dim 128): per unit, microseconds
    after the launch's first workgroup started; mean / p10 / p90 over units and sampled launches."""
    import numpy as np
    import torch
    clk = g.capture_phase_clocks(True)
    acc = []
    for _ in range(launches + 1):
        run_steps(steps_per_launch_sample)
        torch.cuda.synchronize()
        acc.append(clk.cpu().numpy().astype(np.int64).copy())
    g.capture_phase_clocks(False)
    a = np.stack(acc)[1:] * 0.01          # 100 MHz clock -> us
    if dump:
        np.save(dump, a)                  # [launch, unit, stamp] for a look at which units end late
    if groups > 1:                        # one launch per layer: every layer's units against their own launch's start
        a = a.reshape(a.shape[0] * groups, n_units // groups, a.shape[2])
    t0 = a[:, :, 0].min(1, keepdims=True)
    names = ["workgroup start", "end of the K pass", "end of softmax / record", "end of the V pass", "end of the step",
             "last wave at the first barrier", "first wave at the first barrier", "first barrier passed"]
    out = {}
    for i in (0, 6, 5, 7, 1, 2, 3, 4):
        x = a[:, :, i] - t0
        out[names[i]] = [round(float(x.mean()), 2), round(float(np.percentile(x, 10)), 2), round(float(np.percentile(x, 90)), 2)]
    out["kernel span, first start to last end"] = round(float((a[:, :, 4].max(1) - a[:, :, 0].min(1)).mean()), 2)
    return out


def cpu_baseline(wl, Qw, K, V, dec_inputs, n_steps=200, max_seqs=8):
    """The oracle as it stands, on a bounded sample: sequences whose cache is full right after the
    prompt (steady state from the first step), all their KV heads."""
    import torch
    from oracle import ref as oref
    full = [b for b in range(wl.batch) if wl.prompt_lens[b] - wl.R >= wl.C]
    sample = full[:max_seqs] if full else [0]
    wl_s = wl.with_batch_subset(sample)
    ix = torch.tensor(sample, device=K.device)
    Qs, Ks, Vs = (t.index_select(1, ix).cpu().contiguous() for t in (Qw, K, V))
    o = oref.RefMorphKV.from_workload(wl_s)
    t0 = time.perf_counter()
    o.prefill_select(Qs, Ks, Vs, wl_s.prompt_len_tensor().numpy())
    t_prefill = time.perf_counter() - t0
    ins = []
    for t in range(n_steps):
        q, k, v = dec_inputs(t)
        ins.append(tuple(x.index_select(1, ix).cpu().contiguous() for x in (q, k, v)))
    t0 = time.perf_counter()
    for q, k, v in ins:
        o.decode_step(q, k, v)
    dt = time.perf_counter() - t0
    frac = wl_s.n_units / wl.n_units
    return {
        "value": (n_steps / dt) * frac, "unit": "steps/s", "cores": oref.num_threads(), "kind": "oracle",
        "sample": f"{len(sample)} of {wl.batch} sequences ({wl_s.n_units} of {wl.n_units} units), {n_steps} "
                  f"steady-state decode steps in {dt:.2f}s, scaled by {frac:.4f} to the full batch; "
                  f"oracle prefill of the sample took {t_prefill:.1f}s (not in value)",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--repeats", type=int, default=5, help="timed repetitions of --steps; the median is reported")
    ap.add_argument("--per-layer", action="store_true",
                    help="one launch per layer and step (the order a model's layer chain imposes) instead of one "
                         "launch over all layers")
    ap.add_argument("--graph", action="store_true",
                    help="with --per-layer: the launches of two consecutive steps are captured in a HIP graph once "
                         "and replayed (inputs copied into static buffers before each replay), as serving stacks "
                         "run their decode loops; takes the host out of the measurement")
    ap.add_argument("--fusion", default=None, choices=["sum", "max", "cumsum"],
                    help="override the workload's fusion; cumsum = the running-sum comparison policy (H2O's score)")
    ap.add_argument("--evict-every", type=int, default=1,
                    help="T of the coarse schedule (Appendix A.5): selection at every T-th step")
    ap.add_argument("--layers", type=int, default=0,
                    help="override the workload's number of layers (c4 with 1 layer = the launch a per-layer call makes)")
    ap.add_argument("--keep-all-layers", type=int, default=0,
                    help="the first K layers keep every token (Appendix A.6: selective layer retention); their caches "
                         "grow during the run, the bytes are priced at their mean length over the timed region")
    ap.add_argument("--prefill-repeats", type=int, default=3,
                    help="prefill_select is run this many times on the same prompts (it rewrites all state); the "
                         "median is reported as prefill_select_ms")
    ap.add_argument("--prefill-lse", action="store_true",
                    help="also time prefill_select_lse (window rows' log-sum-exp supplied by the caller)")
    ap.add_argument("--prefill-attend", action="store_true",
                    help="also time prefill_attend_select (causal attention over the whole prompt + selection; bf16 "
                         "workloads) and report it against the bf16 matrix-core peak")
    ap.add_argument("--no-stream-ref", action="store_true",
                    help="skip the plain streaming-read measurement reported as roofline.stream_read_GBs")
    ap.add_argument("--phase-clocks", action="store_true",
                    help="after the timed region also run the diagnostics build of the fused kernel and report its phase "
                         "time stamps (config.phase_clocks_us; a table on stderr)")
    ap.add_argument("--phase-clocks-dump", default=None,
                    help="with --phase-clocks: also save the raw time stamps [launch, unit, stamp] (us) to this .npy file")
    ap.add_argument("--phase-clocks-launches", type=int, default=5, help="launches sampled by --phase-clocks")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="after the timed region also run 4 plain copies of this many MiB (yardstick for rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on ONE GPU (units are independent caches; there is no collective to "
              "measure). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2503_00979_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    wl = inputs.workload(args.workload)
    if args.evict_every != 1 or args.fusion:
        import dataclasses
        wl = dataclasses.replace(wl, evict_every=args.evict_every, fusion=args.fusion or wl.fusion)
    K_steps, W = args.steps, args.warmup
    if args.layers:
        import dataclasses
        wl = dataclasses.replace(wl, n_layers=args.layers)
    if args.keep_all_layers:
        import dataclasses
        assert wl.dtype == "bf16" and 0 < args.keep_all_layers <= wl.n_layers and args.no_cpu_baseline, \
            "--keep-all-layers: bf16 workloads, with --no-cpu-baseline"
        fill = max(0, max(wl.C + wl.R - n for n in wl.prompt_lens))
        wl = dataclasses.replace(wl, n_keep_all_layers=args.keep_all_layers,
                                 max_new_tokens=fill + W + max(1, args.repeats) * K_steps + 64)

    # ---- setup (untimed): prompts, prompt-time selection, run until every cache is full
    g = binding.MorphKV.from_workload(wl, dev)
    Qw, K, V = wl.prompt(dev)
    pf = []
    for _ in range(max(1, args.prefill_repeats)):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.prefill_select(Qw, K, V, wl.prompt_len_tensor().numpy())
        e1.record()
        torch.cuda.synchronize()
        pf.append(e0.elapsed_time(e1))
    prefill_ms = sorted(pf)[len(pf) // 2]
    prefill_lse_ms = None
    if args.prefill_lse:
        # what the caller's own attention pass over the prompt would hand over: log-sum-exp of the window rows
        # (computed here with torch, untimed), then the variant that skips the statistics pass
        G, R = wl.G, wl.R
        lse = torch.zeros(wl.n_layers, wl.batch, wl.n_q_heads, R, dtype=torch.float32, device=dev)
        for l in range(wl.n_layers):
            for b in range(wl.batch):
                N = wl.prompt_lens[b]
                Rw = min(R, N)
                lg = torch.einsum("mjd,mnd->mjn", Qw[l, b, :, :Rw].float(),
                                  K[l, b, :, :N].float().repeat_interleave(G, dim=0)) / wl.head_dim ** 0.5
                pj = torch.arange(N - Rw, N, device=dev)[:, None]
                lg.masked_fill_(torch.arange(N, device=dev)[None, :] > pj, float("-inf"))
                lse[l, b, :, :Rw] = torch.logsumexp(lg, -1)
                del lg
        pfl = []
        for _ in range(max(1, args.prefill_repeats)):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.prefill_select(Qw, K, V, wl.prompt_len_tensor().numpy(), lse_window=lse)
            e1.record()
            torch.cuda.synchronize()
            pfl.append(e0.elapsed_time(e1))
        prefill_lse_ms = sorted(pfl)[len(pfl) // 2]
        del lse
    attend = None
    if args.prefill_attend:
        Qall = wl.prompt_queries(dev)
        Oall = torch.empty_like(Qall)
        pa = []
        for _ in range(max(1, args.prefill_repeats)):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.prefill_attend_select(Qall, K, V, wl.prompt_len_tensor().numpy(), O=Oall)
            e1.record()
            torch.cuda.synchronize()
            pa.append(e0.elapsed_time(e1))
        ms = sorted(pa)[len(pa) // 2]
        # 2 d flop per (query, key <= query) pair and head for each of the two products
        flop = sum(4.0 * wl.head_dim * (n * (n + 1) / 2) for n in wl.prompt_lens) * wl.n_q_heads * wl.n_layers
        attend = {"prefill_attend_select_ms": ms, "flop": flop,
                  "whole_call": {"bound": "mfma", "achieved": flop / (ms / 1e3) / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                                 "frac": flop / (ms / 1e3) / 1e12 / 2500.0},
                  "note": "achieved = attention flop / time of the whole call (attention pass + selection passes)"}
        del Qall, Oall
        g.prefill_select(Qw, K, V, wl.prompt_len_tensor().numpy())   # back to the state every other run starts from
    fill_steps = max(0, max(wl.C + wl.R - n for n in wl.prompt_lens))
    step_no = 0
    out = torch.empty(g.out_shape, dtype=torch.float32, device=dev)

    def dec_inputs(t):
        return wl.decode_inputs(t, dev)

    for _ in range(fill_steps):
        q, k, v = dec_inputs(step_no)
        g.decode_step(q, k, v, out)
        step_no += 1
    torch.cuda.synchronize()
    pos, n_snap = g.export_positions()
    assert int(n_snap.min()) >= wl.C, "not in steady state"

    # ---- inputs of the timed region, resident in HBM (a pool that is cycled if K is large)
    pool = min(K_steps + W, 512)
    qs, ks, vs = [], [], []
    for t in range(pool):
        q, k, v = dec_inputs(step_no + t)
        qs.append(q); ks.append(k); vs.append(v)
    Qp, Kp, Vp = torch.stack(qs), torch.stack(ks), torch.stack(vs)
    del qs, ks, vs
    stream = torch.cuda.current_stream(dev)
    sp = ctypes.c_void_p(stream.cuda_stream)
    qb, kb, vb = Qp[0].numel() * Qp.element_size(), Kp[0].numel() * Kp.element_size(), Vp[0].numel() * Vp.element_size()
    qptr = [ctypes.c_void_p(Qp.data_ptr() + i * qb) for i in range(pool)]
    kptr = [ctypes.c_void_p(Kp.data_ptr() + i * kb) for i in range(pool)]
    vptr = [ctypes.c_void_p(Vp.data_ptr() + i * vb) for i in range(pool)]
    optr = ctypes.c_void_p(out.data_ptr())

    nl = wl.n_layers
    ob = out[0].numel() * 4

    graph = None
    if args.graph:
        assert args.per_layer and K_steps % 2 == 0 and W % 2 == 0 and pool % 2 == 0, "--graph: --per-layer, even step counts"
        sQ, sK, sV = torch.empty_like(Qp[:2]), torch.empty_like(Kp[:2]), torch.empty_like(Vp[:2])
        cs = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        spc = ctypes.c_void_p(cs.cuda_stream)
        for i in range(2):  # two eager steps first: kernel attributes are set outside the capture
            for l in range(nl):
                g.decode_step_layer_ptrs(l, qptr[i].value + l * (qb // nl), kptr[i].value + l * (kb // nl),
                                         vptr[i].value + l * (vb // nl), optr.value + l * ob, sp)
        torch.cuda.synchronize()
        with torch.cuda.stream(cs):
            with torch.cuda.graph(graph, stream=cs):
                for i in range(2):
                    for l in range(nl):
                        g.decode_step_layer_ptrs(l, sQ[i].data_ptr() + l * (qb // nl), sK[i].data_ptr() + l * (kb // nl),
                                                 sV[i].data_ptr() + l * (vb // nl), optr.value + l * ob, spc)
        torch.cuda.synchronize()

    def run(nsteps, start):
        if graph is not None:
            for i in range(0, nsteps, 2):
                j = (start + i) % pool
                sQ.copy_(Qp[j:j + 2]); sK.copy_(Kp[j:j + 2]); sV.copy_(Vp[j:j + 2])
                graph.replay()
            return
        if args.per_layer:
            for i in range(nsteps):
                j = (start + i) % pool
                for l in range(nl):
                    g.decode_step_layer_ptrs(l, qptr[j].value + l * (qb // nl), kptr[j].value + l * (kb // nl),
                                             vptr[j].value + l * (vb // nl), optr.value + l * ob, sp)
            return
        for i in range(nsteps):
            j = (start + i) % pool
            g.decode_step_ptrs(qptr[j], kptr[j], vptr[j], optr, sp)

    run(W, 0)
    torch.cuda.synchronize()
    times = []
    for r in range(max(1, args.repeats)):
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record(stream)
        run(K_steps, W + r * K_steps)
        ev1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        times.append((ev0.elapsed_time(ev1) / 1e3, wall))
    phases = None
    if args.phase_clocks:
        cursor = [W + max(1, args.repeats) * K_steps]

        def run_some(n):
            run(n, cursor[0])
            cursor[0] += n
        phases = phase_clocks(g, run_some, wl.n_units, launches=args.phase_clocks_launches, dump=args.phase_clocks_dump,
                              groups=nl if args.per_layer else 1)
        print(f"phase time stamps of the fused decode kernel, {wl.name}: us after the launch's first workgroup start "
              f"(mean / p10 / p90 over units and {args.phase_clocks_launches} launches)", file=sys.stderr)
        for k_, v_ in phases.items():
            print(f"  {k_:40s} {v_}", file=sys.stderr)
    if args.calib_copy_mib > 0:
        src = torch.ones(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            binding.calib_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
    # what this device sustains when a kernel only streams (the practical ceiling next to the data-sheet peak):
    # a plain read of a buffer as large as the step's K+V, 50 launches back to back
    stream_gbs = None
    if not args.no_stream_ref:
        nbytes = (2 * (wl.C + wl.R) * wl.head_dim * wl.elem_bytes * wl.n_units + 15) // 16 * 16
        src = torch.ones(nbytes, dtype=torch.uint8, device=dev)
        sink = torch.zeros(256, dtype=torch.int32, device=dev)
        for _ in range(5):
            binding.calib_read(src, sink)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(stream)
        for _ in range(50):           # back to back, like the decode steps
            binding.calib_read(src, sink)
        ev1.record(stream)
        torch.cuda.synchronize()
        stream_gbs = nbytes / (ev0.elapsed_time(ev1) / 1e3 / 50) / 1e9
        del src, sink
    times.sort()
    dev_s, wall_s = times[len(times) // 2]
    sec = max(dev_s, 0.0)                      # HIP events on the launch stream bracket exactly the K kernels
    ms_per_step = sec / K_steps * 1e3
    # (layers that keep everything: tokens held at the middle of the timed region, mean over the batch)
    keep_tokens = (sum(wl.prompt_lens) / len(wl.prompt_lens) + fill_steps + W + max(1, args.repeats) * K_steps / 2.0
                   if args.keep_all_layers else 0.0)
    A = algorithmic_bytes_per_step(wl, keep_tokens)
    launches = K_steps * (nl if args.per_layer else (2 if 0 < args.keep_all_layers < nl else 1))
    achieved = A / (sec / K_steps) / 1e9
    traffic, traffic_src = ((None, None) if (args.per_layer or wl.evict_every > 1 or args.fusion or args.keep_all_layers)
                            else read_traffic(wl.name))
    res = {
        "metric": "decode steps/s incl. KV selection (B=32, 8B shape) on 1 GPU; % HBM roofline",
        "value": K_steps / sec, "unit": "steps/s", "n_gpus": 1, "steps": K_steps, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: L={wl.n_layers} B={wl.batch} M={wl.n_q_heads} M'={wl.n_kv_heads} "
                               f"d={wl.head_dim} C={wl.C} R={wl.R} fusion={wl.fusion} {wl.dtype}, steady state"
                               + (f", selection every {wl.evict_every} steps" if wl.evict_every > 1 else "")
                               + (f", first {args.keep_all_layers} layers keep every token (about {keep_tokens:.0f} each "
                                  f"during the timed steps)" if args.keep_all_layers else "")
                               + (f", {nl} launches per step (one per layer)" if args.per_layer else "")
                               + (", two steps per HIP graph replay" if args.graph else ""),
                   "units": wl.n_units, "fill_steps": fill_steps, "repeats": args.repeats,
                   "wall_ms_per_step": wall_s / K_steps * 1e3, "prefill_select_ms": prefill_ms,
                   "prefill_select_first_call_ms": pf[0],
                   **({"prefill_select_lse_ms": prefill_lse_ms} if prefill_lse_ms is not None else {}),
                   **({"prompt_attention": attend} if attend is not None else {}),
                   "workgroups_per_unit": g.decode_plan(wl.batch * wl.n_kv_heads if args.per_layer else
                                                       (nl - args.keep_all_layers) * wl.batch * wl.n_kv_heads
                                                       if 0 < args.keep_all_layers < nl else None)[0],
                   **({"phase_clocks_us": phases} if phases is not None else {}),
                   "pct_hbm_roofline": 100.0 * achieved / HBM_PEAK_GBS},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_src,
                     "stream_read_GBs": stream_gbs,
                     "frac_of_stream_read": (achieved / stream_gbs) if stream_gbs else None,
                     "kernel": "decode_fused_kernel" + (" + decode_split_kernel" if args.keep_all_layers else ""),
                     "algorithmic_bytes_per_launch": A * K_steps // launches,
                     "avg_launch_us": sec / launches * 1e6},
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl, Qw, K, V, lambda t: dec_inputs(step_no + t))
    print(json.dumps(res))


if __name__ == "__main__":
    main()
