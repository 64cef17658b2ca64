"""Turns a rocprofv3 results database (rocpd sqlite) into the few lines kept under profiles/.

  python profile_summary.py trace  <results.db> <n_last>   # --kernel-trace runs
  python profile_summary.py pmc    <results.db> <n_last>   # --pmc runs
  python profile_summary.py kernels <results.db> <n_last>  # every kernel of the library

Only the library's kernels are looked at; <n_last> = how many of the last decode dispatches form the
steady-state sample (the timed region of bench.py).
"""
import sqlite3
import statistics as st
import sys
from collections import defaultdict


def trace(db, nlast):
    c = sqlite3.connect(db)
    rows = list(c.execute(
        "select name,start,end,duration,grid_x,workgroup_x,lds_size,vgpr_count,accum_vgpr_count,scratch_size "
        "from kernels where name like '%decode_fused_kernel%' or name like '%decode_split_kernel%' order by start"))
    last = rows[-nlast:]
    d = [r[3] / 1e3 for r in last]
    gaps = [(last[i + 1][1] - last[i][2]) / 1e3 for i in range(len(last) - 1)]
    print(f"kernel: {last[0][0]}")
    print(f"grid_x(threads)={last[0][4]} workgroup={last[0][5]} lds_bytes={last[0][6]} vgpr={last[0][7]} "
          f"agpr={last[0][8]} scratch={last[0][9]}")
    print(f"dispatches total={len(rows)}; steady-state sample = last {nlast} dispatches (the timed region)")
    print(f"duration us: mean={st.mean(d):.2f} median={st.median(d):.2f} min={min(d):.2f} max={max(d):.2f}")
    print(f"start-to-start period us: mean={st.mean([(last[i + 1][1] - last[i][1]) / 1e3 for i in range(len(last) - 1)]):.2f}")
    print(f"gap between consecutive dispatches us: mean={st.mean(gaps):.2f} median={st.median(gaps):.2f}")


def pmc(db, nlast):
    c = sqlite3.connect(db)
    rows = c.execute(
        "select name, counter_name, dispatch_id, sum(counter_value), max(duration) from pmc_events "
        "where name like '%decode_fused%' or name like '%decode_split%' or name like '%decode_keep%' or name like '%calib_copy%' "
        "group by name, counter_name, dispatch_id order by dispatch_id")
    d = defaultdict(list)
    for name, cn, did, val, dur in rows:
        d[(name.split('(')[0][-60:], cn)].append((did, val, dur))
    for (name, cn), v in sorted(d.items()):
        v = v[-nlast:] if 'decode' in name else v
        vals = [x[1] for x in v]
        durs = [x[2] / 1e3 for x in v]
        print(f"{name:60s} {cn:24s} dispatches={len(v):5d} mean={st.mean(vals):.1f} min={min(vals):.1f} "
              f"max={max(vals):.1f} mean_dur_us={st.mean(durs):.2f}")


def kernels(db, nlast):
    """Every kernel of the library: calls, and duration over the last <n_last> calls of each (the first
    call of a process pays code loading and cold caches)."""
    c = sqlite3.connect(db)
    d = defaultdict(list)
    for name, start, dur in c.execute("select name, start, duration from kernels where name like '%mkv::%' order by start"):
        d[name.split('(')[0][-70:]].append(dur / 1e3)
    tot = 0.0
    for name, v in sorted(d.items(), key=lambda kv: -st.mean(kv[1][-nlast:])):
        w = v[-nlast:]
        tot += st.mean(w)
        print(f"{name:70s} calls={len(v):5d} last{len(w)}: mean_us={st.mean(w):9.1f} min_us={min(w):9.1f}")
    print(f"sum of the means: {tot:.1f} us")


if __name__ == "__main__":
    {"trace": trace, "pmc": pmc, "kernels": kernels}[sys.argv[1]](sys.argv[2], int(sys.argv[3]))
