#!/usr/bin/env python3
"""Turns rocprofv3 output into the short summaries under profiles/.

    python profile_summary.py c2 c5a ...        # reads <RESULTS>/prof_<layer>/, writes profiles/<layer>_<kernel>.md
    python profile_summary.py --sq c2 c5a ...   # reads <RESULTS>/prof_<layer>/sq/, writes profiles/sq_lds_counters_all_layers.md
    python profile_summary.py --commands c2     # prints the rocprofv3 commands whose output it expects

Per layer it expects four runs of bench.py under rocprofv3 (each its own run; counters are never
combined with tracing), started from the repository root with TMPDIR=/tmp:

    trace/  --kernel-trace --stats                 kernel durations
    fetch/  --pmc FETCH_SIZE   (with --calibration-copy: a 256 MiB copy of known traffic fixes the counter's scale)
    write/  --pmc WRITE_SIZE   (likewise)
    sq/     --pmc eight SQ counters                matrix-pipe and LDS activity

It also keeps profiles/pmc_traffic.json (measured HBM bytes per launch), which bench.py quotes as
`roofline.traffic`.
"""
from __future__ import annotations

import glob
import json
import os
import sqlite3
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
import workloads as wl  # noqa: E402

RESULTS = "gpurun_out"             # folder (under the repository root) the profiling runs write into
COPY_KIB = 256 * 1024
SQ_COUNTERS = ("SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_LDS_ADDR_CONFLICT SQ_LDS_UNALIGNED_STALL "
               "SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_ACTIVE_INST_LDS SQ_WAIT_INST_LDS")


def commands(name):
    d = "%s/prof_%s" % (RESULTS, name)
    b = "python3 bench.py --workload %s --no-layers --no-cpu" % name
    return [
        "rocprofv3 --kernel-trace --stats -d %s/trace -o trace -- %s --steps 500 --warmup 5" % (d, b),
        "rocprofv3 --pmc FETCH_SIZE -d %s/fetch -o fetch -- %s --steps 50 --warmup 2 --calibration-copy" % (d, b),
        "rocprofv3 --pmc WRITE_SIZE -d %s/write -o write -- %s --steps 50 --warmup 2 --calibration-copy" % (d, b),
        "rocprofv3 --pmc %s -d %s/sq -o sq -- %s --steps 20 --warmup 2" % (SQ_COUNTERS, d, b),
    ]


def q(db, sql):
    c = sqlite3.connect(db)
    r = c.execute(sql).fetchall()
    c.close()
    return r


def one_db(d, sub):
    found = glob.glob(os.path.join(d, sub, "**", "*.db"), recursive=True)
    if not found:
        raise SystemExit("no rocprofv3 database under %s/%s (run: %s)" % (d, sub, "; ".join(commands(os.path.basename(d)[5:]))))
    return found[0]


def summarise(name):
    d = os.path.join(ROOT, RESULTS, "prof_" + name)
    w = wl.WORKLOADS[name]
    tdb, fdb, wdb = one_db(d, "trace"), one_db(d, "fetch"), one_db(d, "write")
    top = q(tdb, "select name,total_calls,total_duration,average,percentage from top_kernels")
    conv = [r for r in top if "cvx::" in r[0]][0]
    kname = conv[0]
    dur = q(tdb, "select count(*), avg(duration), min(duration), max(duration) from kernels where name='%s'" % kname)[0]
    allv = [r[0] for r in q(tdb, "select duration from kernels where name='%s' order by start" % kname)]
    steady = allv[len(allv) // 4:]
    steady_avg = sum(steady) / len(steady)
    bench = json.loads(open(os.path.join(d, "trace_stdout.json")).read().strip().splitlines()[-1])

    def counter(db, cn):
        conv_v = q(db, "select avg(value),min(value),max(value),count(*) from counters_collection where kernel_name='%s' and counter_name='%s'" % (kname, cn))[0]
        copy_v = q(db, "select max(value) from counters_collection where kernel_name like '%%copyBuffer%%' and counter_name='%s'" % cn)[0][0]
        return conv_v, copy_v

    (f_avg, f_min, f_max, f_n), f_copy = counter(fdb, "FETCH_SIZE")
    (w_avg, w_min, w_max, w_n), w_copy = counter(wdb, "WRITE_SIZE")
    f_scale, w_scale = COPY_KIB / f_copy, COPY_KIB / w_copy
    fetch_b, write_b = f_avg * f_scale * 1024, w_avg * w_scale * 1024
    traffic = fetch_b + write_b
    short = kname.split("(")[0].replace("void ", "").replace("cvx::", "")
    variant = bench["config"]["kernel"]
    cmds = commands(name)
    out = os.path.join(ROOT, "profiles", "%s_%s.md" % (name, variant))
    for old in glob.glob(os.path.join(ROOT, "profiles", "%s_*.md" % name)):
        os.remove(old)                       # one summary per layer: the kernel that serves it now
    os.makedirs(os.path.dirname(out), exist_ok=True)
    rf = bench["roofline"]
    with open(out, "w") as fo:
        fo.write("""# rocprofv3 summary: workload %s, kernel variant %s

Workload: %s
Device kernel: `%s` (one launch per cvx_conv_fwd_fused call), MI355X (gfx950), rotating buffer sets = %d.
Written by `python profile_summary.py %s` from the output of the commands below.

## Kernel trace

Command (run from the repository root on the GPU box, `TMPDIR=/tmp`):

    %s

| kernel | calls | avg us | min us | max us | steady-state avg us (last 75 %% of launches) |
|---|---|---|---|---|---|
| %s | %d | %.3f | %.3f | %.3f | %.3f |

bench.py in the same run (HIP events around the graph replays): %.3f us per step,
%.1f %s = %.1f %% of the %s peak (%s %s).  Plain calls without a graph: %s us per step.

Top kernels of the run (name, calls, total us, avg us, %% of GPU time):

""" % (name, variant, bench["config"]["workload"], short, bench["config"]["buffer_sets"], name, cmds[0],
            short, dur[0], dur[1] / 1e3, dur[2] / 1e3, dur[3] / 1e3, steady_avg / 1e3,
            bench["event_ms_per_step"] * 1e3, rf["achieved"], rf["unit"], rf["frac"] * 100, rf["bound"], rf["peak"], rf["unit"],
            "%.3f" % bench["eager_us_per_step"] if bench.get("eager_us_per_step") else "n/a"))
        for r in top[:4]:
            fo.write("    %s  %d  %.1f  %.3f  %.2f\n" % (r[0][:100], r[1], r[2] / 1e3, r[3] / 1e3, r[4]))
        fo.write("""
## HBM traffic (one counter per run)

    %s
    %s

`--calibration-copy` runs one plain 256 MiB device-to-device copy in the same process; the counter's reading for
that copy fixes the scale (KiB of real traffic per counter unit).

| counter | conv kernel, per dispatch (avg / min / max over %d dispatches) | 256 MiB copy reads | scale | conv kernel bytes per launch |
|---|---|---|---|---|
| FETCH_SIZE | %.1f / %.1f / %.1f | %.1f | %.3f | %.2f MB |
| WRITE_SIZE | %.1f / %.1f / %.1f | %.1f | %.3f | %.2f MB |

Measured HBM traffic per launch: %.2f MB; algorithmic bytes (each input, filter and bias element read once,
each output element written once): %.2f MB; ratio %.3f.
""" % (cmds[1], cmds[2], f_n, f_avg, f_min, f_max, f_copy, f_scale, fetch_b / 1e6,
            w_avg, w_min, w_max, w_copy, w_scale, write_b / 1e6, traffic / 1e6, w.algorithmic_bytes / 1e6,
            traffic / w.algorithmic_bytes))
    tj = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    t = json.load(open(tj)) if os.path.exists(tj) else {}
    t[name] = round(traffic)
    json.dump(t, open(tj, "w"), indent=1, sort_keys=True)
    print("%s: kernel avg %.2f us (steady %.2f), traffic %.2f MB vs algorithmic %.2f MB"
          % (out, dur[1] / 1e3, steady_avg / 1e3, traffic / 1e6, w.algorithmic_bytes / 1e6))


def summarise_sq(names):
    rows = []
    for name in names:
        db = one_db(os.path.join(ROOT, RESULTS, "prof_" + name), "sq")
        vals = {}
        kernel = None
        for k, cn, v in q(db, "select kernel_name, counter_name, avg(value) from counters_collection "
                              "where kernel_name like '%cvx::%' group by kernel_name, counter_name"):
            kernel = k.split("(")[0].replace("void ", "").replace("cvx::", "")
            vals[cn] = v
        rows.append((name, kernel, vals))
    out = os.path.join(ROOT, "profiles", "sq_lds_counters_all_layers.md")
    with open(out, "w") as fo:
        fo.write("""# rocprofv3 SQ counters: matrix-pipe and LDS activity of the convolution kernels

Command, once per layer (run from the repository root on the GPU box, `TMPDIR=/tmp`; one pass, eight SQ counters):

    %s

Averages per dispatch of the convolution kernel (counter values are summed over the shader engines as rocprofv3
reports them).  Written by `python profile_summary.py --sq %s`.

| layer | kernel | SQ_BUSY_CYCLES | MFMA_BUSY_CYCLES | LDS_IDX_ACTIVE | LDS_BANK_CONFLICT | bank-conflict cycles / LDS active cycles | ACTIVE_INST_LDS | WAIT_INST_LDS |
|---|---|---|---|---|---|---|---|---|
""" % (commands("<layer>")[3], " ".join(names)))
        for name, kernel, v in rows:
            act = v.get("SQ_LDS_IDX_ACTIVE", 0.0)
            fo.write("| %s | `%s` | %.0f | %.0f | %.0f | %.0f | %.3f | %.0f | %.0f |\n"
                     % (name, kernel, v.get("SQ_BUSY_CYCLES", 0), v.get("SQ_VALU_MFMA_BUSY_CYCLES", 0), act,
                        v.get("SQ_LDS_BANK_CONFLICT", 0), v.get("SQ_LDS_BANK_CONFLICT", 0) / act if act else 0.0,
                        v.get("SQ_ACTIVE_INST_LDS", 0), v.get("SQ_WAIT_INST_LDS", 0)))
        fo.write("\nSQ_LDS_ADDR_CONFLICT and SQ_LDS_UNALIGNED_STALL: %s.\n"
                 % ", ".join("%s %.0f / %.0f" % (n, v.get("SQ_LDS_ADDR_CONFLICT", 0), v.get("SQ_LDS_UNALIGNED_STALL", 0)) for n, _, v in rows))
    print(out)


def main():
    args = sys.argv[1:]
    if not args:
        raise SystemExit(__doc__)
    if args[0] == "--commands":
        for n in args[1:]:
            print("\n".join(commands(n)))
        return
    if args[0] == "--sq":
        summarise_sq(args[1:])
        return
    for n in args:
        summarise(n)


if __name__ == "__main__":
    main()
