"""Turns rocprofv3 result databases into the short text summaries kept under profiles/.  CPU only.

    # per-kernel calls / total / mean duration of a run made with `rocprofv3 --kernel-trace --stats -d DIR -o NAME -- ...`
    python -m paper_2510_19705_amd.profsum trace DIR/NAME_results.db --cmd "<the command>" --out profiles/<file>.txt [--by-grid]

    # HBM bytes per launch of the layer kernels, from two runs of `workloads --config counters` (one with
    # `--pmc FETCH_SIZE --kernel-trace`, one with `--pmc WRITE_SIZE --kernel-trace`) and the manifest that workload printed
    python -m paper_2510_19705_amd.profsum traffic --fetch F_results.db --write W_results.db --manifest manifest.json \
        --cmd "<the command>" --out profiles/<file>.txt

The traffic summary scales both counters by what they read for a plain element-wise kernel of known size in the same
run (the factor is printed) and ends each layer site with a `traffic_bytes_per_launch_<site>: N kernel=<instance> rows=R`
line, which bench.py quotes only if it timed the same kernel instance at the same row count.
"""
import argparse
import json
import sqlite3


def _tables(cur):
    return [r[0] for r in cur.execute("select name from sqlite_master where type in ('table', 'view')")]


def trace(db, cmd, out, note="", by_grid=False):
    """by_grid: one line per (kernel, launch shape) instead of per kernel, so that launches of one template instance
    on matrices of different sizes (the same instance serves every model of a hierarchy) are told apart."""
    cur = sqlite3.connect(db).cursor()
    if by_grid:
        cols = [r[1] for r in cur.execute("pragma table_info(kernels)")]
        gx = "grid_x" if "grid_x" in cols else ("grid_size_x" if "grid_size_x" in cols else None)
        wx = "workgroup_x" if "workgroup_x" in cols else ("workgroup_size_x" if "workgroup_size_x" in cols else None)
        if gx is None or wx is None:
            raise SystemExit("no grid / workgroup columns in the kernels view: %s" % cols)
        gy, wy = gx.replace("_x", "_y"), wx.replace("_x", "_y")
        agg = {}
        for n, st, en, a, b, c, d in cur.execute("select name, start, end, %s, %s, %s, %s from kernels" % (gx, gy, wx, wy)):
            # the profiler reports the grid in work-items: workgroups = items / workgroup size
            key = (n, "%dx%d" % (a // max(1, c), b // max(1, d)))
            e = agg.setdefault(key, [0, 0.0])
            e[0] += 1
            e[1] += (en - st) / 1e3
        total = sum(v[1] for v in agg.values())
        rows = [("%s [%s workgroups]" % (k[0].replace("bool _Accum", "bf16").replace("(anonymous namespace)::", "").split("(")[0], k[1]),
                 v[0], v[1], v[1] / v[0], 100 * v[1] / total)
                for k, v in sorted(agg.items(), key=lambda kv: -kv[1][1])]
    else:
        rows = list(cur.execute("select name, total_calls, total_duration, average, percentage from top_kernels"))
    with open(out, "w") as f:
        f.write("rocprofv3 --kernel-trace --stats summary (durations in microseconds)\n")
        f.write("command: %s\n" % cmd)
        if note:
            f.write(note + "\n")
        f.write("%-96s %9s %14s %10s %7s\n" % ("kernel", "calls", "total_us", "avg_us", "pct"))
        for n, c, t, a, p in rows:
            n = n.replace("bool _Accum", "bf16")
            f.write("%-96s %9d %14.1f %10.3f %7.2f\n" % (n[:96], c, t, a, p))
    return open(out).read()


def _counter_rows(db):
    """[(kernel name, dispatch id, counter value)] in dispatch order."""
    cur = sqlite3.connect(db).cursor()
    return list(cur.execute("select kernel_name, dispatch_id, value from counters_collection order by dispatch_id"))


def traffic(fetch_db, write_db, manifest, cmd, out):
    man = json.load(open(manifest))
    f_rows, w_rows = _counter_rows(fetch_db), _counter_rows(write_db)
    ref_kib = man["reference_MiB_each_way"] * 1024

    def mean_of(rows, pred):
        # the reference launches are the largest of their kind (weight initialisation uses the same element-wise
        # kernels on small tensors)
        v = [val for name, _, val in rows if pred(name)]
        v = [x for x in v if x >= 0.5 * max(v)] if v else v
        return (len(v), sum(v) / len(v)) if v else (0, 0.0)

    is_ref = lambda n: "vectorized_elementwise_kernel" in n and "add" in n.lower()
    nf, rf = mean_of(f_rows, is_ref)
    nw, rw = mean_of(w_rows, is_ref)
    if not nf or not nw:
        raise SystemExit("reference kernel not found in the counter databases")
    sf, sw = ref_kib / rf, ref_kib / rw
    lines = ["HBM traffic per launch from rocprofv3 hardware counters (%s-shaped layers: %s, bf16; %d rows per pass, %d cached positions)"
             % (man["shape"], ", ".join("%s %s" % (k, v) for k, v in man["shape_dims"].items() if k != "n_layers"), man["rows"], man["ctx"]),
             "commands (two runs, one counter each; both run committed files only):"]
    lines += ["  " + c for c in cmd.split(" ;; ")]
    lines.append("scale reference: %s over %d MiB (reads %d KiB, writes %d KiB): FETCH_SIZE read %.1f -> factor %.4f, WRITE_SIZE read %.1f -> factor %.4f"
                 % (man["reference_kernel"], man["reference_MiB_each_way"], ref_kib, ref_kib, rf, sf, rw, sw))
    lines.append("%-44s %-10s %6s %14s %14s %14s %8s" % ("kernel", "site", "calls", "fetch_bytes", "write_bytes", "algorithmic", "ratio"))
    sites = man["sites"]
    # sites that share one kernel instance are told apart by their order inside a layer
    by_kernel = {}
    for site in man["order_within_layer"] + ["head"]:
        by_kernel.setdefault(sites[site]["kernel"], []).append(site)
    for kernel, group in by_kernel.items():
        match = lambda n: kernel in n.replace("bool _Accum", "bf16")
        fv = [val for name, _, val in f_rows if match(name)]
        wv = [val for name, _, val in w_rows if match(name)]
        # the last launches of the run are the ten measured passes (earlier ones: the prefill, at other row counts)
        want = sum(sites[s]["launches"] for s in group)
        fv, wv = fv[-want:], wv[-want:]
        if len(fv) < want or len(wv) < want:
            lines.append("%-44s %-10s   not found in the databases" % (kernel, "/".join(group)))
            continue
        for i, site in enumerate(group):
            # within a pass the group's sites alternate in layer order; the head (one launch per pass) never shares
            if len(group) == 1:
                fs, ws = fv, wv
            else:
                fs, ws = fv[i::len(group)], wv[i::len(group)]
            fb, wb = sum(fs) / len(fs) * sf * 1024, sum(ws) / len(ws) * sw * 1024
            alg = sites[site]["algorithmic_bytes"]
            lines.append("%-44s %-10s %6d %14.0f %14.0f %14.0f %8.3f" % (kernel, site, len(fs), fb, wb, alg, (fb + wb) / alg))
            lines.append("traffic_bytes_per_launch_%s: %d kernel=%s rows=%d" % (site, round(fb + wb), kernel, man["rows"]))
    with open(out, "w") as f:
        f.write("\n".join(lines) + "\n")
    return open(out).read()


def gap(db, report, plain_report, cmd, out):
    """Kernel-busy share of the generations that `workloads --config launch-gap` brackets with two marker launches.
    report: what the workload printed in the profiled run; plain_report: what it printed without the profiler (the
    profiler slows the host's launches, so wall-clock and the graph-replay comparison are quoted from the plain run)."""
    rep = json.load(open(report))
    plain = json.load(open(plain_report))
    cur = sqlite3.connect(db).cursor()
    rows = list(cur.execute("select name, start, end from kernels order by start"))
    marks = [i for i, r in enumerate(rows) if rep["marker_kernel"] in r[0]]
    if len(marks) < 2:
        raise SystemExit("marker launches not found")
    a, b = marks[-2], marks[-1]
    inside = rows[a + 1:b]
    window = (rows[b][1] - rows[a][2]) / 1e3
    busy = sum(e - st for _, st, e in inside) / 1e3
    n = rep["generations_between_markers"]
    per = {}
    for name, st, e in inside:
        k = name.replace("bool _Accum", "bf16").replace("(anonymous namespace)::", "").split("(")[0].replace("void ", "")
        c = per.setdefault(k, [0, 0.0])
        c[0] += 1
        c[1] += (e - st) / 1e3
    lines = ["Kernel-busy share of a generation step on small models (durations in microseconds)",
             "workload: %s; %d generations between the two marker launches" % (rep["workload"], n),
             "command: %s" % cmd,
             "per generation: window %.1f (the workload's own wall-clock under the profiler: %.1f), kernels %.1f = %.1f %% busy; %d launches, mean gap "
             "between launches %.2f" % (window / n, rep["wall_ms_per_generation"] * 1e3, busy / n, 100 * busy / window, len(inside) // n,
                                        (window - busy) / max(1, len(inside))),
             "%-60s %9s %12s %9s %7s" % ("kernel", "launches", "total_us", "avg_us", "pct of window")]
    for k, (c, t) in sorted(per.items(), key=lambda kv: -kv[1][1]):
        lines.append("%-60s %9d %12.1f %9.2f %7.2f" % (k[:60], c // n, t / n, t / c, 100 * t / window))
    lines.append("without the profiler: wall-clock per generation %.1f (%.1f tokens/s): the kernel time above is %.1f %% of it, i.e. the kernels run back "
                 "to back and what separates them is the dispatch of each dependent launch, inside the durations the trace reports"
                 % (plain["wall_ms_per_generation"] * 1e3, plain["tokens_per_s"], 100 * busy / n / (plain["wall_ms_per_generation"] * 1e3)))
    lines.append("one pass issued directly / replayed from a HIP graph of the same launches / host time to enqueue it (plain run):")
    for label, r in plain["graph_replay"].items():
        lines.append("  %-14s direct %.1f  graph replay %.1f  host enqueue %.1f  (replay wrote the same logits: %s)"
                     % (label, r["direct_us"], r["graph_replay_us"], r["host_enqueue_us"], r["same_logits"]))
    with open(out, "w") as f:
        f.write("\n".join(lines) + "\n")
    return open(out).read()


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    t = sub.add_parser("trace")
    t.add_argument("db")
    t.add_argument("--cmd", required=True)
    t.add_argument("--note", default="")
    t.add_argument("--by-grid", action="store_true", help="one line per (kernel, launch shape)")
    t.add_argument("--out", required=True)
    c = sub.add_parser("traffic")
    c.add_argument("--fetch", required=True)
    c.add_argument("--write", required=True)
    c.add_argument("--manifest", required=True)
    c.add_argument("--cmd", required=True, help="the two commands, separated by ' ;; '")
    c.add_argument("--out", required=True)
    g = sub.add_parser("gap")
    g.add_argument("db")
    g.add_argument("--report", required=True, help="the JSON that workloads --config launch-gap printed in the same run")
    g.add_argument("--plain-report", required=True, help="the JSON of a run of the same workload without the profiler")
    g.add_argument("--cmd", required=True)
    g.add_argument("--out", required=True)
    args = ap.parse_args()
    if args.what == "gap":
        print(gap(args.db, args.report, args.plain_report, args.cmd, args.out))
        return
    if args.what == "trace":
        print(trace(args.db, args.cmd, args.out, args.note, args.by_grid))
    else:
        print(traffic(args.fetch, args.write, args.manifest, args.cmd, args.out))


if __name__ == "__main__":
    main()
