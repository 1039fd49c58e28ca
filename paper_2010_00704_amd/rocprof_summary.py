"""Turns rocprofv3 CSV output of a `bench.py` run into the short summaries kept
under profiles/.

    python -m paper_2010_00704_amd.rocprof_summary trace KERNEL_TRACE.csv --out FILE.md --command "..."
    python -m paper_2010_00704_amd.rocprof_summary counters COLLECTION.csv [MORE.csv ...] --out FILE.md --command "..."
    python -m paper_2010_00704_amd.rocprof_summary traffic FETCH.csv WRITE.csv --out FILE.md --command "..."

`trace` reads a `--kernel-trace` CSV, the other two read `--pmc` counter
collection CSVs (one run per counter set; rocprofv3 does not split counters
over passes).  A bench step launches the same kernels in the same order every
time (pack and convolution of each layer shape), so the dispatches at the end
of a run are cut into steps and averaged per position in the step: that keeps
apart layer shapes which share a kernel instance and a grid size.  Everything
before the steps (weight packing at set-up, the probes of `--probes`) is
averaged per kernel and grid.  `traffic` scales FETCH_SIZE / WRITE_SIZE by what
the same counters read for the copy probe of known size and writes, besides
the table, one `traffic_bytes_per_launch <shape> <bytes>` line per layer
shape, which `bench.py` reads for its roofline object.
"""
import argparse
import collections
import csv
import re
import sys

from . import workloads as W


def _short(name):
    name = re.sub(r"^(void )?bcnn::(\(anonymous namespace\)::)?", "", name)
    return re.sub(r"\((?:[^()]|\([^()]*\))*\)\s*$", "", name)


def _rows(path):
    """Dispatches of library kernels in launch order: dicts with name, grid, wg, start, end and the
    counters of that dispatch."""
    by_id = collections.OrderedDict()
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            if "bcnn::" not in r["Kernel_Name"]:
                continue
            did = int(r["Dispatch_Id"])
            d = by_id.get(did)
            if d is None:
                grid = r.get("Grid_Size") or r.get("Grid_Size_X")
                wg = r.get("Workgroup_Size") or r.get("Workgroup_Size_X")
                d = by_id[did] = {"name": _short(r["Kernel_Name"]), "grid": int(grid), "wg": int(wg),
                                  "us": (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3,
                                  "vgpr": r.get("VGPR_Count"), "agpr": r.get("Accum_VGPR_Count"),
                                  "lds": r.get("LDS_Block_Size"), "scratch": r.get("Scratch_Size"), "counters": {}}
            if "Counter_Name" in r:
                d["counters"][r["Counter_Name"]] = d["counters"].get(r["Counter_Name"], 0.0) + float(r["Counter_Value"])
    return [by_id[k] for k in sorted(by_id)]


def step_labels(shapes):
    labels = []
    for i in shapes:
        cfg = W.CONFIGS[i - 1]
        labels.append("pack cfg%d" % i)
        labels += ["conv cfg%d" % i if cfg.layers == 1 else "conv cfg%d L%d" % (i, l + 1) for l in range(cfg.layers)]
    return labels


def split_steps(rows, shapes):
    """(rows before the steps, [steps]) where every step is a list of len(step_labels) dispatches."""
    period = len(step_labels(shapes))
    sig = lambda w: [(d["name"], d["grid"]) for d in w]   # noqa: E731
    steps = []
    end = len(rows)
    while end - period >= 0 and (not steps or sig(rows[end - period:end]) == sig(steps[0])):
        steps.insert(0, rows[end - period:end])
        end -= period
    if len(steps) < 2:
        raise SystemExit("no repeating steps of %d launches at the end of the run: was it a bench.py run "
                         "with --no-aux on shapes %s?" % (period, shapes))
    return rows[:end], steps


def _stats(vals):
    return sum(vals) / len(vals), min(vals), max(vals)


def _kernel_cell(d):
    extra = "vgpr=%s agpr=%s lds=%s scratch=%s grid=%d wg=%d" % (d["vgpr"], d["agpr"], d["lds"], d["scratch"], d["grid"], d["wg"])
    return "`%s` %s" % (d["name"], extra)


def _header(title, command, notes):
    out = ["# " + title, "", "Command (on the MI355X box, from /tmp with TMPDIR=/tmp):", ""]
    out += ["    " + c for c in command]
    out += [""] + notes + [""]
    return out


def cmd_trace(args):
    rows = _rows(args.csv[0])
    before, steps = split_steps(rows, args.shapes)
    labels = step_labels(args.shapes)
    out = _header(args.title or "rocprofv3 kernel trace of `bench.py`", args.command,
                  ["Durations are End - Start of each dispatch, averaged per position in the step over the last %d "
                   "steps of the run (warm-up, graph replays and the evented pass launch the same kernels)." % len(steps)])
    out += ["| step part | kernel | calls | avg us | min us | max us |", "|---|---|---|---|---|---|"]
    total = 0.0
    for p, lab in enumerate(labels):
        avg, lo, hi = _stats([s[p]["us"] for s in steps])
        total += avg
        out.append("| %s | %s | %d | %.1f | %.1f | %.1f |" % (lab, _kernel_cell(steps[0][p]), len(steps), avg, lo, hi))
    out += ["", "Sum of the average kernel durations of one step: %.1f us." % total, ""]
    if before:
        out += ["Launches before the steps (set-up, probes), per kernel and grid:", "",
                "| kernel | calls | avg us |", "|---|---|---|"]
        groups = collections.OrderedDict()
        for d in before:
            groups.setdefault((d["name"], d["grid"]), []).append(d)
        for ds in groups.values():
            out.append("| %s | %d | %.1f |" % (_kernel_cell(ds[0]), len(ds), _stats([d["us"] for d in ds])[0]))
        out.append("")
    return out


def _merge_counter_runs(paths, shapes):
    """Per step position and per set-up kernel: counter name -> average, merged over runs."""
    labels = step_labels(shapes)
    per_pos = [collections.OrderedDict() for _ in labels]
    kernels = [None] * len(labels)
    us = [[] for _ in labels]
    before = collections.OrderedDict()
    for path in paths:
        pre, steps = split_steps(_rows(path), shapes)
        for p in range(len(labels)):
            kernels[p] = steps[0][p]
            us[p] += [s[p]["us"] for s in steps]
            for name in steps[0][p]["counters"]:
                per_pos[p][name] = _stats([s[p]["counters"][name] for s in steps])[0]
        for d in pre:
            g = before.setdefault((d["name"], d["grid"]), {"d": d, "us": [], "c": collections.OrderedDict()})
            g["us"].append(d["us"])
            for name, v in d["counters"].items():
                g["c"].setdefault(name, []).append(v)
    return labels, kernels, per_pos, us, before


def cmd_counters(args):
    labels, kernels, per_pos, us, before = _merge_counter_runs(args.csv, args.shapes)
    names = []
    for c in per_pos:
        names += [n for n in c if n not in names]
    out = _header(args.title or "rocprofv3 counters of `bench.py`", args.command,
                  ["Averages per dispatch and position in the step (one run per counter set; kernels run a few per "
                   "cent longer while counters are collected)."])
    out += ["| step part | kernel | us | " + " | ".join(names) + " |", "|---|---|---|" + "---|" * len(names)]
    for p, lab in enumerate(labels):
        out.append("| %s | %s | %.1f | %s |" % (lab, _kernel_cell(kernels[p]), _stats(us[p])[0],
                                                " | ".join("%.4g" % per_pos[p][n] if n in per_pos[p] else "" for n in names)))
    if before:
        out += ["", "Launches before the steps (set-up, probes), per kernel and grid:", "",
                "| kernel | calls | us | " + " | ".join(names) + " |", "|---|---|---|" + "---|" * len(names)]
        for g in before.values():
            out.append("| %s | %d | %.1f | %s |" % (_kernel_cell(g["d"]), len(g["us"]), _stats(g["us"])[0],
                                                    " | ".join("%.4g" % _stats(g["c"][n])[0] if n in g["c"] else "" for n in names)))
    out.append("")
    return out


def cmd_traffic(args):
    labels, kernels, per_pos, us, before = _merge_counter_runs(args.csv, args.shapes)
    copy = [g for (name, _), g in before.items() if name.startswith("diag_copy_kernel")]
    if not copy or "FETCH_SIZE" not in copy[0]["c"] or "WRITE_SIZE" not in copy[0]["c"]:
        raise SystemExit("the runs must include the copy probe (bench.py --probes) with FETCH_SIZE and WRITE_SIZE")
    copy_kib = args.copy_bytes / 1024.0
    f_fetch = copy_kib / _stats(copy[0]["c"]["FETCH_SIZE"])[0]
    f_write = copy_kib / _stats(copy[0]["c"]["WRITE_SIZE"])[0]
    out = _header(args.title or "HBM traffic per dispatch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) of `bench.py`",
                  args.command,
                  ["Counter values are KiB per dispatch, averaged per position in the step.",
                   "Calibration: the copy probe (`diag_copy_kernel`, %d bytes read and as many written) reads "
                   "FETCH_SIZE = %.0f KiB and WRITE_SIZE = %.0f KiB, so read bytes = FETCH_SIZE x %.3f and written "
                   "bytes = WRITE_SIZE x %.3f." % (args.copy_bytes, _stats(copy[0]["c"]["FETCH_SIZE"])[0],
                                                   _stats(copy[0]["c"]["WRITE_SIZE"])[0], f_fetch, f_write)])
    out += ["| step part | kernel | FETCH_SIZE KiB | read MB | WRITE_SIZE KiB | written MB |", "|---|---|---|---|---|---|"]
    machine = collections.OrderedDict()
    for p, lab in enumerate(labels):
        fk, wk = per_pos[p]["FETCH_SIZE"], per_pos[p]["WRITE_SIZE"]
        rd, wr = fk * f_fetch * 1024, wk * f_write * 1024
        out.append("| %s | %s | %.0f | %.2f | %.0f | %.2f |" % (lab, _kernel_cell(kernels[p]), fk, rd / 1e6, wk, wr / 1e6))
        if lab.startswith("conv cfg"):
            index = int(lab[8])
            machine.setdefault(W.CONFIGS[index - 1].name, []).append(rd + wr)
    out += ["", "Read by bench.py (HBM bytes per convolution launch, read + written, averaged over the layers of a chain):", ""]
    for name, vals in machine.items():
        out.append("traffic_bytes_per_launch %s %.0f" % (name, sum(vals) / len(vals)))
    out.append("")
    return out


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("mode", choices=["trace", "counters", "traffic"])
    ap.add_argument("csv", nargs="+")
    ap.add_argument("--out", required=True)
    ap.add_argument("--command", action="append", default=[], help="the full command of a run (repeatable)")
    ap.add_argument("--title")
    ap.add_argument("--append", action="store_true", help="add to the file instead of replacing it")
    ap.add_argument("--shapes", default="1,2,3,4,5")
    ap.add_argument("--copy-bytes", type=int, default=64 << 20, help="size of the copy probe's buffer")
    args = ap.parse_args(argv)
    args.shapes = [int(v) for v in args.shapes.split(",")]
    lines = {"trace": cmd_trace, "counters": cmd_counters, "traffic": cmd_traffic}[args.mode](args)
    with open(args.out, "a" if args.append else "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", args.out)


if __name__ == "__main__":
    main(sys.argv[1:])
