#!/usr/bin/env python3
"""Writes the tracked result tables of this directory from the JSON lines that bench.py printed.

    python results/make_tables.py five  <title> <out.md> <bench line files, one per seed ...>
    python results/make_tables.py sweep <title> <out.md> <files of `bench.py --sweep` lines ...>

`five`: one row per seed (best-found TFLOP/s after the trial budget, fraction of the MFMA peak, trials to
the best and to 99 % of it, tuning wall time and its compile share, kernels built ahead, invalid trials,
parity failures, best configuration) and a mean +- std row.  `sweep`: one row per setting, mean +- std over
the seeds of the best-found TFLOP/s after 50 / 100 / 200 / ... trials.  Nothing here touches a GPU.
"""
import json
import sys

import numpy as np


def lines_of(paths):
    for path in paths:
        for line in open(path):
            line = line.strip()
            if line.startswith("{"):
                try:
                    yield json.loads(line)
                except ValueError:
                    pass


def five(title, out, paths):
    runs = sorted(lines_of(paths), key=lambda j: j["config"]["seed"])
    assert runs, "no bench lines found"
    c0 = runs[0]["config"]
    rows = ["# %s" % title, "",
            "`python bench.py --workload %s --seed S` (space %s, %d trials, lambda = rho = 8, q = 0.5), one JSON line per seed; "
            "this table: `python results/make_tables.py five ...`." % (c0["workload"].split()[0], c0["space"], c0["trials"]), "",
            "| seed | best TFLOP/s | of MFMA peak | best kernel, ms | trials to best | to 99 % | tuning wall s | compile s | built ahead | invalid | parity failures | MFMA-only ceiling (random operands) | best configuration |",
            "|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
    for j in runs:
        c, r = j["config"], j["roofline"]
        rows.append("| %d | %.1f | %.1f %% | %.5f | %d | %d | %.1f | %.1f | %s | %d | %d | %s | `%s` |" % (
            c["seed"], j["value"], 100 * c["frac_of_peak"], r["kernel_ms"], c["trials_to_best"], c["trials_to_99pct"],
            c["tuning_wall_s"], c["compile_s"], c.get("n_built_ahead", "-"), c["n_invalid"], c["n_parity_fail"],
            r.get("mfma_only_ceiling"), " ".join(map(str, c["best_cfg"]))))
    v = np.array([j["value"] for j in runs])
    tb = np.array([j["config"]["trials_to_best"] for j in runs])
    t99 = np.array([j["config"]["trials_to_99pct"] for j in runs])
    wall = np.array([j["config"]["tuning_wall_s"] for j in runs])
    rows.append("| mean +- std | %.1f +- %.1f | %.1f %% | | %.0f +- %.0f | %.0f +- %.0f | %.1f +- %.1f | | | | %d of %d | | |" % (
        v.mean(), v.std(), 100 * v.mean() / (runs[0]["roofline"]["peak"] if runs[0]["roofline"]["bound"] == "mfma" else 2500.0),
        tb.mean(), tb.std(), t99.mean(), t99.std(), wall.mean(), wall.std(),
        sum(j["config"]["n_parity_fail"] for j in runs), sum(j["config"]["trials"] for j in runs)))
    open(out, "w").write("\n".join(rows) + "\n")


def sweep(title, out, paths):
    summ = [j for j in lines_of(paths) if "mean_best_after" in j]
    runs = [j for j in lines_of(paths) if "best_after" in j]
    assert summ, "no sweep summary lines found"
    rows = ["# %s" % title, "",
            "`python bench.py --sweep --workload W --trials T` (every run parity-gated against the oracle's reference); "
            "best-found TFLOP/s, mean +- std over the seeds; this table: `python results/make_tables.py sweep ...`.", ""]
    for wl in sorted({(j["workload"], j.get("space", "default")) for j in summ}):
        mine = [j for j in summ if (j["workload"], j.get("space", "default")) == wl]
        marks = list(mine[0]["mean_best_after"].keys())
        fails = sum(j.get("n_parity_fail", 0) for j in runs if (j["workload"], j.get("space", "default")) == wl)
        n_runs = sum(1 for j in runs if (j["workload"], j.get("space", "default")) == wl)
        rows += ["## %s (space %s), seeds %s; %d runs, %d parity failures" % (wl[0], wl[1], mine[0]["seeds"], n_runs, fails), "",
                 "| setting | " + " | ".join("after %s" % m for m in marks) + " |", "|---|" + "---|" * len(marks)]
        for j in mine:
            rows.append("| %s | " % j["setting"] + " | ".join("%.0f +- %.0f" % (j["mean_best_after"][m], j["std_best_after"][m]) for m in marks) + " |")
        rows.append("")
    open(out, "w").write("\n".join(rows))


if __name__ == "__main__":
    kind, title, out, paths = sys.argv[1], sys.argv[2], sys.argv[3], sys.argv[4:]
    {"five": five, "sweep": sweep}[kind](title, out, paths)
