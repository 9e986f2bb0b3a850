"""The script that turns bench.py's JSON lines into the tracked tables of results/: its
means and standard deviations, on hand-made lines whose statistics are known."""
import importlib.util
import json
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _module():
    spec = importlib.util.spec_from_file_location("make_tables", os.path.join(ROOT, "results", "make_tables.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _bench_line(seed, value, to_best, to99, wall):
    return {"value": value,
            "config": {"workload": "mm8192_bf16 matmul dims=[8192, 8192, 8192]", "space": "TILE4", "trials": 1000,
                       "seed": seed, "frac_of_peak": value / 2500.0, "trials_to_best": to_best, "trials_to_99pct": to99,
                       "tuning_wall_s": wall, "compile_s": wall / 2, "n_built_ahead": 10, "n_invalid": 3, "n_parity_fail": 0,
                       "best_cfg": [32, 2, 2, 64, 32, 2, 2, 64, 256, 32, 1]},
            "roofline": {"bound": "mfma", "peak": 2500.0, "kernel_ms": 0.8, "mfma_only_ceiling": 1800.0}}


def test_five_seed_table_has_one_row_per_seed_and_the_right_statistics(tmp_path):
    mt = _module()
    paths = []
    for seed, value in enumerate([1000.0, 1100.0, 1200.0]):          # mean 1100, population std 81.6
        p = tmp_path / ("s%d.json" % seed)
        p.write_text("some log line\n" + json.dumps(_bench_line(seed, value, 100 * (seed + 1), 50, 60.0)) + "\n")
        paths.append(str(p))
    out = tmp_path / "t.md"
    mt.five("a title", str(out), paths[::-1])                         # order of the files does not matter
    text = out.read_text().splitlines()
    assert text[0] == "# a title"
    rows = [l for l in text if l.startswith("| ") and not l.startswith("| seed")]
    assert [r.split("|")[1].strip() for r in rows] == ["0", "1", "2", "mean +- std"]
    assert "1100.0 +- 81.6" in rows[-1] and "44.0 %" in rows[-1] and "200 +- 82" in rows[-1] and "0 of 3000" in rows[-1]


def test_sweep_table_groups_settings_by_workload_and_counts_parity_failures(tmp_path):
    mt = _module()
    p = tmp_path / "sweep.jsonl"
    lines = []
    for seed in (0, 1):
        lines.append({"workload": "mm1_bf16", "space": "default", "setting": "q=0.5 lambda=8", "seed": seed, "trials": 100,
                      "best_after": {"50": 10.0 + seed, "100": 20.0}, "n_invalid": 1, "n_parity_fail": seed, "wall_s": 1.0})
    lines.append({"workload": "mm1_bf16", "space": "default", "setting": "q=0.5 lambda=8", "seeds": [0, 1],
                  "mean_best_after": {"50": 10.6, "100": 20.0}, "std_best_after": {"50": 0.7, "100": 0.0}})
    p.write_text("\n".join(json.dumps(l) for l in lines) + "\n")
    out = tmp_path / "s.md"
    mt.sweep("sweeps", str(out), [str(p)])
    text = out.read_text()
    assert "## mm1_bf16 (space default), seeds [0, 1]; 2 runs, 1 parity failures" in text
    assert "| q=0.5 lambda=8 | 11 +- 1 | 20 +- 0 |" in text
