#!/usr/bin/env python3
"""Hyperparameter sensitivity of OpEvo on one MI355X (Sec. 5.5 of the paper: mutation rate q and
parent size lambda), with two controls: Alg. 1 with a mutation that ignores the parameter graphs
(per parameter, with probability p, a uniformly random value: a plain evolutionary algorithm) and
uniform random search without replacement.

Every setting runs `--trials` trials of Alg. 1 through `opevo_tune` for each seed; the control is
the same call with lambda = trials, i.e. the whole budget is the initial, uniformly random
generation.  One JSON line per run (best-found TFLOP/s after 50, 100, 200, ... trials), then one
summary line per setting (mean and standard deviation over the seeds).

    python paper_2006_05664_amd/sweep.py --workload mm1_bf16 --trials 400 --seeds 0,1,2
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="mm1_bf16")
    ap.add_argument("--trials", type=int, default=400)
    ap.add_argument("--seeds", default="0,1,2")
    ap.add_argument("--q", default="0.1,0.3,0.5,0.7,0.9", help="mutation rates tried at lambda = rho = 8")
    ap.add_argument("--lam", default="4,16,32", help="parent sizes tried at q = 0.5 (rho = 8)")
    ap.add_argument("--uniform-mutation", default="0.3,0.5", help="per-parameter resampling probabilities of the plain-EA control")
    ap.add_argument("--variant", default=None, help="TILE4 (default for 16-bit inputs), TILE4X, TILE4P or TILE4K")
    args = ap.parse_args()

    import numpy as np
    import paper_2006_05664_amd as P
    from paper_2006_05664_amd import synth
    P.opevo_compile_pool_start(8)
    import torch

    assert torch.cuda.is_available(), "sweep.py needs the GPU"
    w = synth.WORKLOADS[args.workload]
    kind = {"matmul": P.OPEVO_MATMUL, "bmm": P.OPEVO_BMM, "bmm_ta": P.OPEVO_BMM_TA, "conv2d": P.OPEVO_CONV2D}[w["kind"]]
    dtype = w["dtype"]
    variant = P.OPEVO_TILE2 if args.workload == "mm64_f32" else P.OPEVO_TILE4
    if args.variant:
        variant = {"TILE2": P.OPEVO_TILE2, "TILE4": P.OPEVO_TILE4, "TILE4X": P.OPEVO_TILE4X, "TILE4P": P.OPEVO_TILE4P,
                   "TILE4K": P.OPEVO_TILE4K}[args.variant]
    op = P.opevo_op_create(kind, w["dims"], synth.DTYPE_CODE[dtype])
    flops = P.opevo_op_flops(op)
    a_host, b_host = synth.workload_inputs(args.workload)
    da, db = synth.to_device(a_host, dtype), synth.to_device(b_host, dtype)
    dc = torch.empty(P.opevo_op_sizes(op)[2], dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    timeout_ms = max(10.0, 100.0 * flops / (2.0 * 8192.0 ** 3))
    seeds = [int(s) for s in args.seeds.split(",")]
    marks = [m for m in (50, 100, 200, 300, 400, 500, 750, 1000) if m <= args.trials]

    settings = [("q=%s lambda=8" % q, float(q), 8) for q in args.q.split(",") if q]
    settings += [("q=0.5 lambda=%s" % lam, 0.5, int(lam)) for lam in args.lam.split(",") if lam]
    settings = [(n, q, lam, 0) for n, q, lam in settings]
    # controls: Alg. 1 with a mutation that ignores the parameter graphs (a plain evolutionary
    # algorithm), and no evolution at all
    settings += [("uniform mutation p=%s lambda=8" % q, float(q), 8, 1) for q in args.uniform_mutation.split(",") if q]
    settings += [("uniform random search", 0.5, args.trials, 0)]
    for name, q, lam, mutation in settings:
        curves = []
        for seed in seeds:
            # no reference tensor: parity of every template path is the test suite's business,
            # here only the search is being compared
            res = P.opevo_tune(op, variant, da.data_ptr(), db.data_ptr(), dc.data_ptr(), None, stream,
                               trials=args.trials, lambda_=lam, rho=8, q=q, seed=seed, compile_threads=8,
                               warmup=3, launches_per_sample=0, samples=5, trial_timeout_ms=timeout_ms,
                               progress_every=100, mutation=mutation)
            fit = res["logs"]["fitness"][: int(res["n_trials"])]
            curve = [float(np.max(fit[:m])) if m <= fit.size else float(np.max(fit)) for m in marks]
            curves.append(curve)
            print(json.dumps({"workload": args.workload, "setting": name, "seed": seed, "trials": int(res["n_trials"]),
                              "best_after": dict(zip(map(str, marks), [round(c, 2) for c in curve])),
                              "n_invalid": int(res["n_invalid"]), "wall_s": round(float(res["wall_s"]), 1)}), flush=True)
        arr = np.asarray(curves)
        print(json.dumps({"workload": args.workload, "setting": name, "seeds": seeds,
                          "mean_best_after": dict(zip(map(str, marks), [round(float(x), 2) for x in arr.mean(axis=0)])),
                          "std_best_after": dict(zip(map(str, marks), [round(float(x), 2) for x in arr.std(axis=0)]))}),
              flush=True)
    P.opevo_op_destroy(op)
    P.opevo_compile_pool_stop()
    return 0


if __name__ == "__main__":
    sys.exit(main())
