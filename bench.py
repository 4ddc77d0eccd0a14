"""Benchmark of the tensor-sumcheck prover on one MI355X.

A step is one pass of the kernel micro-benchmark workload: a degree-3 sumcheck
over the product of three tables of 2^24 uniform Fr elements (24 rounds) plus
the partial evaluation of a 4096 x 4096 uniform Fr matrix at a random row point.
Prints one JSON line (see the design doc for the fields).
"""
import argparse
import json
import sys
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--log2-size", type=int, default=24, help="log2 of each sumcheck table (24 = the named workload)")
    ap.add_argument("--no-aggregate", action="store_true", help="skip the 8-layer batch-64 proof timing")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2307_16273_amd as zk
    from workloads import uniform_fr_limbs, fcnn_window, CONFIG_SEED

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    ctx = zk.Context(0)
    d = args.log2_size
    n = 1 << d
    side = 1 << (d // 2)
    rng = np.random.default_rng(CONFIG_SEED + 2)
    tabs = [zk.fr_tensor_upload(ctx, uniform_fr_limbs(rng, n), (n,)) for _ in range(3)]
    mat = zk.fr_tensor_upload(ctx, uniform_fr_limbs(rng, side * side), (side, side))
    point = [int.from_bytes(uniform_fr_limbs(rng, 1).tobytes(), "little") for _ in range(d // 2)]

    def step(k):
        tr = zk.Transcript(CONFIG_SEED + 2 + k)
        zk.sumcheck_product(ctx, tabs, tr)
        zk.mle_partial_eval(ctx, mat, 0, 1, point).free()

    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    elems = (3 * n + side * side) * args.steps

    # the two halves on their own
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            a = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - a)
        return float(np.median(ts)), float(np.min(ts))
    sc_med, sc_min = timed(lambda: zk.sumcheck_product(ctx, tabs, zk.Transcript(5)), max(3, args.steps))
    pe_med, pe_min = timed(lambda: zk.mle_partial_eval(ctx, mat, 0, 1, point).free(), max(3, args.steps))

    out = {
        "metric": "Fr elements/s through sumcheck prover; proof ms per batch-64 8-layer step",
        "value": elems / dt, "unit": "Fr elements/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u32x8 Montgomery (Fr, 255-bit modular integers)",
        "data": "synthetic",
        "config": {"workload": f"kernel microbench: degree-3 sumcheck over 3 tables of 2^{d} uniform Fr "
                               f"({d} rounds) + mle_partial_eval of a {side}x{side} Fr matrix at a row point",
                   "sumcheck_ms_median": 1e3 * sc_med, "sumcheck_ms_min": 1e3 * sc_min,
                   "sumcheck_elems_per_s": 3 * n / sc_med,
                   "partial_eval_ms_median": 1e3 * pe_med, "partial_eval_ms_min": 1e3 * pe_min,
                   "partial_eval_elems_per_s": side * side / pe_med},
    }
    if not args.no_aggregate:
        wit = fcnn_window(CONFIG_SEED + 3, n_layers=8, width=1024, batch=64, steps=1)
        dw = {k: wit[k] for k in ("L", "B", "width", "T", "Q", "R")}
        for k in ("A", "W", "GZ", "Zr", "GA"):
            dw[k] = torch.from_numpy(np.ascontiguousarray(wit[k])).cuda()
        ag_med, ag_min = timed(lambda: zk.aggregate_prove(ctx, dw, zk.Transcript(CONFIG_SEED + 3)), 5)
        out["config"]["proof_ms_batch64_8layer_step"] = 1e3 * ag_med
        out["config"]["proof_ms_batch64_8layer_step_min"] = 1e3 * ag_min
        out["config"]["paper_context"] = "paper: < 1 s per batch-64 update, 8-layer 10M-parameter net, one A100, whole protocol incl. commitments"
    print(json.dumps(out))


if __name__ == "__main__":
    main()
