"""Proves one synthetic training window on the GPU and prints the time of every repetition.

    python -m paper_2307_16273_amd.prove_window --config 3 --reps 5 [--form linked|ft] [--verify]

The windows are the seeded FCNN windows of the benchmark configurations (Sec. 5, Example FCNN):
3 = 8 layers of 1024 x 1024 at batch 64, 4 = the same over 16 steps, 5 = 4 layers of 4096 x 4096 at
batch 256, 1 = one layer of 256 x 256 at batch 16.  One line of JSON per repetition; with --verify the
library's own verifier replays the last proof on the GPU.  Also the program to put behind a profiler to
see one window's kernel sequence on its own.
"""
import argparse
import json
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

SHAPES = {1: (1, 256, 16, 1), 3: (8, 1024, 64, 1), 4: (8, 1024, 64, 16), 5: (4, 4096, 256, 1)}


def main():
    ap = argparse.ArgumentParser(description=__doc__.splitlines()[0])
    ap.add_argument("--config", type=int, default=3, choices=sorted(SHAPES))
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--form", default="plain", choices=["plain", "linked", "ft"])
    ap.add_argument("--verify", action="store_true")
    args = ap.parse_args()
    import numpy as np
    import torch
    import paper_2307_16273_amd as zk
    from workloads import fcnn_window, CONFIG_SEED

    assert torch.cuda.is_available(), "prove_window needs a GPU"
    layers, width, batch, steps = SHAPES[args.config]
    wit = fcnn_window(CONFIG_SEED + args.config, n_layers=layers, width=width, batch=batch, steps=steps)
    dw = {k: wit[k] for k in ("L", "B", "width", "T", "Q", "R")}
    for k in ("A", "W", "GZ", "Zr", "GA"):
        dw[k] = torch.from_numpy(np.ascontiguousarray(wit[k])).cuda()
    ctx = zk.Context(0)
    res = None
    for rep in range(args.reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        res = zk.aggregate_prove(ctx, dw, zk.Transcript(CONFIG_SEED + args.config), linked=args.form == "linked",
                                 ft=args.form == "ft")
        torch.cuda.synchronize()
        print(json.dumps({"config": args.config, "form": args.form, "rep": rep,
                          "proof_ms": 1e3 * (time.perf_counter() - t0), "proof_bytes": len(res["proof"]),
                          "claims_left": len(res["claims_left"])}), flush=True)
    if args.verify and res is not None and args.form != "linked":
        t0 = time.perf_counter()
        got = zk.aggregate_verify(ctx, res["proof"], zk.Transcript(CONFIG_SEED + args.config))
        print(json.dumps({"verify_ms": 1e3 * (time.perf_counter() - t0), "accepted": got["verdict"] == 0}), flush=True)
    ctx.close()


if __name__ == "__main__":
    main()
