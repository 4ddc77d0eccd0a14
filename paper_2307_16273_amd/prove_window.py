"""Proves one synthetic training window on the GPU and prints the time of every repetition.

    python -m paper_2307_16273_amd.prove_window --config 3 --reps 5 [--form linked|ft] [--verify] [--step]

The windows are the seeded FCNN windows of the benchmark configurations (Sec. 5, Example FCNN):
3 = 8 layers of 1024 x 1024 at batch 64, 4 = the same over 16 steps, 5 = 4 layers of 4096 x 4096 at
batch 256, 1 = one layer of 256 x 256 at batch 16.  One line of JSON per repetition; with --verify the
library's own verifier replays the last proof on the GPU; with --step the parameter update of the window's own
gradients is proved and verified and the A and W stacks are committed.  Also the program to put behind a
profiler to see one window's kernel sequence on its own.
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
    ap.add_argument("--step", action="store_true",
                    help="after the window: the proof of the parameter update on the window's own gradients "
                         "G_W = A^T G_Z, its verification, and the row commitments of the A and W stacks")
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
    if args.verify and res is not None:
        t0 = time.perf_counter()
        got = zk.aggregate_verify(ctx, res["proof"], zk.Transcript(CONFIG_SEED + args.config))
        print(json.dumps({"verify_ms": 1e3 * (time.perf_counter() - t0), "accepted": got["verdict"] == 0}), flush=True)
    if args.step:
        # G_W of every slot from the window's own stacks (exact in float64: |a|, |g| < 2^31 would not be, so the
        # products are taken in two 16-bit halves of A)
        a = dw["A"].to(torch.int64)
        gz = dw["GZ"].to(torch.float64)
        a_lo, a_hi = (a & 0xFFFF).to(torch.float64), (a >> 16).to(torch.float64)
        gw = (torch.bmm(a_lo.transpose(1, 2), gz).round().to(torch.int64)
              + (torch.bmm(a_hi.transpose(1, 2), gz).round().to(torch.int64) << 16)).reshape(-1).contiguous()
        r_bits = 16 + 8 + (batch.bit_length() - 1)          # the generator's learning rate, 2^-8 on the batch mean
        q_bits = 56 - r_bits
        assert int(gw.abs().max()) < (1 << 55)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        up = zk.update_prove(ctx, gw, zk.Transcript(CONFIG_SEED + 100), q_bits, r_bits)
        torch.cuda.synchronize()
        t_up = 1e3 * (time.perf_counter() - t0)
        t0 = time.perf_counter()
        ok = zk.aggregate_verify(ctx, up["proof"], zk.Transcript(CONFIG_SEED + 100))["verdict"] == 0
        t_vf = 1e3 * (time.perf_counter() - t0)
        line = {"update_proof_ms": t_up, "update_verify_ms": t_vf, "accepted": ok, "gradients": int(gw.numel()),
                "Q": q_bits, "R": r_bits, "proof_bytes": len(up["proof"])}
        if steps > 1:
            # the claim on U against the window's own weights: W_t - W_{t+1} for the slots of steps 0 .. T-2
            u = {c["tensor"]: c for c in up["claims_left"]}["U"]
            line["note"] = "U~(p) is to be compared with (W - W_next)~(p); slots of the last step have no successor here"
            line["u_claim"] = hex(u["value"])
        print(json.dumps(line), flush=True)
        for nm in ("A", "W"):
            flat = dw[nm].reshape(-1)
            mm = flat.numel().bit_length() - 1
            key = zk.CommitKey(ctx, nm.encode(), 1 << (mm // 2))
            xv = zk.tensor_wrap_int(ctx, flat)
            zk.hyrax_commit(ctx, key, xv)
            t0 = time.perf_counter()
            cm = zk.hyrax_commit(ctx, key, xv)
            line = {"commit": nm, "entries": int(flat.numel()), "rows": len(cm), "commit_ms": 1e3 * (time.perf_counter() - t0)}
            if args.form == "linked" and res is not None:
                # the one claim the chained window leaves on this stack, opened against the commitment and checked
                claim = {c["tensor"]: c for c in res["claims_left"]}[nm]
                t0 = time.perf_counter()
                t_row, _, y = zk.hyrax_open(ctx, xv, None, claim["point"])
                line["open_ms"] = 1e3 * (time.perf_counter() - t0)
                t0 = time.perf_counter()
                verdict, _ = zk.hyrax_verify(ctx, key, cm, claim["point"], t_row, None, claim["value"])
                line["open_verify_ms"] = 1e3 * (time.perf_counter() - t0)
                line["claim_opens"] = bool(y == claim["value"] and verdict == 0)
            print(json.dumps(line), flush=True)
            key.close()
    ctx.close()


if __name__ == "__main__":
    main()
