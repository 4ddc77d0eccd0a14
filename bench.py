"""Benchmark of the tensor-sumcheck prover on one MI355X.

A step is one pass of the kernel micro-benchmark workload: a degree-3 sumcheck
over the product of three tables of 2^24 uniform Fr elements (24 rounds) plus
the partial evaluation of a 4096 x 4096 uniform Fr matrix at a random row point.
Inputs are resident in HBM before the timed region.  Prints one JSON line:
`value` = Fr elements through the step per second; `config` names the workload and carries the
median times of its two parts, of a Hadamard sumcheck on int32 stacks of the same size, of the
one-layer proofs and of the aggregated proofs of the
8 x 1024^2 (batch 64; one step, also with the claims chained, and 16 steps) and 4 x 4096^2
(batch 256) networks; `roofline` =
algorithmic bytes of the fused round kernels over their launch time measured with HIP events on
the library's stream (plus the multiply-add rate and the other kernel classes); `cpu_baseline` =
the CPU oracle's rate on the host cores.
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
HBM_PEAK_GBS = 8000.0                       # MI355X HBM3E, published
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz: one 32x32+64-bit multiply-add per lane and clock
MAD_PEAK_T = 256 * 4 * 16 * 2.4e9 / 1e12
MADS_PER_MODMUL = 153                       # 81 operand + 72 reduction products on 9 x 29-bit limbs
MODMUL_PER_PAIR_K3 = 12                     # fused round, K = 3: 6 folds + 3 points x 2 products (g(1) is derived)


def traffic_from_profiles():
    """Measured HBM bytes per launch of the fused round kernel, if a counter summary is committed."""
    path = os.path.join(ROOT, "profiles", "k_sc_round_fused_microbench_pmc.txt")
    try:
        m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read())
        return float(m.group(1)) if m else None
    except OSError:
        return None


def valu_busy_from_profiles():
    """VALU issue-slot occupancy of the fused round kernel from the committed counter summary (rocprofv3 --pmc)."""
    path = os.path.join(ROOT, "profiles", "valu_lds_counters_bench_workloads.txt")
    try:
        m = re.search(r"^k_sc_round<3,1>\s+\S+\s+\S+\s+([0-9.]+)%", open(path).read(), re.M)
        return float(m.group(1)) / 100.0 if m else None
    except OSError:
        return None


def cpu_baseline(log2_size):
    """The CPU oracle, as it stands, on the same workload: its C tier (OpenMP, all host cores)
    at the full size, and the Python-integer tier (one core) on a reduced sample."""
    from oracle import c_oracle
    from oracle import protocols as P
    from oracle.field import fr_array_from_le
    from oracle.mle import partial_eval
    from oracle.transcript import Transcript as OT
    from workloads import uniform_fr_limbs, CONFIG_SEED
    full = 24
    n, side = 1 << full, 1 << (full // 2)
    rng = np.random.default_rng(CONFIG_SEED + 2)
    raws = [uniform_fr_limbs(rng, n).tobytes() for _ in range(3)]
    mat = uniform_fr_limbs(rng, side * side).tobytes()
    pt = [int.from_bytes(uniform_fr_limbs(rng, 1).tobytes(), "little") for _ in range(full // 2)]
    t0 = time.perf_counter()
    c_oracle.product_prove(raws, CONFIG_SEED + 2)
    c_oracle.partial_eval(mat, 1, side, side, pt)
    dt = time.perf_counter() - t0
    out = {"value": (3 * n + side * side) / dt, "unit": "Fr elements/s", "cores": c_oracle.threads(), "kind": "oracle",
           "sample": f"the whole workload (3 tables of 2^{full}, {side}x{side} matrix) on the oracle's C tier, "
                     f"{dt:.1f} s wall on {c_oracle.threads()} threads"}
    del raws, mat
    n = 1 << log2_size
    side = 1 << (log2_size // 2)
    tabs = [fr_array_from_le(uniform_fr_limbs(rng, n).tobytes(), n) for _ in range(3)]
    mat = fr_array_from_le(uniform_fr_limbs(rng, side * side).tobytes(), side * side)
    pt = [int(x) for x in fr_array_from_le(uniform_fr_limbs(rng, log2_size // 2).tobytes(), log2_size // 2)]
    t0 = time.perf_counter()
    P.product_prove(tabs, OT(CONFIG_SEED + 2))
    partial_eval(mat, [side, side], 0, 1, pt)
    dt = time.perf_counter() - t0
    out["python_tier"] = {"value": (3 * n + side * side) / dt, "unit": "Fr elements/s", "cores": 1,
                          "sample": f"3 tables of 2^{log2_size} and a {side}x{side} matrix, {dt:.1f} s on one core"}
    out["cpu_model"] = cpu_model()
    return out


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline_aggregate():
    """The oracle's C tier proving the 8 x 1024^2, batch-64 window (the one behind 'proof ms per
    batch-64 8-layer step'): the whole window on all host threads, and, as the one-core figure, a
    one-layer window of the same width and batch (an eighth of the rows; the whole window would take
    minutes on one core)."""
    from oracle import c_oracle
    from workloads import fcnn_window, CONFIG_SEED
    wit = fcnn_window(CONFIG_SEED + 3, n_layers=8, width=1024, batch=64, steps=1)
    nthreads = c_oracle.threads()
    t0 = time.perf_counter()
    c_oracle.aggregate_prove(wit, c_oracle.Transcript(CONFIG_SEED + 3))
    t_all = time.perf_counter() - t0
    one = fcnn_window(CONFIG_SEED + 3, n_layers=1, width=1024, batch=64, steps=1)
    c_oracle.set_threads(1)
    t0 = time.perf_counter()
    c_oracle.aggregate_prove(one, c_oracle.Transcript(CONFIG_SEED + 3))
    t_one = time.perf_counter() - t0
    c_oracle.set_threads(nthreads)
    return {"proof_ms_batch64_8layer_step": 1e3 * t_all, "cores": nthreads, "kind": "oracle (C tier)",
            "one_core": {"proof_ms": 1e3 * t_one, "cores": 1,
                         "sample": "one layer of 1024 x 1024, batch 64 (2^16 zkReLU rows: an eighth of the window)"},
            "cpu_model": cpu_model()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--log2-size", type=int, default=24, help="log2 of each sumcheck table (24 = the named workload)")
    ap.add_argument("--no-aggregate", action="store_true", help="skip the 8-layer batch-64 proof timing")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-log2-size", type=int, default=20)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a known size for scaling HBM counters)")
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

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the same steps again with HIP events around every kernel, recorded on the library's
    # stream (two event records per launch would otherwise sit inside the timed region)
    ctx.profile(True)
    for k in range(args.steps):
        step(k)
    prof = ctx.profile_read()
    ctx.profile(False, reset=False)
    elems = (3 * n + side * side) * args.steps

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
    sc_med, sc_min = timed(lambda: zk.sumcheck_product(ctx, tabs, zk.Transcript(5)), 5)
    pe_med, pe_min = timed(lambda: zk.mle_partial_eval(ctx, mat, 0, 1, point).free(), 5)

    # the machine's own rates, measured now on this GPU: a streaming copy, independent v_mad_u64_u32
    # chains in registers, the field multiplier in registers
    copy_gbs = max(ctx.selfbench("copy", 1 << 30) for _ in range(3)) / 1e9
    mad_tps = max(ctx.selfbench("mad", 1 << 12) for _ in range(3)) / 1e12
    modmul_gps = max(ctx.selfbench("modmul", 1 << 10) for _ in range(3)) / 1e9
    fused = prof["sc_round_fused"]
    ach = fused["bytes"] / (fused["ms"] * 1e-3) / 1e9 if fused["ms"] > 0 else 0.0
    pairs = fused["bytes"] / 576.0            # K = 3: 576 algorithmic bytes per pair index
    mad_rate = pairs * MODMUL_PER_PAIR_K3 * MADS_PER_MODMUL / (fused["ms"] * 1e-3) / 1e12 if fused["ms"] > 0 else 0.0
    roofline = {
        "kernel": "k_sc_round<3,1> and <3,2> (fused fold-and-evaluate rounds)",
        "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
        "traffic": traffic_from_profiles(),
        "launches": fused["launches"], "avg_launch_us": 1e3 * fused["ms"] / max(fused["launches"], 1),
        "algorithmic_bytes_per_launch": fused["bytes"] / max(fused["launches"], 1),
        "alu": {"achieved": mad_rate, "peak": MAD_PEAK_T, "unit": "Tmad/s", "frac": mad_rate / MAD_PEAK_T,
                "measured_mad_peak": mad_tps, "frac_of_measured_mad_peak": mad_rate / mad_tps if mad_tps else None,
                "modmul_per_s": mad_rate * 1e12 / MADS_PER_MODMUL,
                "measured_modmul_peak_per_s": modmul_gps * 1e9,
                "frac_of_measured_modmul_peak": mad_rate * 1e3 / MADS_PER_MODMUL / modmul_gps if modmul_gps else None},
        "valu_issue_busy_from_counters": valu_busy_from_profiles(),
        "measured_copy_GBps": copy_gbs, "frac_of_measured_copy": ach / copy_gbs if copy_gbs else None,
        "other_kernels": {k: {"launches": v["launches"], "ms": v["ms"],
                              "GBps": (v["bytes"] / (v["ms"] * 1e-3) / 1e9 if v["ms"] > 0 else 0.0)}
                          for k, v in prof.items() if k != "sc_round_fused" and v["launches"]},
    }
    out = {
        "metric": "Fr elements/s through sumcheck prover; proof ms per batch-64 8-layer step",
        "value": elems / dt, "unit": "Fr elements/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u32 limbs (Fr, 255-bit modular integers)",
        "data": "synthetic",
        "config": {"workload": f"kernel microbench: degree-3 sumcheck over 3 tables of 2^{d} uniform Fr "
                               f"({d} rounds) + mle_partial_eval of a {side}x{side} Fr matrix at a row point",
                   "sumcheck_ms_median": 1e3 * sc_med, "sumcheck_ms_min": 1e3 * sc_min,
                   "sumcheck_elems_per_s": 3 * n / sc_med,
                   "partial_eval_ms_median": 1e3 * pe_med, "partial_eval_ms_min": 1e3 * pe_min,
                   "partial_eval_elems_per_s": side * side / pe_med},
        "roofline": roofline,
    }
    # fr_tensor_upload, reported on its own: 2^24 canonical Fr from host memory (PCIe copy +
    # conversion to Montgomery limb planes), and the conversion alone from a device buffer
    raw = uniform_fr_limbs(rng, n)
    up_med, _ = timed(lambda: zk.fr_tensor_upload(ctx, raw, (n,)).free(), 3)
    out["config"]["upload_fr_host_elems_per_s"] = n / up_med
    del raw
    # sumcheck_hadamard on two int32 stacks of 2^24 values (conversion, the table of beta~(p, .), 24 rounds)
    h0 = torch.from_numpy(rng.integers(-2 ** 31, 2 ** 31, n, dtype=np.int64).astype(np.int32)).cuda()
    h1 = torch.from_numpy(rng.integers(-2 ** 31, 2 ** 31, n, dtype=np.int64).astype(np.int32)).cuda()
    ha, hb = zk.tensor_wrap_int(ctx, h0, (n,)), zk.tensor_wrap_int(ctx, h1, (n,))
    hd_med, _ = timed(lambda: zk.sumcheck_hadamard(ctx, ha, hb, zk.Transcript(6)), 3)
    out["config"]["hadamard_int32_2p24_ms"] = 1e3 * hd_med
    del ha, hb, h0, h1
    if not args.no_aggregate:
        # config 1: one FC layer 16 x 256 x 256 and its ReLU (forward only); latency-dominated
        from workloads import fc_relu_layer
        lay = fc_relu_layer(CONFIG_SEED + 1)
        x1 = zk.tensor_wrap_int(ctx, torch.from_numpy(lay["X"]).cuda(), (1, 16, 256))
        w1 = zk.tensor_wrap_int(ctx, torch.from_numpy(lay["W"]).cuda(), (1, 256, 256))
        z1 = torch.from_numpy(lay["Z"]).cuda().reshape(-1)
        mm_med, _ = timed(lambda: zk.sumcheck_matmul(ctx, x1, w1, zk.Transcript(CONFIG_SEED + 1)), 5)
        zr_med, _ = timed(lambda: zk.zkrelu_prove(ctx, z1, None, zk.Transcript(CONFIG_SEED + 1)), 5)
        ft_med, _ = timed(lambda: zk.sumcheck_matmul_ft(ctx, x1, w1, zk.Transcript(CONFIG_SEED + 1)), 5)
        out["config"]["config1_matmul_us"] = 1e6 * mm_med
        out["config"]["config1_matmul_ft_us"] = 1e6 * ft_med
        out["config"]["config1_zkrelu_us"] = 1e6 * zr_med
        del x1, w1, z1
        wit = fcnn_window(CONFIG_SEED + 3, n_layers=8, width=1024, batch=64, steps=1)
        dw = {k: wit[k] for k in ("L", "B", "width", "T", "Q", "R")}
        for k in ("A", "W", "GZ", "Zr", "GA"):
            dw[k] = torch.from_numpy(np.ascontiguousarray(wit[k])).cuda()
        # the parameter update of the step: rounding of the 8 x 1024^2 gradient stack proved by zkReLU
        gw = torch.from_numpy(np.random.default_rng(CONFIG_SEED + 33).integers(-(1 << 44), 1 << 44, 1 << 23,
                                                                                  dtype=np.int64)).cuda()
        # (Q, R) = (26, 30): learning rate 2^-14 on 16 fractional bits, gradients below 2^55; 56 bits is the widest
        # recomposition whose first two rounds run on the integers
        up_med, _ = timed(lambda: zk.update_prove(ctx, gw, zk.Transcript(CONFIG_SEED + 33), 26, 30), 3)
        out["config"]["update_proof_ms_GW_stack_2p23"] = 1e3 * up_med
        del gw
        # commitments to the window's int32 stacks (Protocol zkdl, the commit line): rows of sqrt(size) entries
        for nm in ("A", "W"):
            flat = dw[nm].reshape(-1)
            mm = flat.numel().bit_length() - 1
            key = zk.CommitKey(ctx, nm.encode(), 1 << (mm // 2))
            xv = zk.tensor_wrap_int(ctx, flat)
            cm_med, _ = timed(lambda: zk.hyrax_commit(ctx, key, xv), 3)
            out["config"]["commit_ms_%s_stack_2p%d" % (nm, mm)] = 1e3 * cm_med
            if nm == "A":   # the proof of evaluation at a random point and the verifier's two sums on the GPU
                prng = np.random.default_rng(CONFIG_SEED + 34)
                pt = [int.from_bytes(prng.bytes(31), "little") for _ in range(mm)]
                coms = zk.hyrax_commit(ctx, key, xv)
                op_med, _ = timed(lambda: zk.hyrax_open(ctx, xv, None, pt), 3)
                t_row, _, y_val = zk.hyrax_open(ctx, xv, None, pt)
                hv_med, _ = timed(lambda: zk.hyrax_verify(ctx, key, coms, pt, t_row, None, y_val, want_combined=False), 3)
                assert zk.hyrax_verify(ctx, key, coms, pt, t_row, None, y_val, want_combined=False)[0] == 0
                out["config"]["open_ms_A_stack_2p%d" % mm] = 1e3 * op_med
                out["config"]["open_verify_ms_A_stack_2p%d" % mm] = 1e3 * hv_med
            key.close()
        ag_med, ag_min = timed(lambda: zk.aggregate_prove(ctx, dw, zk.Transcript(CONFIG_SEED + 3)), 5)
        out["config"]["proof_ms_batch64_8layer_step"] = 1e3 * ag_med
        out["config"]["proof_ms_batch64_8layer_step_min"] = 1e3 * ag_min
        lk_med, _ = timed(lambda: zk.aggregate_prove(ctx, dw, zk.Transcript(CONFIG_SEED + 3), linked=True), 5)
        out["config"]["proof_ms_batch64_8layer_step_linked"] = 1e3 * lk_med
        ft_med, _ = timed(lambda: zk.aggregate_prove(ctx, dw, zk.Transcript(CONFIG_SEED + 3), ft=True), 5)
        out["config"]["proof_ms_batch64_8layer_step_ft"] = 1e3 * ft_med
        pf3 = zk.aggregate_prove(ctx, dw, zk.Transcript(CONFIG_SEED + 3))["proof"]
        vf_med, _ = timed(lambda: zk.aggregate_verify(ctx, pf3, zk.Transcript(CONFIG_SEED + 3)), 5)
        out["config"]["verify_ms_batch64_8layer_step"] = 1e3 * vf_med
        assert zk.aggregate_verify(ctx, pf3, zk.Transcript(CONFIG_SEED + 3))["verdict"] == 0
        pl3 = zk.aggregate_prove(ctx, dw, zk.Transcript(CONFIG_SEED + 3), linked=True)["proof"]
        vl_med, _ = timed(lambda: zk.aggregate_verify(ctx, pl3, zk.Transcript(CONFIG_SEED + 3)), 5)
        out["config"]["verify_ms_batch64_8layer_step_linked"] = 1e3 * vl_med
        assert zk.aggregate_verify(ctx, pl3, zk.Transcript(CONFIG_SEED + 3))["verdict"] == 0
        out["config"]["paper_context"] = ("paper: < 1 s per batch-64 update, 8-layer 10M-parameter net, one "
                                          "Tesla A100, whole protocol including commitments (not comparable)")
        del dw
        # the two larger aggregation windows of the config list, for reference
        for key, (nl, wd, bs, st, cfg) in {"config4_16steps": (8, 1024, 64, 16, 4),
                                           "config5_4x4096_b256": (4, 4096, 256, 1, 5)}.items():
            wit = fcnn_window(CONFIG_SEED + cfg, n_layers=nl, width=wd, batch=bs, steps=st)
            dw = {k: wit[k] for k in ("L", "B", "width", "T", "Q", "R")}
            for k in ("A", "W", "GZ", "Zr", "GA"):
                dw[k] = torch.from_numpy(np.ascontiguousarray(wit[k])).cuda()
            med, _ = timed(lambda: zk.aggregate_prove(ctx, dw, zk.Transcript(CONFIG_SEED + cfg)), 3)
            out["config"]["proof_ms_" + key] = 1e3 * med
            if st > 1:
                out["config"]["proof_ms_" + key + "_per_step"] = 1e3 * med / st
            med, _ = timed(lambda: zk.aggregate_prove(ctx, dw, zk.Transcript(CONFIG_SEED + cfg), linked=True), 3)
            out["config"]["proof_ms_" + key + "_linked"] = 1e3 * med
            med, _ = timed(lambda: zk.aggregate_prove(ctx, dw, zk.Transcript(CONFIG_SEED + cfg), ft=True), 3)
            out["config"]["proof_ms_" + key + "_ft"] = 1e3 * med
            del dw, wit
            ctx.trim()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.cpu_log2_size)
        if not args.no_aggregate:
            out["cpu_baseline"]["aggregate_8x1024_b64"] = cpu_baseline_aggregate()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
