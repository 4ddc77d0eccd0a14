"""Writes the stored expected proofs under tests/golden/ from the CPU oracle.

Run from the repository root:  python tests/golden/make_golden.py
Calls only `oracle/` and the seeded input generators in `workloads/`.  The files freeze
the oracle's output (proof bytes, challenges, transcript digest) for a few small
instances, so that an unintended change of a byte format or of the oracle's arithmetic
shows up as a diff; the paper prints no numeric worked example to store instead
(its protocols are given symbolically: Sec. 2.2, Sec. 3.1, App. A, App. B).
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import protocols as P                      # noqa: E402
from oracle.field import fr_array, fr_array_from_le    # noqa: E402
from oracle.transcript import Transcript               # noqa: E402
from workloads import uniform_fr_limbs, fcnn_window    # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def product_case():
    """Product sumcheck (Sec. 2.2): K = 3 tables of 2^3 uniform field elements."""
    rng = np.random.default_rng(20230716)
    raws = [uniform_fr_limbs(rng, 8).tobytes() for _ in range(3)]
    ts = Transcript(7)
    buf, proof, vs = P.product_prove([fr_array_from_le(r, 8) for r in raws], ts)
    return {"protocol": "sumcheck_product", "cite": "Sec. 2.2", "seed": 7, "tables_le_hex": [r.hex() for r in raws],
            "proof_hex": buf.hex(), "challenges": [hex(v) for v in vs], "digest_hex": ts.digest().hex()}


def matmul_case():
    """Batched matrix product (Eq. exm-matmul-batched): N = 2, 2 x 4 times 4 x 2, small integers."""
    rng = np.random.default_rng(20230717)
    x0 = rng.integers(-50, 50, (2, 2, 4)).astype(np.int64)
    x1 = rng.integers(-50, 50, (2, 4, 2)).astype(np.int64)
    ts = Transcript(8)
    buf, proof, _ = P.matmul_prove(fr_array(x0), [2, 2, 4], fr_array(x1), [2, 4, 2], ts)
    return {"protocol": "sumcheck_matmul", "cite": "Eq. exm-matmul-batched", "seed": 8,
            "x0": x0.reshape(-1).tolist(), "x0_shape": [2, 2, 4], "x1": x1.reshape(-1).tolist(), "x1_shape": [2, 4, 2],
            "proof_hex": buf.hex(), "challenges": [hex(v) for v in ts.challenges], "digest_hex": ts.digest().hex()}


def matmul_ft_case():
    """The same product with the messages of the optimized aggregated protocol (App. B)."""
    rng = np.random.default_rng(20230717)
    x0 = rng.integers(-50, 50, (2, 2, 4)).astype(np.int64)
    x1 = rng.integers(-50, 50, (2, 4, 2)).astype(np.int64)
    ts = Transcript(8)
    buf, info = P.matmul_ft_prove(fr_array(x0), [2, 2, 4], fr_array(x1), [2, 4, 2], ts)
    return {"protocol": "sumcheck_matmul_ft", "cite": "App. B, Protocol tensor-op-aggr-optimized", "seed": 8,
            "x0": x0.reshape(-1).tolist(), "x0_shape": [2, 2, 4], "x1": x1.reshape(-1).tolist(), "x1_shape": [2, 4, 2],
            "proof_hex": buf.hex(), "challenges": [hex(v) for v in ts.challenges], "digest_hex": ts.digest().hex()}


def zkrelu_case():
    """zkReLU (Sec. 3.1, App. A): D = 4, Q = 5, R = 3, with gradients."""
    z = [77, -128, -1, 100]
    ga = [-5, 127, 0, -64]
    ts = Transcript(9)
    buf, info = P.zkrelu_prove(z, ga, 5, 3, ts)
    return {"protocol": "zkrelu_prove", "cite": "Sec. 3.1, App. A", "seed": 9, "Z": z, "GA": ga, "Q": 5, "R": 3,
            "proof_hex": buf.hex(), "challenges": [hex(v) for v in ts.challenges], "digest_hex": ts.digest().hex()}


def zkrelu_at_case():
    """zkReLU at four given points (Sec. 3.2, App. A): the same inputs, points from a seeded generator."""
    z = [77, -128, -1, 100]
    ga = [-5, 127, 0, -64]
    rng = np.random.default_rng(20230719)
    pts = [[int(v) for v in fr_array_from_le(uniform_fr_limbs(rng, 2).tobytes(), 2)] for _ in range(4)]
    ts = Transcript(12)
    buf, info = P.zkrelu_prove(z, ga, 5, 3, ts, points=pts)
    return {"protocol": "zkrelu_prove_at", "cite": "Sec. 3.2, App. A", "seed": 12, "Z": z, "GA": ga, "Q": 5, "R": 3,
            "points": [[hex(v) for v in pt] for pt in pts],
            "proof_hex": buf.hex(), "challenges": [hex(v) for v in ts.challenges], "digest_hex": ts.digest().hex()}


def aggregate_case():
    """Aggregated window (Sec. 5, Example FCNN): L = 2 layers of width 4, batch 2, 2 steps."""
    wit = fcnn_window(2307162730 + 90, 2, 4, 2, 2)
    ts = Transcript(10)
    buf = P.aggregate_prove(wit, ts)
    buf = buf[0] if isinstance(buf, tuple) else buf
    return {"protocol": "aggregate_prove", "cite": "Sec. 5, Example FCNN", "seed": 10,
            "workload": "fcnn_window(2307162730 + 90, n_layers=2, width=4, batch=2, steps=2)",
            "proof_hex": bytes(buf).hex(), "challenges": [hex(v) for v in ts.challenges],
            "digest_hex": ts.digest().hex()}


def aggregate_linked_case():
    """The same window with the claims chained (Sec. 3.2; Eq. sc-reindex; Protocol zkdl)."""
    wit = fcnn_window(2307162730 + 90, 2, 4, 2, 2)
    ts = Transcript(13)
    buf, _ = P.aggregate_linked_prove(wit, ts)
    return {"protocol": "aggregate_prove_linked", "cite": "Sec. 3.2, Eq. sc-reindex, Protocol zkdl", "seed": 13,
            "workload": "fcnn_window(2307162730 + 90, n_layers=2, width=4, batch=2, steps=2)",
            "proof_hex": bytes(buf).hex(), "challenges": [hex(v) for v in ts.challenges],
            "digest_hex": ts.digest().hex()}


def aggregate_ft_case():
    """The same window with the matrix products in the optimized aggregated form (App. B)."""
    wit = fcnn_window(2307162730 + 90, n_layers=2, width=4, batch=2, steps=2)
    ts = Transcript(16)
    buf, _ = P.aggregate_ft_prove(wit, ts)
    return {"protocol": "aggregate_prove_ft", "cite": "App. B, Protocol tensor-op-aggr-optimized; Protocol zkdl",
            "seed": 16, "workload": "fcnn_window(2307162730 + 90, n_layers=2, width=4, batch=2, steps=2)",
            "proof_hex": bytes(buf).hex(), "challenges": [hex(v) for v in ts.challenges],
            "digest_hex": ts.digest().hex()}


def matmul_general_case():
    """The same product in the general aggregated form (Eq. tensor-op-aggr, Protocol tensor-op-aggr)."""
    rng = np.random.default_rng(20230717)
    x0 = rng.integers(-50, 50, (2, 2, 4)).astype(np.int64)
    x1 = rng.integers(-50, 50, (2, 4, 2)).astype(np.int64)
    y = np.einsum("nij,njk->nik", x0, x1)
    ts = Transcript(17)
    buf, info = P.matmul_general_prove(fr_array(x0), [2, 2, 4], fr_array(x1), [2, 4, 2], fr_array(y), ts)
    return {"protocol": "sumcheck_matmul_general", "cite": "Eq. tensor-op-aggr, App. B Protocol tensor-op-aggr", "seed": 17,
            "x0": x0.reshape(-1).tolist(), "x0_shape": [2, 2, 4], "x1": x1.reshape(-1).tolist(), "x1_shape": [2, 4, 2],
            "y": y.reshape(-1).tolist(),
            "proof_hex": buf.hex(), "challenges": [hex(v) for v in ts.challenges], "digest_hex": ts.digest().hex()}


def reindex_case():
    """Re-indexing sumcheck (Eq. sc-reindex): stack of N = 4 tensors of D = 8, two sub-stacks."""
    rng = np.random.default_rng(20230718)
    x = rng.integers(-50, 50, (4, 8)).astype(np.int64)
    maps = [[0, 1, 2, 3], [1, 2, 3, -1]]
    pts = [uniform_fr_limbs(rng, 2).tobytes() for _ in maps]
    u = uniform_fr_limbs(rng, 3).tobytes()
    ts = Transcript(11)
    buf, info = P.reindex_prove(fr_array(x), 4, 8, maps, [list(fr_array_from_le(p, 2)) for p in pts],
                                list(fr_array_from_le(u, 3)), ts)
    return {"protocol": "reindex_prove", "cite": "Eq. sc-reindex", "seed": 11, "x": x.reshape(-1).tolist(),
            "x_shape": [4, 8], "maps": maps, "points_le_hex": [p.hex() for p in pts], "u_le_hex": u.hex(),
            "proof_hex": buf.hex(), "challenges": [hex(v) for v in ts.challenges], "digest_hex": ts.digest().hex()}


def merge_case():
    """Three claims on one tensor of 16 elements merged into one (Sec. 2.2; Eq. sc-reindex over all variables)."""
    rng = np.random.default_rng(20230720)
    x = rng.integers(-50, 50, 16).astype(np.int64)
    pts = [uniform_fr_limbs(rng, 4).tobytes() for _ in range(3)]
    ts = Transcript(14)
    buf, info = P.merge_prove(fr_array(x), [list(fr_array_from_le(p, 4)) for p in pts], ts)
    return {"protocol": "claims_merge_prove", "cite": "Sec. 2.2, Eq. sc-reindex, Protocol zkdl", "seed": 14,
            "x": x.tolist(), "points_le_hex": [p.hex() for p in pts],
            "proof_hex": buf.hex(), "challenges": [hex(v) for v in ts.challenges], "digest_hex": ts.digest().hex()}


def stack_merge_case():
    """Two claims on a stack of 4 tensors of 8 elements merged on tables of the inner size (Eq. sc-reindex)."""
    rng = np.random.default_rng(20230721)
    x = rng.integers(-50, 50, (4, 8)).astype(np.int64)
    pts = [uniform_fr_limbs(rng, 5).tobytes() for _ in range(2)]
    ts = Transcript(15)
    buf, info = P.stack_merge_prove(fr_array(x), 4, 8, [list(fr_array_from_le(p, 5)) for p in pts], ts)
    return {"protocol": "claims_merge_stack_prove", "cite": "Sec. 2.2, Eq. sc-reindex, Protocol zkdl", "seed": 15,
            "x": x.reshape(-1).tolist(), "x_shape": [4, 8], "points_le_hex": [p.hex() for p in pts],
            "proof_hex": buf.hex(), "challenges": [hex(v) for v in ts.challenges], "digest_hex": ts.digest().hex()}


def update_case():
    """Parameter update (Sec. 5, Example FCNN, last item): D = 4 gradients, Q = 5, R = 3, with both ties."""
    gw = [77, -4, 4, -100]
    ts = Transcript(17)
    buf, info = P.update_prove(gw, 5, 3, ts)
    return {"protocol": "update_prove", "cite": "Sec. 5, Example FCNN (parameter updates); Sec. 3.1, App. A", "seed": 17,
            "GW": gw, "Q": 5, "R": 3,
            "proof_hex": buf.hex(), "challenges": [hex(v) for v in ts.challenges], "digest_hex": ts.digest().hex()}


if __name__ == "__main__":
    for name, fn in (("product_k3_d3", product_case), ("matmul_n2_2x4x2", matmul_case),
                     ("matmul_ft_n2_2x4x2", matmul_ft_case), ("matmul_general_n2_2x4x2", matmul_general_case),
                     ("zkrelu_d4_q5_r3", zkrelu_case), ("zkrelu_at_d4_q5_r3", zkrelu_at_case),
                     ("aggregate_l2_w4_b2_t2", aggregate_case),
                     ("aggregate_linked_l2_w4_b2_t2", aggregate_linked_case),
                     ("aggregate_ft_l2_w4_b2_t2", aggregate_ft_case),
                     ("reindex_n4_d8_k2", reindex_case), ("merge_d4_k3", merge_case),
                     ("stack_merge_n4_d8_k2", stack_merge_case), ("update_d4_q5_r3", update_case)):
        with open(os.path.join(HERE, name + ".json"), "w") as f:
            json.dump(fn(), f, indent=1)
            f.write("\n")
        print("wrote", name)
