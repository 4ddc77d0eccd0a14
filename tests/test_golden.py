"""Stored expected proofs (tests/golden/*.json, written by tests/golden/make_golden.py from
the CPU oracle alone): the oracle must still reproduce them byte for byte, and so must the
HIP library."""
import json
import os

import numpy as np
import pytest

from oracle import protocols as P
from oracle.field import fr_array, fr_array_from_le
from oracle.transcript import Transcript as OracleTranscript
from workloads import fcnn_window

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load(name):
    with open(os.path.join(GOLDEN, name + ".json")) as f:
        return json.load(f)


def oracle_run(g):
    ts = OracleTranscript(g["seed"])
    if g["protocol"] == "sumcheck_product":
        buf = P.product_prove([fr_array_from_le(bytes.fromhex(h), 8) for h in g["tables_le_hex"]], ts)[0]
    elif g["protocol"] == "sumcheck_matmul":
        buf = P.matmul_prove(fr_array(np.array(g["x0"])), g["x0_shape"], fr_array(np.array(g["x1"])), g["x1_shape"], ts)[0]
    elif g["protocol"] == "sumcheck_matmul_ft":
        buf = P.matmul_ft_prove(fr_array(np.array(g["x0"])), g["x0_shape"], fr_array(np.array(g["x1"])), g["x1_shape"], ts)[0]
    elif g["protocol"] == "sumcheck_matmul_general":
        buf = P.matmul_general_prove(fr_array(np.array(g["x0"])), g["x0_shape"], fr_array(np.array(g["x1"])), g["x1_shape"],
                                     fr_array(np.array(g["y"])), ts)[0]
    elif g["protocol"] == "update_prove":
        buf = P.update_prove(g["GW"], g["Q"], g["R"], ts)[0]
    elif g["protocol"] == "zkrelu_prove":
        buf = P.zkrelu_prove(g["Z"], g["GA"], g["Q"], g["R"], ts)[0]
    elif g["protocol"] == "zkrelu_prove_at":
        buf = P.zkrelu_prove(g["Z"], g["GA"], g["Q"], g["R"], ts, points=[[int(v, 16) for v in pt] for pt in g["points"]])[0]
    elif g["protocol"] == "reindex_prove":
        n, d = g["x_shape"]
        pts = [[int(v) for v in fr_array_from_le(bytes.fromhex(h), len(h) // 64)] for h in g["points_le_hex"]]
        u = [int(v) for v in fr_array_from_le(bytes.fromhex(g["u_le_hex"]), len(g["u_le_hex"]) // 64)]
        buf = P.reindex_prove(fr_array(np.array(g["x"]).reshape(n, d)), n, d, g["maps"], pts, u, ts)[0]
    elif g["protocol"] == "claims_merge_prove":
        pts = [[int(v) for v in fr_array_from_le(bytes.fromhex(h), len(h) // 64)] for h in g["points_le_hex"]]
        buf = P.merge_prove(fr_array(np.array(g["x"])), pts, ts)[0]
    elif g["protocol"] == "claims_merge_stack_prove":
        pts = [[int(v) for v in fr_array_from_le(bytes.fromhex(h), len(h) // 64)] for h in g["points_le_hex"]]
        buf = P.stack_merge_prove(fr_array(np.array(g["x"])), g["x_shape"][0], g["x_shape"][1], pts, ts)[0]
    elif g["protocol"] == "aggregate_prove_linked":
        buf = P.aggregate_linked_prove(fcnn_window(2307162730 + 90, 2, 4, 2, 2), ts)[0]
    elif g["protocol"] == "aggregate_prove_ft":
        buf = P.aggregate_ft_prove(fcnn_window(2307162730 + 90, 2, 4, 2, 2), ts)[0]
    else:
        out = P.aggregate_prove(fcnn_window(2307162730 + 90, 2, 4, 2, 2), ts)
        buf = out[0] if isinstance(out, tuple) else out
    return bytes(buf), ts


def _without_repeats(points, drawn):
    """Removes from `points` the block of repeated earlier challenges (the points handed to
    zkReLU), so that the drawn ones remain in order."""
    out, k = [], 0
    for v in points:
        if k < len(drawn) and v == drawn[k]:
            out.append(v)
            k += 1
    return out


NAMES = ["product_k3_d3", "matmul_n2_2x4x2", "matmul_ft_n2_2x4x2", "matmul_general_n2_2x4x2", "zkrelu_d4_q5_r3", "zkrelu_at_d4_q5_r3", "aggregate_l2_w4_b2_t2",
         "aggregate_linked_l2_w4_b2_t2", "aggregate_ft_l2_w4_b2_t2", "merge_d4_k3", "stack_merge_n4_d8_k2",
         "reindex_n4_d8_k2", "update_d4_q5_r3"]


@pytest.mark.parametrize("name", NAMES)
def test_oracle_reproduces_stored_proofs(name):
    g = load(name)
    buf, ts = oracle_run(g)
    assert buf.hex() == g["proof_hex"]
    assert [hex(v) for v in ts.challenges] == g["challenges"]
    assert ts.digest().hex() == g["digest_hex"]


@pytest.mark.gpu
@pytest.mark.parametrize("name", NAMES)
def test_library_reproduces_stored_proofs(lib, ctx, name):
    import torch
    g = load(name)
    print(f"[golden] {name}", flush=True)
    tr = lib.Transcript(g["seed"])
    given = []          # points the caller supplies come back in front of the drawn ones
    if g["protocol"] == "sumcheck_product":
        tabs = [lib.fr_tensor_upload(ctx, bytes.fromhex(h), (8,)) for h in g["tables_le_hex"]]
        got = lib.sumcheck_product(ctx, tabs, tr)
    elif g["protocol"] in ("sumcheck_matmul", "sumcheck_matmul_ft"):
        x0 = lib.fr_tensor_upload(ctx, np.array(g["x0"], dtype=np.int64), tuple(g["x0_shape"]))
        x1 = lib.fr_tensor_upload(ctx, np.array(g["x1"], dtype=np.int64), tuple(g["x1_shape"]))
        got = getattr(lib, g["protocol"])(ctx, x0, x1, tr)
    elif g["protocol"] == "sumcheck_matmul_general":
        x0 = lib.fr_tensor_upload(ctx, np.array(g["x0"], dtype=np.int64), tuple(g["x0_shape"]))
        x1 = lib.fr_tensor_upload(ctx, np.array(g["x1"], dtype=np.int64), tuple(g["x1_shape"]))
        yy = lib.fr_tensor_upload(ctx, np.array(g["y"], dtype=np.int64), (g["x0_shape"][0], g["x0_shape"][1], g["x1_shape"][2]))
        got = lib.sumcheck_matmul_general(ctx, x0, x1, yy, tr)
    elif g["protocol"] == "reindex_prove":
        n, d = g["x_shape"]
        x = lib.fr_tensor_upload(ctx, np.array(g["x"], dtype=np.int64), (n, d))
        pts = [[int(v) for v in fr_array_from_le(bytes.fromhex(h), len(h) // 64)] for h in g["points_le_hex"]]
        u = [int(v) for v in fr_array_from_le(bytes.fromhex(g["u_le_hex"]), len(g["u_le_hex"]) // 64)]
        got = lib.reindex_prove(ctx, x, g["maps"], pts, u, tr)
    elif g["protocol"] in ("claims_merge_prove", "claims_merge_stack_prove"):
        stack = g["protocol"] == "claims_merge_stack_prove"
        x = lib.fr_tensor_upload(ctx, np.array(g["x"], dtype=np.int64), tuple(g["x_shape"]) if stack else (len(g["x"]),))
        pts = [[int(v) for v in fr_array_from_le(bytes.fromhex(h), len(h) // 64)] for h in g["points_le_hex"]]
        got = lib.claims_merge_prove(ctx, x, pts, tr, stack=stack)
    elif g["protocol"] == "zkrelu_prove":
        got = lib.zkrelu_prove(ctx, np.array(g["Z"], dtype=np.int64), np.array(g["GA"], dtype=np.int64), tr, g["Q"], g["R"])
    elif g["protocol"] == "update_prove":
        got = lib.update_prove(ctx, np.array(g["GW"], dtype=np.int64), tr, g["Q"], g["R"])
    elif g["protocol"] == "zkrelu_prove_at":
        pts = [[int(v, 16) for v in pt] for pt in g["points"]]
        given = [hex(v) for pt in pts for v in pt]
        got = lib.zkrelu_prove(ctx, np.array(g["Z"], dtype=np.int64), np.array(g["GA"], dtype=np.int64), tr, g["Q"], g["R"],
                               points=pts)
    else:
        wit = fcnn_window(2307162730 + 90, 2, 4, 2, 2)
        dw = {k: wit[k] for k in ("L", "B", "width", "T", "Q", "R")}
        for k in ("A", "W", "GZ", "Zr", "GA"):
            dw[k] = torch.from_numpy(np.ascontiguousarray(wit[k])).cuda()
        got = lib.aggregate_prove(ctx, dw, tr, linked=g["protocol"] == "aggregate_prove_linked",
                                  ft=g["protocol"] == "aggregate_prove_ft")
    if g["protocol"] in ("aggregate_prove_linked", "update_prove"):
        # the four points given to zkReLU are not draws: they come back in front of its own
        drawn = {int(v, 16) for v in g["challenges"]}
        assert [v for v in got["points"] if v not in drawn] == []
        got["points"] = _without_repeats(got["points"], [int(v, 16) for v in g["challenges"]])
    assert got["proof"].hex() == g["proof_hex"]
    assert [hex(v) for v in got["points"]] == given + g["challenges"]
    assert tr.digest().hex() == g["digest_hex"]
