"""Pins for the oracle's zkReLU and aggregated proofs."""
import struct

import numpy as np
import pytest

from oracle.field import R_MOD, fr_array
from oracle.mle import mle_eval, beta_eval, ilog2
from oracle import protocols as P
from oracle.transcript import Transcript
from workloads import fcnn_window, fc_relu_layer, CONFIG_SEED

rng = np.random.default_rng(31)
Q, R = 32, 16


def edge_values():
    lim = 1 << 47
    return [0, 1, -1, lim - 1, -lim, (1 << 15), (1 << 15) - 1, -(1 << 15), -(1 << 15) - 1,
            (1 << 16), -(1 << 16), 3 << 15, -(3 << 15)]


def test_recomposition_vectors():
    s, sp, j = P.recomposition_vectors(Q, R)
    assert j == 64 and len(s) == 64
    assert s[:3] == [1, 2, 4] and s[46] == 1 << 46 and s[47] == -(1 << 47) and s[48:] == [0] * 16
    assert sp[:15] == [0] * 15 and sp[15] == 1 and sp[16] == 1 and sp[17] == 2
    assert sp[46] == 1 << 30 and sp[47] == -(1 << 31) and sp[48:] == [0] * 16
    s, sp, j = P.recomposition_vectors(4, 4)       # Q+R already a power of two
    assert j == 8 and s == [1, 2, 4, 8, 16, 32, 64, -128] and sp == [0, 0, 0, 1, 1, 2, 4, -8]


def test_witness_matches_plain_integer_relu():
    z = edge_values() + rng.integers(-2 ** 47, 2 ** 47, 51).tolist()
    ga = list(reversed(edge_values())) + rng.integers(-2 ** 47, 2 ** 47, 51).tolist()
    w = P.zkrelu_witness(z, ga, Q, R)
    for i, (zi, gi) in enumerate(zip(z, ga)):
        assert w["Z"][i] == zi and w["GA"][i] == gi                 # Eqs. aux-Z, aux-GA
        zp = (zi + (1 << 15)) >> 16                                  # round half up
        gp = (gi + (1 << 15)) >> 16
        assert w["Zp"][i] == zp and w["GAp"][i] == gp
        assert -(1 << 15) <= zi - (zp << 16) < (1 << 15)             # remainder range
        assert w["sgn"][i] == (1 if zi < 0 else 0)
        assert w["A"][i] == (zp if zi >= 0 else 0)                   # Eq. zkrelu-A
        assert w["GZ"][i] == (gp if zi >= 0 else 0)                  # Eq. zkrelu-GZ
        assert w["A"][i] >= 0 or zi >= 0
    assert set(np.unique(w["aux0"]).tolist()) <= {0, 1}
    assert w["aux0"].shape == (64, 64) and not w["aux0"][:, 48:].any()
    with pytest.raises(ValueError):
        P.zkrelu_witness([1 << 47], [0], Q, R)
    with pytest.raises(ValueError):
        P.zkrelu_witness([0], [-(1 << 47) - 1], Q, R)


def test_witness_agrees_with_the_workload_generator():
    lay = fc_relu_layer(CONFIG_SEED, 4, 16)
    w = P.zkrelu_witness(lay["Z"].reshape(-1).tolist(), [0] * 64, Q, R)
    expect = np.where(lay["Z"].reshape(-1) >= 0, (lay["Z"].reshape(-1) + (1 << 15)) >> 16, 0)
    assert [int(x) for x in w["A"]] == expect.tolist()


@pytest.mark.parametrize("d_len,with_ga", [(4, True), (8, False), (1, True)])
def test_zkrelu_rounds_against_direct_double_sum(d_len, with_ga):
    q, r_bits = 5, 3                      # Q+R = 8 columns, small enough to brute-force
    lim = 1 << (q + r_bits - 1)
    z = rng.integers(-lim, lim, d_len).tolist()
    ga = rng.integers(-lim, lim, d_len).tolist() if with_ga else None
    ts = Transcript(8)
    buf, info = P.zkrelu_prove(z, ga, q, r_bits, ts)
    wit = info["wit"]
    s, sp, j_pad = wit["s"], wit["sp"], wit["j_pad"]
    li, lj = ilog2(d_len), ilog2(j_pad)
    r, rp = info["r"], info["rp"]

    def summand(i, j):
        # the six equations of App. A, weights r^2, r, 1, r'r^2, r'r, r'
        a0, a1 = int(wit["aux0"][i, j]), int(wit["aux1"][i, j])
        ns = 1 - int(wit["aux0"][i, q + r_bits - 1])
        bbin = beta_eval(info["u_bin"], i * j_pad + j)
        return (r * r * beta_eval(info["u_z"], i) * a0 * s[j]
                + r * beta_eval(info["u_a"], i) * ns * a0 * sp[j]
                + bbin * (a0 * a0 - a0)
                + rp * (r * r * beta_eval(info["u_ga"], i) * a1 * s[j]
                        + r * beta_eval(info["u_gz"], i) * ns * a1 * sp[j]
                        + bbin * (a1 * a1 - a1))) % R_MOD
    total = sum(summand(i, j) for i in range(d_len) for j in range(j_pad)) % R_MOD
    assert info["proof"].claim0 == total
    c = info["c_in"]
    assert c[0] == mle_eval(fr_array(z), info["u_z"])
    assert c[1] == mle_eval(fr_array([max(0, (x + 4) >> 3) if x >= 0 else 0 for x in z]), info["u_a"])
    if with_ga:
        assert c[2] == mle_eval(fr_array(ga), info["u_ga"])
        gz = [((g + 4) >> 3) if x >= 0 else 0 for x, g in zip(z, ga)]
        assert c[3] == mle_eval(fr_array(gz), info["u_gz"])
    else:
        assert c[2] == 0 and c[3] == 0
    assert total == (r * r * c[0] + r * c[1] + rp * r * r * c[2] + rp * r * c[3]) % R_MOD
    # finals are evaluations of aux; the merged claim is one more
    aux = np.concatenate([fr_array(wit["aux0"]), fr_array(wit["aux1"])])
    v_i, wbar = info["v"][:li], info["v"][li:]
    assert info["proof"].finals[0] == mle_eval(aux, [0] + v_i + wbar)
    assert info["proof"].finals[1] == mle_eval(aux, [1] + v_i + wbar)
    assert info["proof"].finals[2] == mle_eval(aux, [0] + v_i + P.index_bits(q + r_bits - 1, lj))
    vm = info["vm"]
    assert info["merge"].finals[0] == mle_eval(aux, [vm[0]] + v_i + vm[1:])
    # proof size: 3 log2(D J) + O(1) and 2 log2(J) + O(1) elements, one more per round here
    assert len(info["proof"].rounds) == li + lj and len(info["merge"].rounds) == 1 + lj
    tv = Transcript(8)
    end, out = P.zkrelu_verify(buf, tv)
    assert end == len(buf) and tv.digest() == ts.digest()
    assert out["aux_claim"]["value"] == mle_eval(aux, out["aux_claim"]["point"])


def _direct_double_sum(info, q, r_bits, d_len):
    """The combined sum of App. A written out over all (i, j), from the witness bits."""
    wit = info["wit"]
    s, sp, j_pad = wit["s"], wit["sp"], wit["j_pad"]
    r, rp = info["r"], info["rp"]
    total = 0
    for i in range(d_len):
        ns = 1 - int(wit["aux0"][i, q + r_bits - 1])
        bz, ba = beta_eval(info["u_z"], i), beta_eval(info["u_a"], i)
        bga, bgz = beta_eval(info["u_ga"], i), beta_eval(info["u_gz"], i)
        for j in range(j_pad):
            a0, a1 = int(wit["aux0"][i, j]), int(wit["aux1"][i, j])
            bbin = beta_eval(info["u_bin"], i * j_pad + j)
            total += (r * r * bz * a0 * s[j] + r * ba * ns * a0 * sp[j] + bbin * (a0 * a0 - a0)
                      + rp * (r * r * bga * a1 * s[j] + r * bgz * ns * a1 * sp[j] + bbin * (a1 * a1 - a1)))
    return total % R_MOD


@pytest.mark.parametrize("bind", [True, False])
def test_zkrelu_at_given_points(bind):
    # the four points of the input claims come from outside (Sec. 3.2: the sumchecks of the
    # operations that Z, A, G_A, G_Z take part in leave them)
    q, r_bits, d_len = 5, 3, 8
    lim = 1 << (q + r_bits - 1)
    z = rng.integers(-lim, lim, d_len).tolist()
    ga = rng.integers(-lim, lim, d_len).tolist()
    pts = [[int.from_bytes(rng.bytes(40), "little") % R_MOD for _ in range(3)] for _ in range(4)]
    ts = Transcript(21)
    buf, info = P.zkrelu_prove(z, ga, q, r_bits, ts, points=pts, bind_points=bind)
    assert [info["u_z"], info["u_a"], info["u_ga"], info["u_gz"]] == pts
    c = info["c_in"]
    assert c[0] == mle_eval(fr_array(z), pts[0])
    assert c[1] == mle_eval(fr_array([((x + 4) >> 3) if x >= 0 else 0 for x in z]), pts[1])
    assert c[2] == mle_eval(fr_array(ga), pts[2])
    assert c[3] == mle_eval(fr_array([((g + 4) >> 3) if x >= 0 else 0 for x, g in zip(z, ga)]), pts[3])
    assert info["proof"].claim0 == _direct_double_sum(info, q, r_bits, d_len)
    assert buf[20] == (1 if bind else 2)
    tv = Transcript(21)
    end, out = P.zkrelu_verify(buf, tv, points=pts)
    assert end == len(buf) and tv.digest() == ts.digest()
    # the drawn-points proof is a different transcript; modes cannot be swapped
    plain, _ = P.zkrelu_prove(z, ga, q, r_bits, Transcript(21))
    assert plain[20] == 0 and plain[32:] != buf[32:]
    with pytest.raises(AssertionError):
        P.zkrelu_verify(buf, Transcript(21))
    with pytest.raises(AssertionError):
        P.zkrelu_verify(plain, Transcript(21), points=pts)
    # any changed coordinate of any point is rejected (bound: other challenges; unbound: the
    # final check uses the verifier's own points)
    for k in range(4):
        bad = [list(pt) for pt in pts]
        bad[k][1] = (bad[k][1] + 1) % R_MOD
        with pytest.raises(AssertionError):
            P.zkrelu_verify(buf, Transcript(21), points=bad)
    # a proof made in one mode does not verify as the other
    flipped = bytearray(buf)
    flipped[20] = 2 if bind else 1
    with pytest.raises(AssertionError):
        P.zkrelu_verify(bytes(flipped), Transcript(21), points=pts)


def test_zkrelu_forward_only_equals_zero_gradient():
    z = rng.integers(-2 ** 40, 2 ** 40, 4).tolist()
    b1, _ = P.zkrelu_prove(z, None, Q, R, Transcript(2))
    b2, _ = P.zkrelu_prove(z, [0] * 4, Q, R, Transcript(2))
    # same arithmetic; the has_ga word is in the header and in the transcript
    assert b1[:16] == b2[:16] and b1[16] == 0 and b2[16] == 1
    i1 = P.zkrelu_prove(z, None, Q, R, Transcript(2))[1]
    assert i1["c_in"][2] == 0 and i1["c_in"][3] == 0 and i1["proof"].finals[1] == 0


def test_zkrelu_verifier_rejects_tampering():
    z = rng.integers(-2 ** 40, 2 ** 40, 4).tolist()
    ga = rng.integers(-2 ** 40, 2 ** 40, 4).tolist()
    buf, _ = P.zkrelu_prove(z, ga, Q, R, Transcript(2))
    P.zkrelu_verify(buf, Transcript(2))
    for off in (32, 32 + 128 + 16, 32 + 128 + 16 + 32 * 5, len(buf) - 32, len(buf) - 64):
        bad = bytearray(buf)
        bad[off] ^= 1
        with pytest.raises(AssertionError):
            P.zkrelu_verify(bytes(bad), Transcript(2))


def test_non_binary_aux_breaks_the_binarity_sum():
    # Soundness direction, on the CPU: with one aux entry set to 2 the binarity
    # part of the summand no longer sums to zero.
    u = [int.from_bytes(rng.bytes(40), "little") % R_MOD for _ in range(5)]
    aux = np.zeros(32, dtype=object)
    aux[5] = 1
    total = sum(beta_eval(u, k) * (int(aux[k]) ** 2 - int(aux[k])) for k in range(32)) % R_MOD
    assert total == 0
    aux[7] = 2
    total = sum(beta_eval(u, k) * (int(aux[k]) ** 2 - int(aux[k])) for k in range(32)) % R_MOD
    assert total != 0


def test_aggregate_small_network():
    wit = fcnn_window(CONFIG_SEED + 100, n_layers=2, width=8, batch=4, steps=2)
    n, b, w = 4, 4, 8
    ts = Transcript(12)
    buf, infos = P.aggregate_prove(wit, ts)
    tv = Transcript(12)
    P.aggregate_verify(buf, tv)
    assert tv.digest() == ts.digest()
    a, wt, gz = (wit[k].astype(object) for k in ("A", "W", "GZ"))
    # forward: claim on the stacked Z = A W (all layers), finals on A and W
    f = infos["fwd"]
    z = np.einsum("nij,njk->nik", a, wt)
    vn, vi = f["v"][:2], f["v"][2:]
    fwd_proof = P.SumcheckProof.from_bytes(buf, 32)[0]
    assert fwd_proof.claim0 == mle_eval(fr_array(z), f["w"] + f["u0"] + f["u1"])
    assert fwd_proof.finals[1] == mle_eval(fr_array(a), vn + f["u0"] + vi)
    assert fwd_proof.finals[2] == mle_eval(fr_array(wt), vn + vi + f["u1"])
    # the ReLU'd slots of Z are what zkReLU is given
    for k in range(n):
        if k % 2 == 0:
            assert (z[k] == wit["Zr"][k]).all()
        else:
            assert not wit["Zr"][k].any() and not wit["GA"][k].any()
    # gradA: Y = G_A (unscaled) in the slots that have one
    g = infos["gradA"]
    off = 32 + len(fwd_proof.to_bytes())
    ga_proof, off2 = P.SumcheckProof.from_bytes(buf, off)
    assert ga_proof.claim0 == mle_eval(fr_array(wit["GA"]), g["w"] + g["u0"] + g["u1"])
    # its X1 final is an evaluation of the W stack with the layer axis shifted and the
    # matrix axes swapped: W~shift(v_n, u1, v_i)
    vn, vi = g["v"][:2], g["v"][2:]
    w_shift = P.shift_layers(wit["W"], 2)
    assert ga_proof.finals[2] == mle_eval(fr_array(w_shift), vn + g["u1"] + vi)
    # gradW: Y = A^T G_Z, finals on A (feature axis bound to u0) and G_Z
    h = infos["gradW"]
    gw_proof, _ = P.SumcheckProof.from_bytes(buf, off2)
    gw = np.einsum("nji,njk->nik", a, gz)
    assert gw_proof.claim0 == mle_eval(fr_array(gw), h["w"] + h["u0"] + h["u1"])
    vn, vi = h["v"][:2], h["v"][2:]
    assert gw_proof.finals[1] == mle_eval(fr_array(a), vn + vi + h["u0"])
    assert gw_proof.finals[2] == mle_eval(fr_array(gz), vn + vi + h["u1"])
    # the workload's activations follow from Z by the zkReLU witness equations
    zw = P.zkrelu_witness(wit["Zr"].reshape(-1).tolist(), wit["GA"].reshape(-1).tolist(), Q, R)
    a_next = np.array([int(x) for x in zw["A"]]).reshape(n, b, w)
    gz_prev = np.array([int(x) for x in zw["GZ"]]).reshape(n, b, w)
    for k in range(n):
        if k % 2 == 0:
            assert (a_next[k] == wit["A"][k + 1]).all()
            assert (gz_prev[k] == wit["GZ"][k]).all()


@pytest.mark.parametrize("n_layers,width,batch,steps", [(2, 8, 4, 2), (4, 4, 2, 1), (1, 8, 2, 1)])
def test_aggregate_ft_claims_are_evaluations_of_the_stacks(n_layers, width, batch, steps):
    """The window with the optimized aggregated protocol for its matrix products: the verifier accepts,
    each family's claim_0 is the MLE of the exact integer product, its finals are MLEs of the operand
    stacks, the same tensor evaluations as the g_t form leaves at its own challenges, and a flipped
    byte anywhere is refused."""
    wit = fcnn_window(CONFIG_SEED + 120, n_layers=n_layers, width=width, batch=batch, steps=steps)
    n = n_layers * steps
    ln = n.bit_length() - 1
    ts = Transcript(21)
    buf, infos = P.aggregate_ft_prove(wit, ts)
    tv = Transcript(21)
    res = P.aggregate_ft_verify(buf, tv)
    assert tv.digest() == ts.digest() and tv.challenges == ts.challenges
    a, wt, gz = (wit[k].astype(object) for k in ("A", "W", "GZ"))
    prods = {"fwd": np.einsum("nij,njk->nik", a, wt), "gradA": wit["GA"].astype(object),
             "gradW": np.einsum("nji,njk->nik", a, gz)}
    ops = {"fwd": (a, wt), "gradA": (P.shift_layers(wit["GZ"], n_layers).astype(object),
                                     np.transpose(P.shift_layers(wit["W"], n_layers), (0, 2, 1)).astype(object)),
           "gradW": (np.transpose(a, (0, 2, 1)), gz)}
    for fam in ("fwd", "gradA", "gradW"):
        claim0, finals, pt = res[fam]
        vn, vi = pt["v"][:ln], pt["v"][ln:]
        assert claim0 == mle_eval(fr_array(prods[fam]), pt["w"] + pt["u0"] + pt["u1"]), fam
        assert finals[0] == mle_eval(fr_array(ops[fam][0]), vn + pt["u0"] + vi), fam
        assert finals[1] == mle_eval(fr_array(ops[fam][1]), vn + vi + pt["u1"]), fam
    # shorter than the g_t form: per round one evaluation less, one final less, one more block header and claim
    buf_g, _ = P.aggregate_prove(wit, Transcript(21))
    lw, lb = width.bit_length() - 1, batch.bit_length() - 1
    assert len(buf_g) - len(buf) == 3 * (32 * ln - 16) + 32 * (2 * lw + lb)
    for pos in (40, len(buf) // 3, len(buf) // 2, len(buf) - 5):
        bad = bytearray(buf)
        bad[pos] ^= 1
        with pytest.raises(AssertionError):
            P.aggregate_ft_verify(bytes(bad), Transcript(21))


@pytest.mark.parametrize("n_layers,width,batch,steps", [(2, 8, 4, 2), (4, 4, 2, 1), (2, 4, 2, 4)])
def test_aggregate_linked_claims_are_evaluations_of_the_stacks(n_layers, width, batch, steps):
    """Every claim the linked proof leaves is the MLE of the tensor it names at the point it
    names (Sec. 4: one sumcheck's outputs are the next one's inputs; Eq. sc-reindex for the
    shifted stacks)."""
    wit = fcnn_window(CONFIG_SEED + 200 + n_layers, n_layers=n_layers, width=width, batch=batch, steps=steps)
    n = n_layers * steps
    ts = Transcript(13)
    buf, infos = P.aggregate_linked_prove(wit, ts)
    tv = Transcript(13)
    left = P.aggregate_linked_verify(buf, tv)
    assert tv.digest() == ts.digest()
    a, wt, gz = (np.asarray(wit[k]).astype(object) for k in ("A", "W", "GZ"))
    for name, stack in (("A", a), ("W", wt), ("GZ", gz)):
        for point, value in left[name]:
            assert value == mle_eval(fr_array(stack), point), name
    z = np.einsum("nij,njk->nik", a, wt)
    point, value = left["Zlast"]
    assert value == mle_eval(fr_array(z[n_layers - 1::n_layers]), point)
    point, value = left["GZlast"]
    assert value == mle_eval(fr_array(gz[n_layers - 1::n_layers]), point)
    point, value = left["GW"]
    assert value == mle_eval(fr_array(np.einsum("nbi,nbk->nik", a, gz)), point)
    # zkReLU ran at the points the matmul sumchecks left, on the stacks the witness holds
    f = infos["fwd"]
    ln = ilog2(n)
    zk = infos["zkrelu"]
    assert zk["u_z"] == f["w"] + f["u0"] + f["u1"] and zk["u_a"] == f["v"][:ln] + f["u0"] + f["v"][ln:]
    assert zk["c_in"][0] == mle_eval(fr_array(np.asarray(wit["Zr"])), zk["u_z"])
    # the shifted stack of A is what ReLU put out
    a_out = np.zeros_like(a)
    for k in range(n):
        if k % n_layers != n_layers - 1:
            a_out[k] = a[k + 1]
    assert zk["c_in"][1] == mle_eval(fr_array(a_out), zk["u_a"])
    # any flipped byte is rejected
    for off in (40, 32 + 16 + 5, len(buf) // 3, len(buf) // 2, 2 * len(buf) // 3, len(buf) - 40, len(buf) - 1):
        bad = bytearray(buf)
        bad[off] ^= 1
        with pytest.raises((AssertionError, struct.error, ValueError)):
            P.aggregate_linked_verify(bytes(bad), Transcript(13))


def test_aggregate_linked_prover_refuses_an_inconsistent_window():
    base = fcnn_window(CONFIG_SEED + 202, n_layers=2, width=4, batch=2, steps=2)
    # the input of layer 2 is not the ReLU output of layer 1
    wit = dict(base)
    wit["A"] = np.array(base["A"], copy=True)
    wit["A"][1, 0, 0] += 1
    with pytest.raises(AssertionError):
        P.aggregate_linked_prove(wit, Transcript(1))
    # G_A is not the product of the next layer's G_Z and W
    wit = dict(base)
    wit["GA"] = np.array(base["GA"], copy=True)
    wit["GA"][0, 0, 0] += 1 << 16
    with pytest.raises(AssertionError):
        P.aggregate_linked_prove(wit, Transcript(1))
    # a weight of layer 2 changed after the gradient was taken
    wit = dict(base)
    wit["W"] = np.array(base["W"], copy=True)
    wit["W"][1, 0, 0] += 1
    with pytest.raises(AssertionError):
        P.aggregate_linked_prove(wit, Transcript(1))
