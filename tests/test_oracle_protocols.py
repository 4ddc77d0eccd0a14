"""Pins for the oracle's sumcheck prover and the matmul / Hadamard instances."""
import itertools

import numpy as np
import pytest

from oracle.field import R_MOD, fr_array, to_le
from oracle.mle import mle_eval, beta_table, ilog2
from oracle.sumcheck import lagrange_eval, prove, SumcheckProof
from oracle import protocols as P
from oracle.transcript import Transcript

rng = np.random.default_rng(23)


def rand_fr(n):
    return [int.from_bytes(rng.bytes(40), "little") % R_MOD for _ in range(n)]


def test_lagrange_on_known_polynomials():
    # x^3 through its values at 0..3 ; 2x^2 - 3x + 5 through 0..2
    assert lagrange_eval([0, 1, 8, 27], 5) == 125
    assert lagrange_eval([0, 1, 8, 27], R_MOD - 2) == (-8) % R_MOD
    assert lagrange_eval([5, 4, 7], 10) == 175
    ys = rand_fr(4)
    for k in range(4):
        assert lagrange_eval(ys, k) == ys[k]


@pytest.mark.parametrize("k,d", [(1, 3), (2, 4), (3, 5), (3, 1)])
def test_product_sumcheck_against_brute_force(k, d):
    tabs = [fr_array(rand_fr(1 << d)) for _ in range(k)]
    ts = Transcript(3)
    buf, proof, vs = P.product_prove(tabs, ts)
    # claim_0 is the sum over the Boolean hypercube, written as a plain loop
    brute = 0
    for b in range(1 << d):
        term = 1
        for t in tabs:
            term = term * t[b] % R_MOD
        brute = (brute + term) % R_MOD
    assert proof.claim0 == brute
    # every round polynomial equals the definition: bind the past challenges, set
    # the current variable to x, sum the rest over Boolean values
    for t, g in enumerate(proof.rounds):
        for x in range(k + 1):
            acc = 0
            for rest in itertools.product((0, 1), repeat=d - t - 1):
                pt = vs[:t] + [x] + list(rest)
                term = 1
                for tab in tabs:
                    term = term * mle_eval(tab, pt) % R_MOD
                acc = (acc + term) % R_MOD
            assert g[x] == acc
    # finals are the evaluations of the original tables at the challenge point
    assert proof.finals == [mle_eval(t, vs) for t in tabs]
    # bytes round-trip and the verifier accepts, ending in the same transcript state
    assert SumcheckProof.from_bytes(buf)[0].to_bytes() == buf
    assert len(buf) == 16 + 32 * (1 + d * (k + 1) + k)
    tv = Transcript(3)
    P.product_verify(buf, k, d, tv)
    assert tv.digest() == ts.digest() and tv.challenges == ts.challenges


def test_product_sumcheck_transcript_stream_written_out():
    """The Fiat-Shamir schedule of a product sumcheck, rebuilt as one explicit byte stream from
    the proof: header, claim_0, per round g_t without g_t(1), one draw per round, finals."""
    import hashlib
    import struct
    k, d = 3, 3
    tabs = [fr_array(rand_fr(1 << d)) for _ in range(k)]
    ts = Transcript(12)
    _, proof, vs = P.product_prove(tabs, ts)

    def frame(label, data):
        return bytes([len(label)]) + label + struct.pack("<Q", len(data)) + data
    stream = b"zkdl-mi355x/v3" + b"\0" * 42 + struct.pack("<Q", 12)
    stream += frame(b"sumcheck_product", struct.pack("<II", k, d))
    stream += frame(b"c", to_le(proof.claim0))
    for t, g in enumerate(proof.rounds):
        stream += frame(b"g", to_le(g[0]) + to_le(g[2]) + to_le(g[3]))
        halves = [hashlib.sha256(stream + bytes([tag]) + struct.pack("<I", 0)).digest() for tag in (0xF0, 0xF1)]
        assert vs[t] == int.from_bytes(halves[0] + halves[1], "little") % R_MOD
        stream += b"\xf2"
        stream += b"\0" * (-len(stream) % 64)
    stream += frame(b"f", b"".join(to_le(x) for x in proof.finals))
    assert ts.digest() == hashlib.sha256(stream).digest()


def test_product_verifier_rejects_any_tampered_element():
    tabs = [fr_array(rand_fr(8)) for _ in range(3)]
    buf, _, _ = P.product_prove(tabs, Transcript(1))
    n_el = (len(buf) - 16) // 32
    for e in range(n_el):
        bad = bytearray(buf)
        bad[16 + 32 * e] ^= 1
        with pytest.raises(AssertionError):
            P.product_verify(bytes(bad), 3, 3, Transcript(1))


def test_prover_asserts_on_inconsistent_tables():
    # a planted mistake in the oracle's own fold must trip its round invariant:
    # here the "table" is changed between claim and rounds by a wrong term list
    tabs = [fr_array(rand_fr(8)) for _ in range(2)]
    ts = Transcript(1)
    good, _ = prove(tabs, [(1, [0, 1])], 2, ts)
    ts = Transcript(1)
    with pytest.raises(AssertionError):
        prove(tabs, [(1, [0, 1])], 1, ts)      # degree too low: g(v) != next sum


@pytest.mark.parametrize("n,d1,d2,d3", [(1, 4, 8, 2), (4, 2, 4, 8), (2, 1, 2, 1)])
def test_matmul_claim_is_mle_of_integer_matmul(n, d1, d2, d3):
    x0 = rng.integers(-2 ** 31, 2 ** 31, (n, d1, d2))
    x1 = rng.integers(-2 ** 31, 2 ** 31, (n, d2, d3))
    y = np.einsum("nij,njk->nik", x0.astype(object), x1.astype(object))   # exact integers
    ts = Transcript(4)
    buf, proof, pts = P.matmul_prove(fr_array(x0), [n, d1, d2], fr_array(x1), [n, d2, d3], ts)
    assert proof.claim0 == mle_eval(fr_array(y), pts["w"] + pts["u0"] + pts["u1"])
    ln = len(pts["w"])
    vn, vi = pts["v"][:ln], pts["v"][ln:]
    assert proof.finals[0] == mle_eval(beta_table(pts["w"]), vn)
    assert proof.finals[1] == mle_eval(fr_array(x0), vn + pts["u0"] + vi)
    assert proof.finals[2] == mle_eval(fr_array(x1), vn + vi + pts["u1"])
    tv = Transcript(4)
    P.matmul_verify(buf, n, d1, d2, d3, tv)
    assert tv.digest() == ts.digest()
    bad = bytearray(buf)
    bad[16 + 32 * 3] ^= 1
    with pytest.raises(AssertionError):
        P.matmul_verify(bytes(bad), n, d1, d2, d3, Transcript(4))


def test_hadamard_claim_is_mle_of_integer_product():
    shape = (2, 4, 4)
    x0 = rng.integers(-2 ** 31, 2 ** 31, shape)
    x1 = rng.integers(-2 ** 31, 2 ** 31, shape)
    y = x0.astype(object) * x1.astype(object)
    ts = Transcript(6)
    buf, proof, pts = P.hadamard_prove(fr_array(x0), fr_array(x1), ts)
    assert proof.claim0 == mle_eval(fr_array(y), pts["p"])
    assert proof.finals[1] == mle_eval(fr_array(x0), pts["v"])
    assert proof.finals[2] == mle_eval(fr_array(x1), pts["v"])
    tv = Transcript(6)
    P.hadamard_verify(buf, 5, tv)
    assert tv.digest() == ts.digest()


# ---- optimized aggregated matrix-product protocol (App. B) ----
@pytest.mark.parametrize("n,d1,d2,d3", [(4, 2, 4, 2), (1, 2, 8, 4), (8, 1, 2, 1), (2, 4, 1, 2)])
def test_matmul_ft_against_definitions(n, d1, d2, d3):
    """Every message of the optimized protocol against its definition written out with MLE
    evaluations: claim_0 = Y~(w,u0,u1) for the integer product Y, f_t(x) as the double sum over
    n' and i, the finals as evaluations of the inputs; and the verifier accepts."""
    rng = np.random.default_rng(n * 100 + d2)
    x0 = rng.integers(-9, 10, (n, d1, d2))
    x1 = rng.integers(-9, 10, (n, d2, d3))
    ts = Transcript(14)
    buf, info = P.matmul_ft_prove(fr_array(x0), [n, d1, d2], fr_array(x1), [n, d2, d3], ts)
    w, u0, u1, vs = info["w"], info["u0"], info["u1"], info["v"]
    ln, l2 = len(w), d2.bit_length() - 1
    y = np.einsum("nij,njk->nik", x0.astype(object), x1.astype(object))
    assert info["claim0"] == mle_eval(fr_array(y), w + u0 + u1)
    f0, f1 = fr_array(x0), fr_array(x1)
    for t, f in enumerate(info["stack_rounds"]):
        rest = ln - t - 1
        for x in range(3):
            acc = 0
            for npr in itertools.product((0, 1), repeat=rest):
                wt = 1
                for k, bit in enumerate(npr):
                    wt = wt * (w[t + 1 + k] if bit else 1 - w[t + 1 + k]) % R_MOD
                for i in range(d2):
                    ibits = [(i >> (l2 - 1 - k)) & 1 for k in range(l2)]
                    npt = vs[:t] + [x] + list(npr)
                    a = mle_eval(f0, npt + u0 + ibits)
                    b = mle_eval(f1, npt + ibits + u1)
                    acc = (acc + wt * a % R_MOD * b) % R_MOD
            assert f[x] == acc
    assert info["inner"].finals == [mle_eval(f0, vs[:ln] + u0 + vs[ln:]), mle_eval(f1, vs[:ln] + vs[ln:] + u1)]
    assert len(buf) == 16 + 32 + 96 * ln + 16 + 32 * (1 + 3 * l2 + 2)
    tv = Transcript(14)
    claim0, finals, pts = P.matmul_ft_verify(buf, n, d1, d2, d3, tv)
    assert claim0 == info["claim0"] and finals == info["inner"].finals and pts["v"] == vs
    assert tv.digest() == ts.digest()


def test_matmul_ft_verifier_rejects_tampering():
    """Flip one bit in every field element of the proof: the verifier either rejects, or - for
    the two kinds of value it hands to its caller to check against Y and the inputs, claim_0 and
    the finals - returns a value that differs from the honest one."""
    rng = np.random.default_rng(5)
    n, d1, d2, d3 = 4, 2, 4, 2
    x0 = rng.integers(-9, 10, (n, d1, d2))
    x1 = rng.integers(-9, 10, (n, d2, d3))
    buf, info = P.matmul_ft_prove(fr_array(x0), [n, d1, d2], fr_array(x1), [n, d2, d3], Transcript(2))
    honest = (info["claim0"], info["inner"].finals)
    inner_at = 16 + 32 + 96 * 2
    slots = list(range(16, inner_at, 32)) + list(range(inner_at + 16, len(buf), 32))
    assert len(slots) == 1 + 3 * 2 + 1 + 3 * 2 + 2
    caught = 0
    for off in slots:
        bad = bytearray(buf)
        bad[off] ^= 1
        try:
            claim0, finals, _ = P.matmul_ft_verify(bytes(bad), n, d1, d2, d3, Transcript(2))
        except AssertionError:
            caught += 1
            continue
        assert (claim0, finals) != honest
    assert caught >= len(slots) - 3      # all but claim_0 and the two finals are rejected outright


# ---- re-indexing of stacked tensors (Eq. sc-reindex) ----
def _reindex_case(seed, n, d, maps):
    rng = np.random.default_rng(seed)
    x = rng.integers(-1000, 1000, (n, d))
    points = [rand_fr(len(m).bit_length() - 1) for m in maps]
    u = rand_fr(d.bit_length() - 1)
    return x, points, u


@pytest.mark.parametrize("n,d,maps", [
    (4, 8, [[0, 1, 2, 3], [1, 2, 3, -1]]),                  # all layers / all but the first, padded
    (8, 4, [[7, 6, 5, 4, 3, 2, 1, 0], [2, 5], [0, 0, 3, -1]]),
    (1, 2, [[0]]),
    (2, 1, [[1, 0], [0, -1]]),
])
def test_reindex_against_definitions(n, d, maps):
    """The claims are the MLEs of the explicitly re-stacked tensors; the relation of
    Eq. sc-reindex holds as a plain sum; the final claim is X~(v, u); the verifier accepts."""
    x, points, u = _reindex_case(n * 10 + d, n, d, maps)
    ts = Transcript(4)
    buf, info = P.reindex_prove(fr_array(x), n, d, maps, points, u, ts)
    fx = fr_array(x)
    for k, m in enumerate(maps):
        sub = np.array([x[i] if i >= 0 else np.zeros(d, dtype=x.dtype) for i in m])     # X_k, re-stacked
        assert info["claims"][k] == mle_eval(fr_array(sub), points[k] + u)
    lhs = sum(rk * ck for rk, ck in zip(info["r"], info["claims"])) % R_MOD
    ln = n.bit_length() - 1
    rhs = 0
    for i in range(n):
        ibits = [(i >> (ln - 1 - b)) & 1 for b in range(ln)]
        rhs = (rhs + info["weights"][i] * mle_eval(fx, ibits + u)) % R_MOD
    assert lhs == rhs == info["inner"].claim0
    assert info["inner"].finals[1] == mle_eval(fx, info["v"] + u)
    tv = Transcript(4)
    claims, vs, xw = P.reindex_verify(buf, n, d, maps, points, u, tv)
    assert claims == info["claims"] and vs == info["v"] and xw == info["inner"].finals[1]
    assert tv.digest() == ts.digest()


def test_reindex_verifier_rejects_tampering_and_wrong_maps():
    n, d, maps = 4, 8, [[0, 1, 2, 3], [1, 2, 3, -1]]
    x, points, u = _reindex_case(3, n, d, maps)
    buf, info = P.reindex_prove(fr_array(x), n, d, maps, points, u, Transcript(4))
    k = len(maps)
    inner_at = 16 + 32 * k
    slots = list(range(16, inner_at, 32)) + list(range(inner_at + 16, len(buf), 32))
    for off in slots:
        bad = bytearray(buf)
        bad[off] ^= 1
        with pytest.raises(AssertionError):
            claims, _, xw = P.reindex_verify(bytes(bad), n, d, maps, points, u, Transcript(4))
            # a changed sub-stack claim or final X~ is caught by whoever holds those values
            assert claims == info["claims"] and xw == info["inner"].finals[1]
    with pytest.raises(AssertionError):
        P.reindex_verify(buf, n, d, [[0, 1, 2, 3], [1, 2, 3, 0]], points, u, Transcript(4))


@pytest.mark.parametrize("d,k", [(3, 2), (4, 3), (0, 2), (5, 1)])
def test_merge_against_definitions(d, k):
    """Several claims on one tensor become one: the claims are MLE evaluations, the combined
    claim is the plain sum over the cube of P[b] X(b), the claim left is X~(v)."""
    rng = np.random.default_rng(400 + 10 * d + k)
    x = fr_array(rng.integers(-1000, 1000, 1 << d))
    pts = [[int.from_bytes(rng.bytes(40), "little") % R_MOD for _ in range(d)] for _ in range(k)]
    ts = Transcript(15)
    buf, info = P.merge_prove(x, pts, ts)
    assert info["claims"] == [mle_eval(x, pt) for pt in pts]
    weights = [sum(r * int(beta_table(pt)[b]) for r, pt in zip(info["r"], pts)) % R_MOD for b in range(1 << d)]
    assert info["inner"].claim0 == sum(w * int(v) for w, v in zip(weights, x)) % R_MOD
    tv = Transcript(15)
    claims, vs, left = P.merge_verify(buf, d, pts, tv)
    assert tv.digest() == ts.digest() and claims == info["claims"]
    assert left == mle_eval(x, vs)
    # inside a larger proof the header is short and the transcript differs
    buf2, _ = P.merge_prove(x, pts, Transcript(15), bind_statement=False)
    assert buf2[:16] == buf[:16] and (d == 0 or buf2 != buf)
    P.merge_verify(buf2, d, pts, Transcript(15), bind_statement=False)


def test_merge_verifier_rejects_tampering_and_wrong_points():
    rng = np.random.default_rng(77)
    d = 3
    x = fr_array(rng.integers(-50, 50, 8))
    pts = [[int.from_bytes(rng.bytes(40), "little") % R_MOD for _ in range(d)] for _ in range(2)]
    buf, _ = P.merge_prove(x, pts, Transcript(16))
    P.merge_verify(buf, d, pts, Transcript(16))
    for off in list(range(16, len(buf), 37)) + [len(buf) - 1]:
        bad = bytearray(buf)
        bad[off] ^= 1
        with pytest.raises(AssertionError):
            P.merge_verify(bytes(bad), d, pts, Transcript(16))
    for bind in (True, False):
        b2, _ = P.merge_prove(x, pts, Transcript(16), bind_statement=bind)
        other = [list(pts[0]), list(pts[1])]
        other[1][2] = (other[1][2] + 1) % R_MOD
        with pytest.raises(AssertionError):
            P.merge_verify(b2, d, other, Transcript(16), bind_statement=bind)


@pytest.mark.parametrize("n,d,k", [(4, 8, 2), (2, 4, 3), (1, 8, 2), (8, 1, 2), (4, 4, 1), (2, 2, 5)])
def test_stack_merge_against_definitions(n, d, k):
    """The two-step merge on a stack: claims are MLE evaluations; the inner sumcheck's claim is
    the plain double sum over (k, x); its final on T is the combination of evaluations at the
    common inner point v that Eq. sc-reindex starts from; the claim left is X~(v_n, v)."""
    rng = np.random.default_rng(500 + 100 * n + 10 * d + k)
    flat = fr_array(rng.integers(-1000, 1000, (n, d)))
    x = np.asarray(flat, dtype=object).reshape(n, d)
    ln, ld = ilog2(n), ilog2(d)
    pts = [[int.from_bytes(rng.bytes(40), "little") % R_MOD for _ in range(ln + ld)] for _ in range(k)]
    ts = Transcript(17)
    buf, info = P.stack_merge_prove(flat, n, d, pts, ts)
    assert info["claims"] == [mle_eval(flat, pt) for pt in pts]
    r, rho, v, vn = info["r"], info["rho"], info["v"], info["vn"]
    # inner claim: sum_k r_k sum_x beta~(q_k, x) X~(s_k, x), every X~(s_k, x) from the definition
    total = 0
    for rk, pt in zip(r, pts):
        bs, bq = beta_table(pt[:ln]), beta_table(pt[ln:])
        for xx in range(d):
            t = sum(int(bs[i]) * int(x[i, xx]) for i in range(n)) % R_MOD
            total += rk * int(bq[xx]) * t
    assert info["inner"].claim0 == total % R_MOD
    b_rho = beta_table(rho)
    assert info["inner"].finals[1] == sum(int(b_rho[j]) * mle_eval(flat, pt[:ln] + v)
                                          for j, pt in enumerate(pts)) % R_MOD
    assert info["outer"].claim0 == info["inner"].finals[1]
    assert info["outer"].finals[1] == mle_eval(flat, vn + v)
    tv = Transcript(17)
    claims, point, left = P.stack_merge_verify(buf, n, d, pts, tv)
    assert tv.digest() == ts.digest() and claims == info["claims"]
    assert point == vn + v and left == mle_eval(flat, point)
    buf2, _ = P.stack_merge_prove(flat, n, d, pts, Transcript(17), bind_statement=False)
    P.stack_merge_verify(buf2, n, d, pts, Transcript(17), bind_statement=False)
    assert buf2[:16] == buf[:16]


def test_stack_merge_verifier_rejects_tampering_and_wrong_points():
    rng = np.random.default_rng(78)
    n, d = 4, 4
    x = fr_array(rng.integers(-50, 50, n * d))
    pts = [[int.from_bytes(rng.bytes(40), "little") % R_MOD for _ in range(4)] for _ in range(2)]
    buf, _ = P.stack_merge_prove(x, n, d, pts, Transcript(18))
    P.stack_merge_verify(buf, n, d, pts, Transcript(18))
    for off in list(range(16, len(buf), 41)) + [len(buf) - 1]:
        bad = bytearray(buf)
        bad[off] ^= 1
        with pytest.raises(AssertionError):
            P.stack_merge_verify(bytes(bad), n, d, pts, Transcript(18))
    for bind in (True, False):
        b2, _ = P.stack_merge_prove(x, n, d, pts, Transcript(18), bind_statement=bind)
        for which in (0, 3):       # a stack coordinate, an inner coordinate
            other = [list(pts[0]), list(pts[1])]
            other[1][which] = (other[1][which] + 1) % R_MOD
            with pytest.raises(AssertionError):
                P.stack_merge_verify(b2, n, d, other, Transcript(18), bind_statement=bind)


# --------------------------------------------------------------------------
# general aggregated form (Eq. tensor-op-aggr, Protocol tensor-op-aggr)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("n,d1,d2,d3", [(4, 2, 4, 2), (1, 2, 2, 4), (2, 1, 8, 1), (8, 2, 1, 2), (1, 1, 1, 1)])
def test_matmul_general_form(n, d1, d2, d3):
    """Honest stacks: the verifier accepts, the finals are the MLEs of Y, X0, X1 at the challenge point, and
    every f_t(x) equals the triple sum of Protocol tensor-op-aggr written out with MLE evaluations."""
    rng = np.random.default_rng(1000 * n + 10 * d2 + d3)
    x0 = rng.integers(-50, 50, (n, d1, d2)).astype(object)
    x1 = rng.integers(-50, 50, (n, d2, d3)).astype(object)
    y = np.einsum("nij,njk->nik", x0, x1)
    ts = Transcript(41)
    buf, info = P.matmul_general_prove(fr_array(x0), [n, d1, d2], fr_array(x1), [n, d2, d3], fr_array(y), ts)
    tv = Transcript(41)
    finals, pts = P.matmul_general_verify(buf, n, d1, d2, d3, tv)
    assert tv.digest() == ts.digest() and pts["v"] == info["v"]
    ln, l1, l2, l3 = (k.bit_length() - 1 for k in (n, d1, d2, d3))
    v = info["v"]
    vn, vi0, vi1, vj = v[:ln], v[ln:ln + l1], v[ln + l1:ln + l1 + l3], v[ln + l1 + l3:]
    assert finals[0] == mle_eval(fr_array(y), vn + vi0 + vi1)
    assert finals[1] == mle_eval(fr_array(x0), vn + vi0 + vj)
    assert finals[2] == mle_eval(fr_array(x1), vn + vj + vi1)
    # f_t(x) from the definition: sum over n', i, j of beta~(w_[t+1:], n') beta~(u, i) (Y/D_in - X0 X1) at (v_<t, x, n')
    dinv = pow(d2, -1, R_MOD)
    bu = beta_table(info["u"])
    for t in range(ln):
        bs = beta_table(info["w"][t + 1:])
        for x in range(3):
            tot = 0
            for np_ in range(1 << (ln - t - 1)):
                pn = v[:t] + [x] + P.index_bits(np_, ln - t - 1)
                for i in range(d1 * d3):
                    i0, i1 = divmod(i, d3)
                    bi0, bi1 = P.index_bits(i0, l1), P.index_bits(i1, l3)
                    acc = mle_eval(fr_array(y), pn + bi0 + bi1)
                    for j in range(d2):
                        bj = P.index_bits(j, l2)
                        acc -= mle_eval(fr_array(x0), pn + bi0 + bj) * mle_eval(fr_array(x1), pn + bj + bi1)
                    tot += int(bs[np_]) * int(bu[i]) * acc
            assert info["stack_rounds"][t][x] == tot % R_MOD, (t, x)
    del dinv
    # tampering
    for pos in (36, len(buf) // 2, len(buf) - 4):
        bad = bytearray(buf)
        bad[pos] ^= 1
        with pytest.raises(AssertionError):
            P.matmul_general_verify(bytes(bad), n, d1, d2, d3, Transcript(41))


def test_matmul_general_form_refuses_a_wrong_product():
    rng = np.random.default_rng(77)
    x0 = rng.integers(-9, 9, (2, 2, 4)).astype(object)
    x1 = rng.integers(-9, 9, (2, 4, 2)).astype(object)
    y = np.einsum("nij,njk->nik", x0, x1)
    y[1, 0, 1] += 1
    with pytest.raises(AssertionError):
        P.matmul_general_prove(fr_array(x0), [2, 2, 4], fr_array(x1), [2, 4, 2], fr_array(y), Transcript(1))
