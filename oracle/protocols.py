"""The sumcheck instances of zkDL: product, matmul, Hadamard, zkReLU, aggregate.

Each prover draws its points from the transcript, runs the textbook sumcheck of
`oracle.sumcheck`, and returns proof bytes in the format the HIP library also
emits (layout in the repository's design notes).  Each has a verifier that
replays the transcript and checks the final claim against the reported finals.
Test infrastructure; not used by the product.
"""
import struct

import numpy as np

from .field import R_MOD, fr_array, to_le, from_le
from .mle import ilog2, beta_table, mle_eval, partial_eval
from .sumcheck import SumcheckProof, prove, verify_rounds, lagrange_eval as _lagrange

ZKRL_MAGIC = 0x4C524B5A   # bytes "ZKRL"
ZKAG_MAGIC = 0x47414B5A   # bytes "ZKAG"


def beta_point(u, v):
    """beta~(u, v) for two field points: prod_k (u_k v_k + (1-u_k)(1-v_k))."""
    assert len(u) == len(v)
    acc = 1
    for a, b in zip(u, v):
        acc = acc * ((a * b + (1 - a) * (1 - b)) % R_MOD) % R_MOD
    return acc


def index_bits(index, nbits):
    """Boolean point of an index, most significant bit first."""
    return [(index >> (nbits - 1 - k)) & 1 for k in range(nbits)]


# --------------------------------------------------------------------------
# generic product of K tables (the micro-benchmark instance)
# --------------------------------------------------------------------------
def product_prove(tables, ts):
    k = len(tables)
    d = ilog2(len(tables[0]))
    ts.absorb_u32(b"sumcheck_product", [k, d])
    proof, vs = prove(tables, [(1, list(range(k)))], k, ts)
    return proof.to_bytes(), proof, vs


def product_verify(buf, k, d, ts):
    proof, _ = SumcheckProof.from_bytes(buf)
    assert proof.n_finals == k and proof.degree == k and len(proof.rounds) == d
    ts.absorb_u32(b"sumcheck_product", [k, d])
    claim, vs = verify_rounds(proof, ts)
    prod = 1
    for f in proof.finals:
        prod = prod * f % R_MOD
    assert prod == claim, "final claim != product of finals"
    return proof, vs


# --------------------------------------------------------------------------
# batched matrix product (Eq. exm-matmul-batched)
# --------------------------------------------------------------------------
def matmul_prove(x0, shape0, x1, shape1, ts):
    """Y[n] = X0[n] X1[n], X0 [N,D1,D2], X1 [N,D2,D3]: prove
    Y~(w,u0,u1) = sum_{n,i} beta~(w,n) X0~(n,u0,i) X1~(n,i,u1).
    Draws w, u0, u1 in that order.  Finals: beta~(w,v_n), X0~(v_n,u0,v_i),
    X1~(v_n,v_i,u1)."""
    n, d1, d2 = shape0
    n_, d2_, d3 = shape1
    assert n == n_ and d2 == d2_
    ts.absorb_u32(b"sumcheck_matmul", [n, d1, d2, d3])
    ln, l1, l3 = ilog2(n), ilog2(d1), ilog2(d3)
    pt = ts.challenges_vec(ln + l1 + l3)          # the point (w, u0, u1): one draw
    w, u0, u1 = pt[:ln], pt[ln:ln + l1], pt[ln + l1:]
    t0, _ = partial_eval(x0, [n, d1, d2], 1, 2, u0)          # [N, D2]
    t1, _ = partial_eval(x1, [n, d2, d3], 2, 3, u1)          # [N, D2]
    tb = np.repeat(beta_table(w), d2)                         # beta~(w,n), every i
    proof, vs = prove([tb, t0, t1], [(1, [0, 1, 2])], 3, ts)
    return proof.to_bytes(), proof, dict(w=w, u0=u0, u1=u1, v=vs)


def matmul_verify(buf, n, d1, d2, d3, ts):
    proof, _ = SumcheckProof.from_bytes(buf)
    assert proof.n_finals == 3 and proof.degree == 3
    assert len(proof.rounds) == ilog2(n) + ilog2(d2)
    ts.absorb_u32(b"sumcheck_matmul", [n, d1, d2, d3])
    ln, l1, l3 = ilog2(n), ilog2(d1), ilog2(d3)
    pt = ts.challenges_vec(ln + l1 + l3)          # the point (w, u0, u1): one draw
    w, u0, u1 = pt[:ln], pt[ln:ln + l1], pt[ln + l1:]
    claim, vs = verify_rounds(proof, ts)
    fb, f0, f1 = proof.finals
    assert fb == beta_point(w, vs[:len(w)]), "beta final is not beta~(w, v_n)"
    assert fb * f0 % R_MOD * f1 % R_MOD == claim, "final claim mismatch"
    return proof, dict(w=w, u0=u0, u1=u1, v=vs)


# --------------------------------------------------------------------------
# batched matrix product, optimized aggregated protocol (App. B, Protocol
# tensor-op-aggr-optimized; Eqs. tensor-op-aggr-optimized, tensor-op-compressed-optimized)
# --------------------------------------------------------------------------
FT_MAGIC = 0x46534B5A   # "ZKSF"


def matmul_ft_prove(x0, shape0, x1, shape1, ts):
    """Y[n] = X0[n] X1[n] with the prover's messages of the optimized protocol.

    Stack rounds t = 0..log N - 1: the prover sends, at x = 0, 1, 2,
      f_t(x) = sum_{n'} beta~(w_[t+1:], n') sum_i X0~(v_<t, x, n', u0, i) X1~(v_<t, x, n', i, u1),
    that is the round polynomial WITHOUT its factor beta~(w_t, x) (degree 2 instead of 3, and
    no table for beta~(w, .) is ever folded); the verifier forms g_t(x) = beta~(w_t, x) f_t(x)
    and checks g_t(0) + g_t(1) = claim, where claim is Y~(w, u0, u1) for t = 0 and
    f_{t-1}(v_{t-1}) afterwards.  With the stack bound, the sumcheck of a single matrix
    product follows on f_{n-1}(v_{n-1}) = sum_i X0~(v, u0, i) X1~(v, i, u1): K = 2, degree 2.

    Transcript: header "sumcheck_matmul_ft" (N, D1, D2, D3); one draw (w, u0, u1); "c"
    claim_0; per stack round "f" (f_t(0), f_t(1), f_t(2)) and a draw; then the product
    sumcheck's rounds and finals (its claim_0 is not absorbed: the transcript fixes it).
    Proof bytes: "ZKSF", u32 log N, u32 log D2, u32 0, claim_0, log N x 3 evaluations,
    then the SC block of the second part (finals X0~(v_n, u0, v_i), X1~(v_n, v_i, u1)).
    """
    n, d1, d2 = shape0
    n_, d2_, d3 = shape1
    assert n == n_ and d2 == d2_
    ts.absorb_u32(b"sumcheck_matmul_ft", [n, d1, d2, d3])
    ln, l1, l2, l3 = ilog2(n), ilog2(d1), ilog2(d2), ilog2(d3)
    pt = ts.challenges_vec(ln + l1 + l3)          # the point (w, u0, u1): one draw
    w, u0, u1 = pt[:ln], pt[ln:ln + l1], pt[ln + l1:]
    t0, _ = partial_eval(x0, [n, d1, d2], 1, 2, u0)          # [N, D2]
    t1, _ = partial_eval(x1, [n, d2, d3], 2, 3, u1)          # [N, D2]
    cur0 = np.asarray(t0, dtype=object).reshape(n, d2)
    cur1 = np.asarray(t1, dtype=object).reshape(n, d2)
    bw = beta_table(w)
    claim0 = 0
    for row in range(n):
        claim0 = (claim0 + int(bw[row]) * int(np.sum(cur0[row] * cur1[row]) % R_MOD)) % R_MOD
    ts.absorb_fr(b"c", [claim0])
    claim = claim0
    stack_rounds, vs = [], []
    for t in range(ln):
        half = cur0.shape[0] // 2
        bs = beta_table(w[t + 1:])                           # beta~(w_[t+1:], n'), half entries
        lo0, hi0, lo1, hi1 = cur0[:half], cur0[half:], cur1[:half], cur1[half:]
        f = []
        for x in range(3):
            a = (lo0 + x * (hi0 - lo0)) % R_MOD
            b = (lo1 + x * (hi1 - lo1)) % R_MOD
            tot = 0
            for row in range(half):
                tot = (tot + int(bs[row]) * int(np.sum(a[row] * b[row]) % R_MOD)) % R_MOD
            f.append(tot)
        assert ((1 - w[t]) * f[0] + w[t] * f[1]) % R_MOD == claim, "stack round invariant broken"
        ts.absorb_fr(b"f", f)
        v = ts.challenge()
        cur0 = (lo0 + v * (hi0 - lo0)) % R_MOD
        cur1 = (lo1 + v * (hi1 - lo1)) % R_MOD
        claim = _lagrange(f, v)
        stack_rounds.append(f)
        vs.append(v)
    inner, vi = prove([cur0.reshape(-1), cur1.reshape(-1)], [(1, [0, 1])], 2, ts, absorb_claim=False)
    assert inner.claim0 == claim, "the single-product sumcheck does not start at f_{n-1}(v_{n-1})"
    out = [struct.pack("<IIII", FT_MAGIC, ln, l2, 0), to_le(claim0)]
    for f in stack_rounds:
        out.extend(to_le(x) for x in f)
    out.append(inner.to_bytes())
    info = dict(w=w, u0=u0, u1=u1, v=vs + vi, claim0=claim0, stack_rounds=stack_rounds, inner=inner)
    return b"".join(out), info


def matmul_ft_verify(buf, n, d1, d2, d3, ts):
    """Replays the optimized protocol; returns (claim_0, finals (X0~, X1~), points).  The caller
    checks claim_0 against Y~(w, u0, u1) and the finals against the committed tensors."""
    magic, ln, l2, zero = struct.unpack_from("<IIII", buf, 0)
    assert magic == FT_MAGIC and ln == ilog2(n) and l2 == ilog2(d2) and zero == 0
    ts.absorb_u32(b"sumcheck_matmul_ft", [n, d1, d2, d3])
    l1, l3 = ilog2(d1), ilog2(d3)
    pt = ts.challenges_vec(ln + l1 + l3)
    w, u0, u1 = pt[:ln], pt[ln:ln + l1], pt[ln + l1:]
    off = 16
    claim0 = from_le(buf[off:off + 32])
    off += 32
    ts.absorb_fr(b"c", [claim0])
    claim, vs = claim0, []
    for t in range(ln):
        f = [from_le(buf[off + 32 * x:off + 32 * x + 32]) for x in range(3)]
        off += 96
        # g_t(x) = beta~(w_t, x) f_t(x): g_t(0) + g_t(1) = (1 - w_t) f_t(0) + w_t f_t(1)
        assert ((1 - w[t]) * f[0] + w[t] * f[1]) % R_MOD == claim, "g(0)+g(1) != claim"
        ts.absorb_fr(b"f", f)
        v = ts.challenge()
        claim = _lagrange(f, v)
        vs.append(v)
    inner, end = SumcheckProof.from_bytes(buf, off)
    assert end == len(buf) and inner.n_finals == 2 and inner.degree == 2 and len(inner.rounds) == l2
    last, vi = verify_rounds(inner, ts, absorb_claim=False, expected_claim0=claim)
    assert inner.finals[0] * inner.finals[1] % R_MOD == last, "final claim mismatch"
    return claim0, inner.finals, dict(w=w, u0=u0, u1=u1, v=vs + vi)


# --------------------------------------------------------------------------
# batched matrix product, general aggregated form (Sec. 4, Eq. tensor-op-aggr; App. B, Protocol
# tensor-op-aggr): the output Y is a (committed) input of the sumcheck, not a claim
# --------------------------------------------------------------------------
GA_MAGIC = 0x41474B5A   # "ZKGA"


def matmul_general_prove(x0, shape0, x1, shape1, y, ts):
    """N instances Y[n] = X0[n] X1[n] proved from the three stacks themselves:
      0 = sum_n sum_i sum_j beta~(w, n) beta~(u, i) (D_in^{-1} Y(n, i) - X0(n, i0, j) X1(n, j, i1)),
    i = (i0, i1) the output index (D_out = D1 D3 values), j the inner index (D_in = D2), w over the stack
    and u over the output index drawn by the verifier (Eq. tensor-op-aggr with f(a, b) = a b).
    Stack rounds t = 0..log N - 1 (Protocol tensor-op-aggr): the prover sends f_t at x = 0, 1, 2, the
    round polynomial without the factor beta~(w_t, x) and with beta~(w_[t+1:], n') over the unbound stack
    variables; the verifier checks (1 - w_t) f_t(0) + w_t f_t(1) = claim (0 for t = 0, f_{t-1}(v_{t-1})
    after).  Then the textbook sumcheck of Eq. tensor-op-compressed over (i0, i1, j), in that order,
    degree 2, whose claim_0 = f_{n-1}(v_{n-1}) the transcript already fixes (not absorbed).
    Finals: Y~(v_n, v_i0, v_i1), X0~(v_n, v_i0, v_j), X1~(v_n, v_j, v_i1); beta~(u, v_i) is the verifier's.
    Transcript: header "tensor_op_aggr" (N, D1, D2, D3); one draw (w, u); per stack round "f" (three
    evaluations) and a draw; the inner rounds and finals.  Proof: "ZKGA", log N, log D1, log D3, log D2,
    0, 0, 0; log N x 3 evaluations; one SC block (3 finals, degree 2)."""
    n, d1, d2 = shape0
    n_, d2_, d3 = shape1
    assert n == n_ and d2 == d2_
    ln, l1, l2, l3 = ilog2(n), ilog2(d1), ilog2(d2), ilog2(d3)
    ts.absorb_u32(b"tensor_op_aggr", [n, d1, d2, d3])
    pt = ts.challenges_vec(ln + l1 + l3)
    w, u = pt[:ln], pt[ln:]
    m = d1 * d3 * d2
    a = np.asarray(x0, dtype=object).reshape(n, d1, 1, d2)
    b = np.transpose(np.asarray(x1, dtype=object).reshape(n, d2, d3), (0, 2, 1)).reshape(n, 1, d3, d2)
    yy = np.asarray(y, dtype=object).reshape(n, d1, d3, 1)
    ones = np.ones((n, d1, d3, d2), dtype=object)
    cur_y = (yy * ones).reshape(n, m) % R_MOD           # every table over (n; i0, i1, j), broadcast written out
    cur_0 = (a * ones).reshape(n, m) % R_MOD
    cur_1 = (b * ones).reshape(n, m) % R_MOD
    bu = np.repeat(beta_table(u), d2)                   # beta~(u, (i0, i1)), every j
    dinv = pow(d2, -1, R_MOD)

    def weighted(ty, t0, t1, bs):
        tot = 0
        for row in range(ty.shape[0]):
            tot += int(bs[row]) * int(np.sum(bu * (dinv * ty[row] - t0[row] * t1[row])) % R_MOD)
        return tot % R_MOD
    claim = 0
    assert weighted(cur_y, cur_0, cur_1, beta_table(w)) == 0, "Y is not the product of X0 and X1"
    stack_rounds, vs = [], []
    for t in range(ln):
        half = cur_y.shape[0] // 2
        bs = beta_table(w[t + 1:])
        f = []
        for x in range(3):
            at = [(c[:half] + x * (c[half:] - c[:half])) % R_MOD for c in (cur_y, cur_0, cur_1)]
            f.append(weighted(at[0], at[1], at[2], bs))
        assert ((1 - w[t]) * f[0] + w[t] * f[1]) % R_MOD == claim, "stack round invariant broken"
        ts.absorb_fr(b"f", f)
        v = ts.challenge()
        cur_y, cur_0, cur_1 = [(c[:half] + v * (c[half:] - c[:half])) % R_MOD for c in (cur_y, cur_0, cur_1)]
        claim = _lagrange(f, v)
        stack_rounds.append(f)
        vs.append(v)
    inner, vi = prove([bu, cur_y.reshape(-1), cur_0.reshape(-1), cur_1.reshape(-1)],
                      [(dinv, [0, 1]), (R_MOD - 1, [0, 2, 3])], 2, ts, absorb_claim=False,
                      report=lambda f: [f[1], f[2], f[3]])
    assert inner.claim0 == claim, "the compressed sumcheck does not start at f_{n-1}(v_{n-1})"
    out = [struct.pack("<IIIIIIII", GA_MAGIC, ln, l1, l3, l2, 0, 0, 0)]
    for f in stack_rounds:
        out.extend(to_le(x) for x in f)
    out.append(inner.to_bytes())
    info = dict(w=w, u=u, v=vs + vi, stack_rounds=stack_rounds, inner=inner)
    return b"".join(out), info


def matmul_general_verify(buf, n, d1, d2, d3, ts):
    """Replays the general aggregated protocol; returns (finals (Y~, X0~, X1~), points).  The caller checks
    the finals against the (committed) stacks: Y~ at (v_n, v_i0, v_i1), X0~ at (v_n, v_i0, v_j), X1~ at
    (v_n, v_j, v_i1)."""
    magic, ln, l1, l3, l2, z0, z1, z2 = struct.unpack_from("<IIIIIIII", buf, 0)
    assert magic == GA_MAGIC and (ln, l1, l3, l2) == (ilog2(n), ilog2(d1), ilog2(d3), ilog2(d2))
    assert z0 == z1 == z2 == 0
    ts.absorb_u32(b"tensor_op_aggr", [n, d1, d2, d3])
    pt = ts.challenges_vec(ln + l1 + l3)
    w, u = pt[:ln], pt[ln:]
    off = 32
    claim, vs = 0, []
    for t in range(ln):
        f = [from_le(buf[off + 32 * x:off + 32 * x + 32]) for x in range(3)]
        off += 96
        assert ((1 - w[t]) * f[0] + w[t] * f[1]) % R_MOD == claim, "g(0)+g(1) != claim"
        ts.absorb_fr(b"f", f)
        v = ts.challenge()
        claim = _lagrange(f, v)
        vs.append(v)
    inner, end = SumcheckProof.from_bytes(buf, off)
    assert end == len(buf) and inner.n_finals == 3 and inner.degree == 2 and len(inner.rounds) == l1 + l3 + l2
    last, vi = verify_rounds(inner, ts, absorb_claim=False, expected_claim0=claim)
    yf, f0, f1 = inner.finals
    dinv = pow(d2, -1, R_MOD)
    assert beta_point(u, vi[:l1 + l3]) * (dinv * yf - f0 * f1) % R_MOD == last, "final claim mismatch"
    return inner.finals, dict(w=w, u=u, v=vs + vi)


# --------------------------------------------------------------------------
# re-indexing of stacked tensors (Sec. 4, Eq. sc-reindex; Protocol zkdl, the re-indexing line)
# --------------------------------------------------------------------------
RI_MAGIC = 0x49524B5A   # "ZKRI"


def _reindex_statement_digest(n, d, maps, points, u):
    """SHA-256 of the public part of the statement: shapes, index maps, points."""
    import hashlib
    h = hashlib.sha256()
    h.update(struct.pack("<III", n, d, len(maps)))
    for m in maps:
        h.update(struct.pack("<I", len(m)))
        h.update(b"".join(struct.pack("<i", int(j)) for j in m))
    for pt in points:
        h.update(b"".join(to_le(x) for x in pt))
    h.update(b"".join(to_le(x) for x in u))
    return h.digest()


def _reindex_header(ts, n, d, maps, points, u, bind_statement):
    if bind_statement:
        ts.absorb(b"reindex", _reindex_statement_digest(n, d, maps, points, u))
    else:
        ts.absorb_u32(b"reindex", [n, d, len(maps)])


def reindex_weights(n, maps, points, r):
    """P[i] = sum_k r_k sum_j beta~(u_k, j) p_k(i, j), p_k(i, j) = [maps[k][j] == i]."""
    p = [0] * n
    for k, m in enumerate(maps):
        bk = beta_table(points[k])
        for j, i in enumerate(m):
            if i >= 0:
                p[i] = (p[i] + r[k] * int(bk[j])) % R_MOD
    return p


def reindex_prove(x, n, d, maps, points, u, ts, bind_statement=True):
    """K sub-stacks X_k = (X^(maps[k][0]), X^(maps[k][1]), ..) of the stack X [N, D] (an entry
    -1 is a zero tensor: padding), each with a claim X_k~(u_k, u) at its own stack point u_k
    and the common point u over the other dimensions.  With verifier coefficients r_k,
      sum_k r_k X_k~(u_k, u) = sum_i P[i] X~(i, u),  P as in reindex_weights,
    is proved by a sumcheck over i (two tables, degree 2), which leaves ONE claim X~(v, u) on
    the whole stack; the verifier evaluates P~(v) itself (Eq. sc-reindex).

    Transcript: "reindex" (digest of shapes, maps and points: they are public or come from the
    preceding sumchecks); "c" the K claims; one draw of K coefficients; then the product
    sumcheck on (P, X~(., u)) as in product_prove's rounds (its claim_0 = sum_k r_k c_k is
    absorbed like any claim_0).  Proof: "ZKRI", N, D, K, 0, the K claims, one SC block.
    bind_statement=False is the use inside a larger proof whose transcript already fixes the
    maps (public architecture) and the points (earlier challenges): "reindex" then carries
    the three words N, D, K only.
    """
    k_sub = len(maps)
    assert 1 <= k_sub <= 8 and len(points) == k_sub and len(u) == ilog2(d)
    for m, pt in zip(maps, points):
        assert len(pt) == ilog2(len(m)) and all(-1 <= int(j) < n for j in m)
    _reindex_header(ts, n, d, maps, points, u, bind_statement)
    t, _ = partial_eval(x, [n, d], 1, 2, u)                  # X~(i, u) for every i
    t = [int(v) for v in t]
    claims = []
    for m, pt in zip(maps, points):
        bk = beta_table(pt)
        claims.append(sum(int(bk[j]) * t[i] for j, i in enumerate(m) if i >= 0) % R_MOD)
    ts.absorb_fr(b"c", claims)
    r = ts.challenges_vec(k_sub)
    p = reindex_weights(n, maps, points, r)
    proof, vs = prove([np.array(p, dtype=object), np.array(t, dtype=object)], [(1, [0, 1])], 2, ts)
    assert proof.claim0 == sum(rk * ck for rk, ck in zip(r, claims)) % R_MOD
    out = [struct.pack("<IIII", RI_MAGIC, n, d, k_sub)] + [to_le(c) for c in claims] + [proof.to_bytes()]
    return b"".join(out), dict(claims=claims, r=r, v=vs, inner=proof, weights=p)


def reindex_verify(buf, n, d, maps, points, u, ts, bind_statement=True):
    """Returns (the K claims, the point v, the remaining claim X~(v, u))."""
    magic, n_, d_, k_sub = struct.unpack_from("<IIII", buf, 0)
    assert magic == RI_MAGIC and n_ == n and d_ == d and k_sub == len(maps)
    _reindex_header(ts, n, d, maps, points, u, bind_statement)
    claims = [from_le(buf[16 + 32 * k:48 + 32 * k]) for k in range(k_sub)]
    ts.absorb_fr(b"c", claims)
    r = ts.challenges_vec(k_sub)
    proof, end = SumcheckProof.from_bytes(buf, 16 + 32 * k_sub)
    assert end == len(buf) and proof.n_finals == 2 and proof.degree == 2 and len(proof.rounds) == ilog2(n)
    expect0 = sum(rk * ck for rk, ck in zip(r, claims)) % R_MOD
    last, vs = verify_rounds(proof, ts, expected_claim0=expect0)
    pw, xw = proof.finals
    assert pw * xw % R_MOD == last, "final claim mismatch"
    assert pw == mle_eval(np.array(reindex_weights(n, maps, points, r), dtype=object), vs), "P~(v) mismatch"
    return claims, vs, xw


# --------------------------------------------------------------------------
# several claims on one tensor -> one (the identity behind Eq. sc-reindex, taken over all
# variables: Protocol zkdl ends with ONE evaluation per stack to be opened)
# --------------------------------------------------------------------------
MG_MAGIC = 0x474D4B5A   # "ZKMG"


def _merge_header(ts, d, points, bind_statement):
    if bind_statement:
        import hashlib
        h = hashlib.sha256(struct.pack("<II", d, len(points)))
        for pt in points:
            h.update(b"".join(to_le(x) for x in pt))
        ts.absorb(b"merge", h.digest())
    else:
        ts.absorb_u32(b"merge", [d, len(points)])


def merge_weights(points, r):
    """P[b] = sum_k r_k beta~(p_k, b)."""
    p = np.zeros(1 << len(points[0]), dtype=object)
    for rk, pt in zip(r, points):
        p = (p + rk * beta_table(pt)) % R_MOD
    return p


def merge_prove(x, points, ts, bind_statement=True):
    """K claims X~(p_k) on one tensor X (2^d entries, every p_k over all d variables) become
    one: with verifier coefficients r_k,
      sum_k r_k X~(p_k) = sum_b P[b] X(b),  P = merge_weights(points, r),
    by the definition of the multilinear extension; a sumcheck over b (two tables, degree 2)
    leaves the single claim X~(v), and the verifier evaluates P~(v) = sum_k r_k beta~(p_k, v)
    itself.  It is Eq. sc-reindex with every sub-stack the stack itself and no common point.
    Transcript: "merge" (digest of d, K and the points; inside a larger proof that fixes the
    points, the two words d, K); "c" the K claims; one draw of K coefficients; the product
    sumcheck.  Proof: "ZKMG", d, K, 0, the K claims, one SC block."""
    d = ilog2(len(x))
    k_sub = len(points)
    assert 1 <= k_sub <= 8 and all(len(pt) == d for pt in points)
    _merge_header(ts, d, points, bind_statement)
    claims = [mle_eval(x, pt) for pt in points]
    ts.absorb_fr(b"c", claims)
    r = ts.challenges_vec(k_sub)
    proof, vs = prove([merge_weights(points, r), np.asarray(x, dtype=object)], [(1, [0, 1])], 2, ts)
    assert proof.claim0 == sum(rk * ck for rk, ck in zip(r, claims)) % R_MOD
    out = [struct.pack("<IIII", MG_MAGIC, d, k_sub, 0)] + [to_le(c) for c in claims] + [proof.to_bytes()]
    return b"".join(out), dict(claims=claims, r=r, v=vs, inner=proof)


def merge_verify(buf, d, points, ts, bind_statement=True):
    """Returns (the K claims, the point v, the remaining claim X~(v))."""
    magic, d_, k_sub, _ = struct.unpack_from("<IIII", buf, 0)
    assert magic == MG_MAGIC and d_ == d and k_sub == len(points)
    _merge_header(ts, d, points, bind_statement)
    claims = [from_le(buf[16 + 32 * k:48 + 32 * k]) for k in range(k_sub)]
    ts.absorb_fr(b"c", claims)
    r = ts.challenges_vec(k_sub)
    proof, end = SumcheckProof.from_bytes(buf, 16 + 32 * k_sub)
    assert end == len(buf) and proof.n_finals == 2 and proof.degree == 2 and len(proof.rounds) == d
    expect0 = sum(rk * ck for rk, ck in zip(r, claims)) % R_MOD
    last, vs = verify_rounds(proof, ts, expected_claim0=expect0)
    pw, xw = proof.finals
    assert pw * xw % R_MOD == last, "final claim mismatch"
    assert pw == sum(rk * beta_point(pt, vs) for rk, pt in zip(r, points)) % R_MOD, "P~(v) mismatch"
    return claims, vs, xw


MS_MAGIC = 0x534D4B5A   # "ZKMS"


def _stack_merge_header(ts, n, d, points, bind_statement):
    if bind_statement:
        import hashlib
        h = hashlib.sha256(struct.pack("<III", n, d, len(points)))
        for pt in points:
            h.update(b"".join(to_le(x) for x in pt))
        ts.absorb(b"merge_stack", h.digest())
    else:
        ts.absorb_u32(b"merge_stack", [n, d, len(points)])


def _stack_merge_tables(k_sub, r, inner_points, t_rows, d):
    """The two tables of the inner sumcheck, the claim index k as the leading variables:
    E[k, x] = r_k beta~(q_k, x), T[k, x] = X~(s_k, x); zero rows up to a power of two."""
    k_pad = 1 << max(0, (k_sub - 1).bit_length())
    e = np.zeros(k_pad * d, dtype=object)
    t = np.zeros(k_pad * d, dtype=object)
    for k in range(k_sub):
        e[k * d:(k + 1) * d] = (r[k] * beta_table(inner_points[k])) % R_MOD
        t[k * d:(k + 1) * d] = t_rows[k]
    return e, t, ilog2(k_pad)


def stack_merge_prove(x, n, d, points, ts, bind_statement=True):
    """merge_prove's statement for a stack X [N, D] at the cost of tables of D (not N D)
    entries: K claims X~(s_k, q_k), s_k over the stack axis, q_k over the rest.
    1. The prover binds the stack axis of every claim: T_k(x) = X~(s_k, x).
    2. With coefficients r_k,  sum_k r_k X~(s_k, q_k) = sum_{k, x} E[k, x] T[k, x]  (tables of
       _stack_merge_tables): one product sumcheck over (k, x), challenges (rho, v).  It leaves
       T~(rho, v) = sum_k beta~(rho, k) X~(s_k, v), a combination of claims with the common
       point v over the inner dimensions, which is the left-hand side of Eq. sc-reindex with
       the sub-stacks the stack itself and the coefficients beta~(rho, k).
    3. Eq. sc-reindex: T~(rho, v) = sum_i Pn[i] X~(i, v), Pn[i] = sum_k beta~(rho, k) beta~(s_k, i):
       a product sumcheck over i leaves the one claim X~(v_n, v).
    The verifier computes E~(rho, v) = sum_k beta~(rho, k) r_k beta~(q_k, v) and
    Pn~(v_n) = sum_k beta~(rho, k) beta~(s_k, v_n), and checks that the second sumcheck starts
    from the first one's final on T.
    Transcript: "merge_stack" (digest of N, D, K and the points; inside a larger proof the
    three words N, D, K); "c" the K claims; draw K; the two product sumchecks one after the
    other (each absorbs its claim_0).  Proof: "ZKMS", N, D, K, the K claims, two SC blocks."""
    ln, ld = ilog2(n), ilog2(d)
    k_sub = len(points)
    assert 1 <= k_sub <= 8 and all(len(pt) == ln + ld for pt in points)
    _stack_merge_header(ts, n, d, points, bind_statement)
    t_rows = [[int(v) for v in partial_eval(x, [1, n, d], 1, 2, pt[:ln])[0]] for pt in points]
    claims = [mle_eval(np.array(t, dtype=object), pt[ln:]) for t, pt in zip(t_rows, points)]
    ts.absorb_fr(b"c", claims)
    r = ts.challenges_vec(k_sub)
    e_tab, t_tab, lk = _stack_merge_tables(k_sub, r, [pt[ln:] for pt in points], t_rows, d)
    inner, vs = prove([e_tab, t_tab], [(1, [0, 1])], 2, ts)
    assert inner.claim0 == sum(rk * ck for rk, ck in zip(r, claims)) % R_MOD
    rho, v = vs[:lk], vs[lk:]
    b_rho = beta_table(rho)
    pn = np.zeros(n, dtype=object)
    for k, pt in enumerate(points):
        pn = (pn + int(b_rho[k]) * beta_table(pt[:ln])) % R_MOD
    tn, _ = partial_eval(x, [n, d], 1, 2, v)
    outer, vn = prove([pn, np.asarray(tn, dtype=object)], [(1, [0, 1])], 2, ts)
    assert outer.claim0 == inner.finals[1]
    out = ([struct.pack("<IIII", MS_MAGIC, n, d, k_sub)] + [to_le(c) for c in claims]
           + [inner.to_bytes(), outer.to_bytes()])
    return b"".join(out), dict(claims=claims, r=r, rho=rho, v=v, vn=vn, inner=inner, outer=outer)


def stack_merge_verify(buf, n, d, points, ts, bind_statement=True):
    """Returns (the K claims, the point (v_n, v), the remaining claim X~(v_n, v))."""
    magic, n_, d_, k_sub = struct.unpack_from("<IIII", buf, 0)
    assert magic == MS_MAGIC and n_ == n and d_ == d and k_sub == len(points)
    ln, ld = ilog2(n), ilog2(d)
    lk = max(0, (k_sub - 1).bit_length())
    _stack_merge_header(ts, n, d, points, bind_statement)
    claims = [from_le(buf[16 + 32 * k:48 + 32 * k]) for k in range(k_sub)]
    ts.absorb_fr(b"c", claims)
    r = ts.challenges_vec(k_sub)
    inner, off = SumcheckProof.from_bytes(buf, 16 + 32 * k_sub)
    outer, end = SumcheckProof.from_bytes(buf, off)
    assert end == len(buf)
    assert inner.n_finals == 2 and inner.degree == 2 and len(inner.rounds) == lk + ld
    assert outer.n_finals == 2 and outer.degree == 2 and len(outer.rounds) == ln
    expect0 = sum(rk * ck for rk, ck in zip(r, claims)) % R_MOD
    last, vs = verify_rounds(inner, ts, expected_claim0=expect0)
    rho, v = vs[:lk], vs[lk:]
    ef, tf = inner.finals
    assert ef * tf % R_MOD == last, "inner final claim mismatch"
    b_rho = beta_table(rho)
    assert ef == sum(int(b_rho[k]) * r[k] % R_MOD * beta_point(points[k][ln:], v)
                     for k in range(k_sub)) % R_MOD, "E~(rho, v) mismatch"
    last2, vn = verify_rounds(outer, ts, expected_claim0=tf)
    pf, xf = outer.finals
    assert pf * xf % R_MOD == last2, "outer final claim mismatch"
    assert pf == sum(int(b_rho[k]) * beta_point(points[k][:ln], vn) for k in range(k_sub)) % R_MOD, \
        "Pn~(v_n) mismatch"
    return claims, vn + v, xf


# --------------------------------------------------------------------------
# batched Hadamard product (Eq. exm-hadamard-batched)
# --------------------------------------------------------------------------
def hadamard_prove(x0, x1, ts):
    """Y = X0 (.) X1 over the whole stack: Y~(p) = sum_b beta~(p,b) X0(b) X1(b);
    p = (w, u) is drawn as one point over all variables."""
    d = ilog2(len(x0))
    assert len(x1) == len(x0)
    ts.absorb_u32(b"sumcheck_hadamard", [d])
    p = ts.challenges_vec(d)
    proof, vs = prove([beta_table(p), x0, x1], [(1, [0, 1, 2])], 3, ts)
    return proof.to_bytes(), proof, dict(p=p, v=vs)


def hadamard_verify(buf, d, ts):
    proof, _ = SumcheckProof.from_bytes(buf)
    assert proof.n_finals == 3 and proof.degree == 3 and len(proof.rounds) == d
    ts.absorb_u32(b"sumcheck_hadamard", [d])
    p = ts.challenges_vec(d)
    claim, vs = verify_rounds(proof, ts)
    fb, f0, f1 = proof.finals
    assert fb == beta_point(p, vs)
    assert fb * f0 % R_MOD * f1 % R_MOD == claim
    return proof, dict(p=p, v=vs)


# --------------------------------------------------------------------------
# zkReLU (Sec. 3.1, App. A)
# --------------------------------------------------------------------------
def recomposition_vectors(q, r_bits):
    """s_{Q+R} and s' padded with zeros to the next power of two J.

    s_B = (1, 2, ..., 2^{B-2}, -2^{B-1}) (Sec. 3.1).  s' picks out the rescaled
    value: aux[R:Q+R] . s_Q + aux[R-1], i.e. (0^{R-1}, 1, 1, 2, ..., 2^{Q-2},
    -2^{Q-1}) (App. A)."""
    b = q + r_bits
    j_pad = 1 << (b - 1).bit_length()
    s = [0] * j_pad
    sp = [0] * j_pad
    for j in range(b - 1):
        s[j] = 1 << j
    s[b - 1] = -(1 << (b - 1))
    sp[r_bits - 1] = 1
    for j in range(r_bits, b - 1):
        sp[j] = 1 << (j - r_bits)
    sp[b - 1] = -(1 << (q - 1))
    return s, sp, j_pad


def aux_bits(values, nbits, j_pad):
    """Two's-complement bits of (Q+R)-bit integers, zero-padded to j_pad columns
    (Eqs. aux-Z, aux-GA).  Raises ValueError on a value outside the range the
    completeness theorem assumes."""
    lim = 1 << (nbits - 1)
    out = np.zeros((len(values), j_pad), dtype=object)
    for i, x in enumerate(values):
        x = int(x)
        if not (-lim <= x < lim):
            raise ValueError(f"value {x} is not a {nbits}-bit signed integer")
        for j in range(nbits):
            out[i, j] = (x >> j) & 1
    return out


def zkrelu_witness(z, ga, q, r_bits):
    """aux and every tensor recomposed from it (Sec. 3.1): Z, Z', sign, A,
    G_A, G_A', G_Z as signed Python ints."""
    s, sp, j_pad = recomposition_vectors(q, r_bits)
    b = q + r_bits
    aux0 = aux_bits(z, b, j_pad)
    aux1 = aux_bits(ga, b, j_pad)
    sv = np.array(s, dtype=object)
    spv = np.array(sp, dtype=object)
    z_rec = aux0.dot(sv)
    ga_rec = aux1.dot(sv)
    zp = aux0.dot(spv)
    gap = aux1.dot(spv)
    sgn = aux0[:, b - 1].copy()
    a = (1 - sgn) * zp
    gz = (1 - sgn) * gap
    return dict(aux0=aux0, aux1=aux1, s=s, sp=sp, j_pad=j_pad, Z=z_rec, GA=ga_rec,
                Zp=zp, GAp=gap, sgn=sgn, A=a, GZ=gz)


def _merge_tables(m_table, wbar, rho, b, lj):
    """E = rho0 beta~((0,wbar),.) + rho1 beta~((1,wbar),.) + rho2 beta~((0,e_{B-1}),.)"""
    e_sign = index_bits(b - 1, lj)
    e = (rho[0] * beta_table([0] + list(wbar))
         + rho[1] * beta_table([1] + list(wbar))
         + rho[2] * beta_table([0] + e_sign)) % R_MOD
    return [np.asarray(m_table, dtype=object).reshape(-1), e]


def _points_digest(points):
    """SHA-256 of the four points u_Z, u_A, u_GA, u_GZ, 32 B little-endian per coordinate."""
    import hashlib
    return hashlib.sha256(b"".join(to_le(x) for pt in points for x in pt)).digest()


def _zkrelu_points(ts, li, lj, q, r_bits, has_ga, points, bind_points):
    """Header and the five points.  points=None: all five drawn (one draw).  Otherwise the
    four points of the input claims are the caller's (Sec. 3.2 and App. A: they are left by
    the sumchecks of the operations the four tensors take part in) and only u_bin is drawn;
    with bind_points they are bound through their digest (a call on its own), without it
    they must be functions of this transcript already (a call inside a larger proof)."""
    if points is None:
        ts.absorb_u32(b"zkrelu", [li, q, r_bits, 1 if has_ga else 0])
        pt = ts.challenges_vec(5 * li + lj)
        return pt[:li], pt[li:2 * li], pt[2 * li:3 * li], pt[3 * li:4 * li], pt[4 * li:], 0
    assert len(points) == 4 and all(len(pt) == li for pt in points)
    mode = 1 if bind_points else 2
    ts.absorb_u32(b"zkrelu_at", [li, q, r_bits, 1 if has_ga else 0, mode])
    if bind_points:
        ts.absorb(b"u", _points_digest(points))
    u_bin = ts.challenges_vec(li + lj)
    return [list(pt) for pt in points] + [u_bin, mode]


def zkrelu_prove(z, ga, q, r_bits, ts, points=None, bind_points=True):
    """Combined zkReLU sumcheck (App. A) followed by the merge of the three
    claims on aux into one.

    `ga=None` is the forward-only use: it stands for G_A = 0, for which the
    three backward equations hold trivially.
    Transcript order: header; u_Z, u_A, u_GA, u_GZ (log D each), u_bin
    (log D + log J); absorb the four input claims; r, r'; rounds; finals
    (aux~(0,v,wbar), aux~(1,v,wbar), aux~(0,v,Q+R-1)); rho0..2; merge rounds;
    merge finals (aux~(k*,v,w*), E~(k*,w*)).
    `points` = (u_Z, u_A, u_GA, u_GZ) replaces the draw of these four (see _zkrelu_points);
    word 5 of the proof header then holds the mode (1 bound by digest, 2 unbound)."""
    d_len = len(z)
    has_ga = ga is not None
    if ga is None:
        ga = [0] * d_len
    assert len(ga) == d_len
    wit = zkrelu_witness(z, ga, q, r_bits)
    j_pad = wit["j_pad"]
    li, lj = ilog2(d_len), ilog2(j_pad)
    b = q + r_bits
    u_z, u_a, u_ga, u_gz, u_bin, mode = _zkrelu_points(ts, li, lj, q, r_bits, has_ga, points, bind_points)
    c_in = [mle_eval(fr_array(wit["Z"]), u_z), mle_eval(fr_array(wit["A"]), u_a),
            mle_eval(fr_array(wit["GA"]), u_ga), mle_eval(fr_array(wit["GZ"]), u_gz)]
    ts.absorb_fr(b"c", c_in)
    r, rp = ts.challenges_vec(2)

    def over_i(col):      # a table of D values, constant in j
        return np.repeat(np.asarray(col, dtype=object), j_pad)

    def over_j(row):      # a table of J values, constant in i
        return np.tile(fr_array(row), d_len)

    tables = [
        over_i(beta_table(u_z)),            # 0  beta~(u_Z, i)
        over_i(beta_table(u_a)),            # 1  beta~(u_A, i)
        over_i(beta_table(u_ga)),           # 2  beta~(u_GA, i)
        over_i(beta_table(u_gz)),           # 3  beta~(u_GZ, i)
        beta_table(u_bin),                  # 4  beta~(u_bin, (i,j))
        fr_array(wit["aux0"]),              # 5  aux(0,i,j)
        fr_array(wit["aux1"]),              # 6  aux(1,i,j)
        over_i(fr_array(1 - wit["sgn"])),   # 7  1 - aux(0,i,Q+R-1)
        over_j(wit["s"]),                   # 8  s_{Q+R}(j)
        over_j(wit["sp"]),                  # 9  s'(j)
    ]
    r2 = r * r % R_MOD
    terms = [
        (r2, [0, 5, 8]),                    # forward in   (weight r^2)
        (r, [1, 7, 5, 9]),                  # forward out  (weight r)
        (1, [4, 5, 5]), (R_MOD - 1, [4, 5]),            # forward binarity (weight 1)
        (rp * r2 % R_MOD, [2, 6, 8]),       # backward in  (weight r' r^2)
        (rp * r % R_MOD, [3, 7, 6, 9]),     # backward out (weight r' r)
        (rp, [4, 6, 6]), (R_MOD - rp, [4, 6]),          # backward binarity (weight r')
    ]
    proof, vs = prove(tables, terms, 3, ts, absorb_claim=False,
                      report=lambda f: [f[5], f[6], 1 - f[7]])
    expect0 = (r2 * c_in[0] + r * c_in[1] + rp * r2 * c_in[2] + rp * r * c_in[3]) % R_MOD
    assert proof.claim0 == expect0, "combined claim is not the weighted sum of the input claims"
    v_i, wbar = vs[:li], vs[li:]

    # merge: M[k, j] = aux~(k, v, j)
    aux = np.concatenate([fr_array(wit["aux0"]), fr_array(wit["aux1"])])
    m_table, _ = partial_eval(aux, [2, d_len, j_pad], 1, 2, v_i)
    assert mle_eval(m_table[:j_pad], wbar) == proof.finals[0]
    assert mle_eval(m_table[j_pad:], wbar) == proof.finals[1]
    assert m_table[b - 1] == proof.finals[2]
    rho = ts.challenges_vec(3)
    merge, vm = prove(_merge_tables(m_table, wbar, rho, b, lj), [(1, [0, 1])], 2, ts,
                      absorb_claim=False)
    assert merge.claim0 == sum(x * y for x, y in zip(rho, proof.finals)) % R_MOD

    head = struct.pack("<IIIIIIII", ZKRL_MAGIC, li, q, r_bits, 1 if has_ga else 0, mode, 0, 0)
    buf = head + b"".join(to_le(c) for c in c_in) + proof.to_bytes() + merge.to_bytes()
    info = dict(u_z=u_z, u_a=u_a, u_ga=u_ga, u_gz=u_gz, u_bin=u_bin, c_in=c_in, r=r, rp=rp,
                v=vs, rho=rho, vm=vm, proof=proof, merge=merge, wit=wit)
    return buf, info


def zkrelu_verify(buf, ts, off=0, points=None):
    """Replay a zkReLU proof.  Checks every round, the final combined claim and
    the merge; the one remaining claim on aux, (k*, v, w*) -> value, is returned
    for the (out-of-scope) proof of evaluation.  `points`: the verifier's own copy of the
    four points when the proof was made at given points (header mode 1 or 2)."""
    magic, li, q, r_bits, has_ga, mode, _, _ = struct.unpack_from("<IIIIIIII", buf, off)
    assert magic == ZKRL_MAGIC
    assert (mode == 0) == (points is None), "proof mode and the verifier's points disagree"
    off += 32
    c_in = [from_le(buf[off + 32 * k: off + 32 * k + 32]) for k in range(4)]
    off += 128
    proof, off = SumcheckProof.from_bytes(buf, off)
    merge, off = SumcheckProof.from_bytes(buf, off)
    s, sp, j_pad = recomposition_vectors(q, r_bits)
    lj = ilog2(j_pad)
    b = q + r_bits
    assert proof.degree == 3 and len(proof.rounds) == li + lj and proof.n_finals == 3
    assert merge.degree == 2 and len(merge.rounds) == 1 + lj and merge.n_finals == 2
    u_z, u_a, u_ga, u_gz, u_bin, _ = _zkrelu_points(ts, li, lj, q, r_bits, has_ga, points, mode == 1)
    ts.absorb_fr(b"c", c_in)
    r, rp = ts.challenges_vec(2)
    r2 = r * r % R_MOD
    expect0 = (r2 * c_in[0] + r * c_in[1] + rp * r2 * c_in[2] + rp * r * c_in[3]) % R_MOD
    claim, vs = verify_rounds(proof, ts, absorb_claim=False, expected_claim0=expect0)
    v_i, wbar = vs[:li], vs[li:]
    a0, a1, sg = proof.finals
    s_w = mle_eval(fr_array(s), wbar)
    sp_w = mle_eval(fr_array(sp), wbar)
    b_bin = beta_point(u_bin, vs)
    rhs = (r2 * beta_point(u_z, v_i) % R_MOD * a0 % R_MOD * s_w
           + r * beta_point(u_a, v_i) % R_MOD * (1 - sg) % R_MOD * a0 % R_MOD * sp_w
           + b_bin * (a0 * a0 - a0)
           + rp * (r2 * beta_point(u_ga, v_i) % R_MOD * a1 % R_MOD * s_w
                   + r * beta_point(u_gz, v_i) % R_MOD * (1 - sg) % R_MOD * a1 % R_MOD * sp_w
                   + b_bin * (a1 * a1 - a1))) % R_MOD
    assert rhs == claim, "zkReLU final claim mismatch"
    rho = ts.challenges_vec(3)
    expect_m = (rho[0] * a0 + rho[1] * a1 + rho[2] * sg) % R_MOD
    claim_m, vm = verify_rounds(merge, ts, absorb_claim=False, expected_claim0=expect_m)
    m_f, e_f = merge.finals
    e_pub = (rho[0] * beta_point([0] + wbar, vm) + rho[1] * beta_point([1] + wbar, vm)
             + rho[2] * beta_point([0] + index_bits(b - 1, lj), vm)) % R_MOD
    assert e_f == e_pub, "E final is not the public combination of beta values"
    assert m_f * e_f % R_MOD == claim_m, "merge final claim mismatch"
    aux_claim = dict(point=[vm[0]] + v_i + vm[1:], value=m_f)
    return off, dict(c_in=c_in, points=dict(u_z=u_z, u_a=u_a, u_ga=u_ga, u_gz=u_gz),
                     aux_claim=aux_claim, v=vs, vm=vm)


# --------------------------------------------------------------------------
# aggregated proof of one window of training steps (Sec. 5, Example FCNN)
# --------------------------------------------------------------------------
def shift_layers(stack, n_layers):
    """Slot (t, l) <- slot (t, l+1); the last layer's slot of every step is zero.
    `stack` has the stack axis first."""
    stack = np.asarray(stack)
    out = np.zeros_like(stack)
    n = stack.shape[0]
    for k in range(n):
        if k % n_layers != n_layers - 1:
            out[k] = stack[k + 1]
    return out


def aggregate_prove(wit, ts):
    """One proof for a window of T' steps of an L-layer FCNN (Protocol zkdl,
    the sumcheck line only).  Families, in order: forward Z = A W; gradA
    G_A = G_Z^{(l+1)} W^{(l+1)T}; gradW G_W = A^T G_Z; zkReLU on the stacked Z, G_A.
    `wit`: dict with L, B, width, T, Q, R and integer stacks A [N,B,w], W [N,w,w],
    GZ [N,B,w], Zr [N,B,w], GA [N,B,w], N = T L, slot n = t L + (l-1)."""
    n_layers, bsz, width, steps = wit["L"], wit["B"], wit["width"], wit["T"]
    q, r_bits = wit["Q"], wit["R"]
    n = n_layers * steps
    a = np.asarray(wit["A"]).reshape(n, bsz, width)
    w = np.asarray(wit["W"]).reshape(n, width, width)
    gz = np.asarray(wit["GZ"]).reshape(n, bsz, width)
    ts.absorb_u32(b"aggregate", [n_layers, bsz, width, steps, q, r_bits])
    parts = [struct.pack("<IIIIIIII", ZKAG_MAGIC, n_layers, bsz, width, steps, q, r_bits, 0)]
    infos = {}
    # forward: X0 = A [N,B,w], X1 = W [N,w,w]
    buf, _, infos["fwd"] = matmul_prove(fr_array(a), [n, bsz, width], fr_array(w),
                                        [n, width, width], ts)
    parts.append(buf)
    # gradA: X0 = G_Z of the next layer [N,B,w], X1 = W of the next layer, transposed
    gz_next = shift_layers(gz, n_layers)
    wt_next = np.transpose(shift_layers(w, n_layers), (0, 2, 1))
    buf, _, infos["gradA"] = matmul_prove(fr_array(gz_next), [n, bsz, width], fr_array(wt_next),
                                          [n, width, width], ts)
    parts.append(buf)
    # gradW: X0 = A^T [N,w,B], X1 = G_Z [N,B,w]
    a_t = np.transpose(a, (0, 2, 1))
    buf, _, infos["gradW"] = matmul_prove(fr_array(a_t), [n, width, bsz], fr_array(gz),
                                          [n, bsz, width], ts)
    parts.append(buf)
    buf, infos["zkrelu"] = zkrelu_prove(np.asarray(wit["Zr"]).reshape(-1).tolist(),
                                        np.asarray(wit["GA"]).reshape(-1).tolist(), q, r_bits, ts)
    parts.append(buf)
    return b"".join(parts), infos


def aggregate_verify(buf, ts):
    magic, n_layers, bsz, width, steps, q, r_bits, _ = struct.unpack_from("<IIIIIIII", buf, 0)
    assert magic == ZKAG_MAGIC
    n = n_layers * steps
    ts.absorb_u32(b"aggregate", [n_layers, bsz, width, steps, q, r_bits])
    off = 32
    out = {}
    for name, (d1, d2, d3) in (("fwd", (bsz, width, width)), ("gradA", (bsz, width, width)),
                               ("gradW", (width, bsz, width))):
        proof, end = SumcheckProof.from_bytes(buf, off)
        out[name] = matmul_verify(buf[off:end], n, d1, d2, d3, ts)
        off = end
    off, out["zkrelu"] = zkrelu_verify(buf, ts, off)
    assert off == len(buf)
    return out


# --------------------------------------------------------------------------
# the same window with the matrix-product families in the optimized aggregated form (App. B,
# Protocol tensor-op-aggr-optimized): f_t for the stack rounds, then one matrix product's sumcheck
# --------------------------------------------------------------------------
ZKAF_MAGIC = 0x46414B5A   # bytes "ZKAF"


def aggregate_ft_prove(wit, ts):
    """aggregate_prove with matmul_ft_prove for forward, gradA and gradW: per family the log N stack
    rounds carry f_t (degree 2, no table for beta~(w, .)), then the single product's sumcheck
    (K = 2).  zkReLU as before.  Header label "aggregate_ft", proof "ZKAF" + the same eight words."""
    n_layers, bsz, width, steps = wit["L"], wit["B"], wit["width"], wit["T"]
    q, r_bits = wit["Q"], wit["R"]
    n = n_layers * steps
    a = np.asarray(wit["A"]).reshape(n, bsz, width)
    w = np.asarray(wit["W"]).reshape(n, width, width)
    gz = np.asarray(wit["GZ"]).reshape(n, bsz, width)
    ts.absorb_u32(b"aggregate_ft", [n_layers, bsz, width, steps, q, r_bits])
    parts = [struct.pack("<IIIIIIII", ZKAF_MAGIC, n_layers, bsz, width, steps, q, r_bits, 0)]
    infos = {}
    buf, infos["fwd"] = matmul_ft_prove(fr_array(a), [n, bsz, width], fr_array(w), [n, width, width], ts)
    parts.append(buf)
    gz_next = shift_layers(gz, n_layers)
    wt_next = np.transpose(shift_layers(w, n_layers), (0, 2, 1))
    buf, infos["gradA"] = matmul_ft_prove(fr_array(gz_next), [n, bsz, width], fr_array(wt_next),
                                          [n, width, width], ts)
    parts.append(buf)
    buf, infos["gradW"] = matmul_ft_prove(fr_array(np.transpose(a, (0, 2, 1))), [n, width, bsz], fr_array(gz),
                                          [n, bsz, width], ts)
    parts.append(buf)
    buf, infos["zkrelu"] = zkrelu_prove(np.asarray(wit["Zr"]).reshape(-1).tolist(),
                                        np.asarray(wit["GA"]).reshape(-1).tolist(), q, r_bits, ts)
    parts.append(buf)
    return b"".join(parts), infos


def _ft_block_end(buf, off):
    """End of the "ZKSF" block that starts at off."""
    magic, ln, _, _ = struct.unpack_from("<IIII", buf, off)
    assert magic == FT_MAGIC
    _, end = SumcheckProof.from_bytes(buf, off + 16 + 32 + 96 * ln)
    return end


def aggregate_ft_verify(buf, ts):
    """Per family (claim_0, finals (X0~, X1~), points), then zkReLU's result."""
    magic, n_layers, bsz, width, steps, q, r_bits, _ = struct.unpack_from("<IIIIIIII", buf, 0)
    assert magic == ZKAF_MAGIC
    n = n_layers * steps
    ts.absorb_u32(b"aggregate_ft", [n_layers, bsz, width, steps, q, r_bits])
    off = 32
    out = {}
    for name, (d1, d2, d3) in (("fwd", (bsz, width, width)), ("gradA", (bsz, width, width)),
                               ("gradW", (width, bsz, width))):
        end = _ft_block_end(buf, off)
        out[name] = matmul_ft_verify(buf[off:end], n, d1, d2, d3, ts)
        off = end
    off, out["zkrelu"] = zkrelu_verify(buf, ts, off)
    assert off == len(buf)
    return out


# --------------------------------------------------------------------------
# the same window with the claims linked (Sec. 3.2, Sec. 4 Eq. sc-reindex, Protocol zkdl)
# --------------------------------------------------------------------------
ZKAL_MAGIC = 0x4C414B5A   # "ZKAL"


def down_map(n, n_layers):
    """Sub-stack whose slot (t, l) is slot (t, l+1) of the stack; the last layer's slot is a
    zero tensor (shift_layers as an index map)."""
    return [j + 1 if j % n_layers != n_layers - 1 else -1 for j in range(n)]


def _linked_zkrelu_points(f, g, h, ln):
    """u_Z: point of the forward family's claim_0 (on the stacked Z); u_A: point of its final
    on A; u_GA: point of gradA's claim_0 (it is G_A); u_GZ: point of gradW's final on G_Z."""
    return [f["w"] + f["u0"] + f["u1"], f["v"][:ln] + f["u0"] + f["v"][ln:],
            g["w"] + g["u0"] + g["u1"], h["v"][:ln] + h["v"][ln:] + h["u1"]]


def _last_layer_factor(stack_point, n_layers):
    """beta~ of the layer coordinates (the low bits of the slot index) at the last layer."""
    ll = ilog2(n_layers)
    lay = stack_point[len(stack_point) - ll:]
    return beta_point(lay, index_bits(n_layers - 1, ll)) if ll else 1


def aggregate_linked_prove(wit, ts):
    """aggregate_prove's four families with the claims chained instead of left side by side:

    1. forward, gradA, gradW matmul sumchecks as in aggregate_prove.
    2. zkReLU at the points these have left (_linked_zkrelu_points), unbound mode.  Its input
       claims c_Z, c_A, c_GA, c_GZ then satisfy, for the verifier to check,
         c_GA = claim_0 of gradA,
         claim_0 of forward = c_Z + beta~(w_layer, L-1) Zlast~(w_step, u0, u1),
         gradW's final on G_Z = c_GZ + beta~(v_layer, L-1) GZlast~(v_step, v_i, u1),
       (the stacks given to zkReLU are zero in the last layer's slots, which have no ReLU;
       Zlast / GZlast [T', B, width] are the last layer's outputs and their gradients: the two
       claims on them are outputs of this proof, computed by the verifier).
    3. Re-indexing (Eq. sc-reindex) on the stack A with two sub-stacks at the stack point v_n
       of the forward family: A itself (claim: forward's final on A) and the shifted stack
       whose slot (t, l) is the input of layer l+1 = the output of this layer's ReLU (claim:
       c_A).  One claim on A is left.
    4. Re-indexing on G_Z and on W, one shifted sub-stack each: gradA's finals (they are
       evaluations of the stacks of the next layer's G_Z and W) become claims on the stacks.
    5. The two claims now standing on A (from 3 and gradW's final on A^T) are merged into one,
       and so are the two on W (forward's final and the one from 4): stack_merge_prove.
    One claim per stack is left (Protocol zkdl opens one evaluation per stack).
    Proof: "ZKAL" header, the three SC blocks, the zkReLU proof, the three ZKRI proofs, the
    two ZKMS proofs."""
    n_layers, bsz, width, steps = wit["L"], wit["B"], wit["width"], wit["T"]
    q, r_bits = wit["Q"], wit["R"]
    n = n_layers * steps
    ln = ilog2(n)
    a = np.asarray(wit["A"]).reshape(n, bsz, width)
    w = np.asarray(wit["W"]).reshape(n, width, width)
    gz = np.asarray(wit["GZ"]).reshape(n, bsz, width)
    ts.absorb_u32(b"aggregate_linked", [n_layers, bsz, width, steps, q, r_bits])
    parts = [struct.pack("<IIIIIIII", ZKAL_MAGIC, n_layers, bsz, width, steps, q, r_bits, 0)]
    infos = {}
    proofs = {}
    buf, proofs["fwd"], infos["fwd"] = matmul_prove(fr_array(a), [n, bsz, width], fr_array(w),
                                                    [n, width, width], ts)
    parts.append(buf)
    gz_next = shift_layers(gz, n_layers)
    wt_next = np.transpose(shift_layers(w, n_layers), (0, 2, 1))
    buf, proofs["gradA"], infos["gradA"] = matmul_prove(fr_array(gz_next), [n, bsz, width],
                                                        fr_array(wt_next), [n, width, width], ts)
    parts.append(buf)
    buf, proofs["gradW"], infos["gradW"] = matmul_prove(fr_array(np.transpose(a, (0, 2, 1))),
                                                        [n, width, bsz], fr_array(gz), [n, bsz, width], ts)
    parts.append(buf)
    f, g, h = infos["fwd"], infos["gradA"], infos["gradW"]
    pts = _linked_zkrelu_points(f, g, h, ln)
    buf, infos["zkrelu"] = zkrelu_prove(np.asarray(wit["Zr"]).reshape(-1).tolist(),
                                        np.asarray(wit["GA"]).reshape(-1).tolist(), q, r_bits, ts,
                                        points=pts, bind_points=False)
    parts.append(buf)
    c_in = infos["zkrelu"]["c_in"]
    assert c_in[2] == proofs["gradA"].claim0, "G_A of the witness is not the gradA family's product"
    down = down_map(n, n_layers)
    vn_f, vi_f = f["v"][:ln], f["v"][ln:]
    vn_a, vi_a = g["v"][:ln], g["v"][ln:]
    buf, infos["reindex_A"] = reindex_prove(fr_array(a.reshape(n, -1)), n, bsz * width,
                                            [list(range(n)), down], [vn_f, vn_f], f["u0"] + vi_f, ts,
                                            bind_statement=False)
    assert infos["reindex_A"]["claims"] == [proofs["fwd"].finals[1], c_in[1]], \
        "the next layer's input is not this layer's ReLU output"
    parts.append(buf)
    buf, infos["reindex_GZ"] = reindex_prove(fr_array(gz.reshape(n, -1)), n, bsz * width, [down], [vn_a],
                                             g["u0"] + vi_a, ts, bind_statement=False)
    assert infos["reindex_GZ"]["claims"] == [proofs["gradA"].finals[1]]
    parts.append(buf)
    buf, infos["reindex_W"] = reindex_prove(fr_array(w.reshape(n, -1)), n, width * width, [down], [vn_a],
                                            g["u1"] + vi_a, ts, bind_statement=False)
    assert infos["reindex_W"]["claims"] == [proofs["gradA"].finals[2]]
    parts.append(buf)
    vn_w, vi_w = h["v"][:ln], h["v"][ln:]
    buf, infos["merge_A"] = stack_merge_prove(fr_array(a.reshape(-1)), n, bsz * width,
                                              [infos["reindex_A"]["v"] + f["u0"] + vi_f, vn_w + vi_w + h["u0"]],
                                              ts, bind_statement=False)
    assert infos["merge_A"]["claims"] == [infos["reindex_A"]["inner"].finals[1], proofs["gradW"].finals[1]]
    parts.append(buf)
    buf, infos["merge_W"] = stack_merge_prove(fr_array(w.reshape(-1)), n, width * width,
                                              [vn_f + vi_f + f["u1"], infos["reindex_W"]["v"] + g["u1"] + vi_a],
                                              ts, bind_statement=False)
    assert infos["merge_W"]["claims"] == [proofs["fwd"].finals[2], infos["reindex_W"]["inner"].finals[1]]
    parts.append(buf)
    return b"".join(parts), infos


def aggregate_linked_verify(buf, ts):
    """Replays the linked proof and checks every link.  Returns the claims that are left, each
    as (point, value): one on A, one on W, one on G_Z (from the re-indexing; gradW's final is
    consumed by zkReLU), the last layer's Z and G_Z, G_W, aux."""
    magic, n_layers, bsz, width, steps, q, r_bits, _ = struct.unpack_from("<IIIIIIII", buf, 0)
    assert magic == ZKAL_MAGIC
    n = n_layers * steps
    ln, lt = ilog2(n), ilog2(steps)
    ts.absorb_u32(b"aggregate_linked", [n_layers, bsz, width, steps, q, r_bits])
    off = 32
    pr, inf = {}, {}
    for name, (d1, d2, d3) in (("fwd", (bsz, width, width)), ("gradA", (bsz, width, width)),
                               ("gradW", (width, bsz, width))):
        _, end = SumcheckProof.from_bytes(buf, off)
        pr[name], inf[name] = matmul_verify(buf[off:end], n, d1, d2, d3, ts)
        off = end
    f, g, h = inf["fwd"], inf["gradA"], inf["gradW"]
    pts = _linked_zkrelu_points(f, g, h, ln)
    assert struct.unpack_from("<I", buf, off + 20)[0] == 2, "zkReLU must take its points from this transcript"
    off, zk = zkrelu_verify(buf, ts, off, points=pts)
    c_z, c_a, c_ga, c_gz = zk["c_in"]
    assert c_ga == pr["gradA"].claim0, "G_A link"
    vn_f, vi_f = f["v"][:ln], f["v"][ln:]
    vn_a, vi_a = g["v"][:ln], g["v"][ln:]
    vn_w, vi_w = h["v"][:ln], h["v"][ln:]

    def last_layer_claim(total, part, stack_point):
        fac = _last_layer_factor(stack_point, n_layers)
        if fac == 0:                      # the point lies where the last layer has weight 0
            assert total == part
            return None
        return (total - part) * pow(fac, R_MOD - 2, R_MOD) % R_MOD
    z_last = last_layer_claim(pr["fwd"].claim0, c_z, f["w"])
    gz_last = last_layer_claim(pr["gradW"].finals[2], c_gz, vn_w)
    down = down_map(n, n_layers)

    def reindex_at(off, d, maps, points, u):
        k_sub = len(maps)
        _, end = SumcheckProof.from_bytes(buf, off + 16 + 32 * k_sub)
        claims, vs, left = reindex_verify(buf[off:end], n, d, maps, points, u, ts, bind_statement=False)
        return end, claims, vs, left
    off, cl, v_ra, a_left = reindex_at(off, bsz * width, [list(range(n)), down], [vn_f, vn_f], f["u0"] + vi_f)
    assert cl == [pr["fwd"].finals[1], c_a], "A link"
    off, cl, v_rg, gz_left = reindex_at(off, bsz * width, [down], [vn_a], g["u0"] + vi_a)
    assert cl == [pr["gradA"].finals[1]], "G_Z link"
    off, cl, v_rw, w_left = reindex_at(off, width * width, [down], [vn_a], g["u1"] + vi_a)
    assert cl == [pr["gradA"].finals[2]], "W link"

    def merge_at(off, d, points):
        _, mid = SumcheckProof.from_bytes(buf, off + 16 + 32 * len(points))
        _, end = SumcheckProof.from_bytes(buf, mid)
        claims, vs, left = stack_merge_verify(buf[off:end], n, d, points, ts, bind_statement=False)
        return end, claims, vs, left
    off, cl, v_ma, a_one = merge_at(off, bsz * width, [v_ra + f["u0"] + vi_f, vn_w + vi_w + h["u0"]])
    assert cl == [a_left, pr["gradW"].finals[1]], "claims on A"
    off, cl, v_mw, w_one = merge_at(off, width * width, [vn_f + vi_f + f["u1"], v_rw + g["u1"] + vi_a])
    assert cl == [pr["fwd"].finals[2], w_left], "claims on W"
    assert off == len(buf)
    return dict(
        A=[(v_ma, a_one)],
        W=[(v_mw, w_one)],
        GZ=[(v_rg + g["u0"] + vi_a, gz_left)],
        Zlast=(f["w"][:lt] + f["u0"] + f["u1"], z_last),
        GZlast=(vn_w[:lt] + vi_w + h["u1"], gz_last),
        GW=(h["w"] + h["u0"] + h["u1"], pr["gradW"].claim0),
        aux=(zk["aux_claim"]["point"], zk["aux_claim"]["value"]))


# --------------------------------------------------------------------------
# proof of the parameter update (Sec. 5, Example FCNN, last item: "parameter updates, based on
# the selected optimizer", a family of its own in Protocol zkdl).  The paper fixes no optimizer;
# this build's reading: plain SGD on fixed-point weights with a power-of-two learning rate,
#   W_next = W - U,  U = sround(G_W / 2^R)   (rounded to nearest, halves away from zero),
# and since U = ReLU(rescale(G_W)) - ReLU(rescale(-G_W)) with zkReLU's own rescaling (round
# half up), the rounding is proved by zkReLU's forward half on the stack Zu = [G_W; -G_W]:
#   1. p drawn over the D entries; the prover claims a0 = Au~(0, p), a1 = Au~(1, p) for
#      Au = ReLU(rescale(Zu)) = [U+; U-]; U~(p) = a0 - a1 is what the verifier compares with
#      W~(p) - W_next~(p) (two openings of commitments, or claims of other sumchecks);
#   2. a multilinear extension is linear in each coordinate (Eq. multilinear-extension), so the two
#      claims lie on a line: with rho drawn after they are absorbed, Au~(rho, p) = (1 - rho) a0 + rho a1
#      is ONE claim that stands for both (wrong a0 or a1 give a different line, which agrees with the
#      true one at one rho at most);
#   3. u_Z drawn over the 1 + log D variables of Zu; zkReLU at the given points u_A = (rho, p)
#      and u_Z proves that Au and Zu are what their bit decompositions say; its claim on Zu is
#      Zu~(u_Z) = (1 - 2 u_Z[0]) G_W~(u_Z[1:]), a claim on the (committed) gradients.
# --------------------------------------------------------------------------
ZKUP_MAGIC = 0x50554B5A   # "ZKUP"


def sround(g, r_bits):
    """g / 2^r_bits rounded to the nearest integer, halves away from zero."""
    g = int(g)
    mag = (abs(g) + (1 << (r_bits - 1))) >> r_bits
    return mag if g >= 0 else -mag


def update_prove(gw, q, r_bits, ts):
    """gw: D = 2^k signed integers below 2^(q + r_bits - 1) in magnitude (q + r_bits <= 63).
    Transcript: header "update" (log D, Q, R); draw p; "c" the two claims a0, a1; one draw of
    rho and u_Z (2 + log D elements); zkReLU at given points (mode 2).
    Proof: "ZKUP", log D, Q, R, 0, 0, 0, 0; a0, a1; the "ZKRL" block."""
    d = len(gw)
    ld = ilog2(d)
    assert q + r_bits <= 63
    ts.absorb_u32(b"update", [ld, q, r_bits])
    p = ts.challenges_vec(ld)
    zu = [int(g) for g in gw] + [-int(g) for g in gw]
    wit = zkrelu_witness(zu, [0] * (2 * d), q, r_bits)
    au = [int(a) for a in wit["A"]]
    a0, a1 = mle_eval(fr_array(au[:d]), p), mle_eval(fr_array(au[d:]), p)
    ts.absorb_fr(b"c", [a0, a1])
    drawn = ts.challenges_vec(2 + ld)
    rho, u_z = drawn[0], drawn[1:]
    u_a = [rho] + p
    zk_buf, zk = zkrelu_prove(zu, None, q, r_bits, ts, points=(u_z, u_a, u_z, u_z), bind_points=False)
    assert zk["c_in"][1] == ((1 - rho) * a0 + rho * a1) % R_MOD, "zkReLU does not start from the claim on the line"
    head = struct.pack("<IIIIIIII", ZKUP_MAGIC, ld, q, r_bits, 0, 0, 0, 0)
    return head + to_le(a0) + to_le(a1) + zk_buf, dict(p=p, a=[a0, a1], rho=rho, u_a=u_a, u_z=u_z, zkrelu=zk)


def update_verify(buf, ld, q, r_bits, ts):
    """Replays the proof.  Returns the claims it leaves: u = (p, U~(p)), gw = (u_Z[1:], G_W~(u_Z[1:])),
    aux = zkReLU's one claim on the bit tensor of Zu."""
    magic, ld_, q_, r_, z0, z1, z2, z3 = struct.unpack_from("<IIIIIIII", buf, 0)
    assert magic == ZKUP_MAGIC and (ld_, q_, r_) == (ld, q, r_bits) and z0 == z1 == z2 == z3 == 0
    ts.absorb_u32(b"update", [ld, q, r_bits])
    p = ts.challenges_vec(ld)
    a0, a1 = from_le(buf[32:64]), from_le(buf[64:96])
    ts.absorb_fr(b"c", [a0, a1])
    drawn = ts.challenges_vec(2 + ld)
    rho, u_z = drawn[0], drawn[1:]
    end, zk = zkrelu_verify(buf, ts, off=96, points=(u_z, [rho] + p, u_z, u_z))
    assert end == len(buf), "trailing bytes"
    li, q2, r2, has_ga = struct.unpack_from("<IIII", buf, 96 + 4)
    assert (li, q2, r2, has_ga) == (1 + ld, q, r_bits, 0)
    assert zk["c_in"][1] == ((1 - rho) * a0 + rho * a1) % R_MOD, "zkReLU's claim on Au is not the one on the line"
    assert zk["c_in"][2] == 0 and zk["c_in"][3] == 0
    den = (1 - 2 * u_z[0]) % R_MOD
    assert den != 0
    gw_val = zk["c_in"][0] * pow(den, -1, R_MOD) % R_MOD
    return dict(u=(p, (a0 - a1) % R_MOD), gw=(u_z[1:], gw_val), aux=zk["aux_claim"])
