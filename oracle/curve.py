"""Pedersen commitments on BLS12-381 G1 and the row-wise (Hyrax-style) commitment of a tensor
with its proof of evaluation (Sec. 2.3; Sec. 1.1; Protocol zkdl, the commit and proof-of-evaluation lines).

Plain Python integers: the base field F_q by `%`, points in affine coordinates with the chord and tangent
formulas, scalar multiplication by double-and-add, a commitment as the sum it is defined to be.
Test infrastructure; not used by the product and sharing nothing with it.

What the paper fixes: Commit(S; rho) = h^rho prod_i g_i^{S_i} in a group of prime order r with independent
generators (Sec. 2.3), written additively here as rho H + sum_i S_i G_i; its homomorphism; commitment sizes
that grow like the square root of the tensor (Sec. 1.1: Hyrax), i.e. one commitment per row of the tensor
laid out as a matrix.  Readings where it is silent:
 * the group is G1 of BLS12-381, y^2 = x^3 + 4 over F_q (Sec. 6 names the curve), the subgroup of order r;
 * generators: for index i and counter ctr = 0, 1, .. the candidate x = int_be(SHA256(tag || u32be(i) ||
   u32be(ctr) || 0) || SHA256(.. || 1)) mod q; the first ctr for which x^3 + 4 is a square gives the point
   (x, y) with the smaller of the two roots y, multiplied by the cofactor to land in the subgroup (a
   candidate that becomes the identity is skipped).  tag = b"zkdl-mi355x/g1/" + label; the blinding
   generator H is index 0xFFFFFFFF of the same label.  Nobody knows a discrete-log relation between them;
 * the verifier of an opening checks that every row commitment it is given lies in that subgroup, r C = O: Sec. 2.3
   states the scheme and its homomorphism for a group of prime order, and the curve's group is larger than the
   subgroup (cofactor 0x396C8C00..AAAB), so a point on the curve is not yet an element of the group;
 * layout: a tensor of 2^m entries is a matrix of R = 2^ceil(m/2) rows and C = 2^floor(m/2) columns, row
   index = the leading variables; row j is committed with the C generators and its own blinding rho_j;
 * proof of evaluation at (v_row, v_col): the prover sends T = sum_j beta~(v_row, j) S[j, :] and
   rho* = sum_j beta~(v_row, j) rho_j; the verifier forms C* = sum_j beta~(v_row, j) C_j from the row
   commitments (the homomorphism of Sec. 2.3), checks Commit(T; rho*) = C* and <T, beta~(v_col, .)> = y.
   This is the reduction to one committed row; the logarithmic-size argument that Hyrax puts on top of it is
   not described in the paper and is not reproduced (the opening here has C field elements).
"""
import hashlib
import struct

from .field import R_MOD
from .mle import beta_table, ilog2

Q_MOD = 0x1A0111EA397FE69A4B1BA7B6434BACD764774B84F38512BF6730D2A0F6B0F6241EABFFFEB153FFFFB9FEFFFFFFFFAAAB
CURVE_B = 4
COFACTOR = 0x396C8C005555E1568C00AAAB0000AAAB
INF = None                      # the identity
H_INDEX = 0xFFFFFFFF


def on_curve(p):
    if p is INF:
        return True
    x, y = p
    return (y * y - x * x * x - CURVE_B) % Q_MOD == 0


def neg(p):
    if p is INF:
        return INF
    return (p[0], (-p[1]) % Q_MOD)


def add(p1, p2):
    """Chord-and-tangent addition in affine coordinates."""
    if p1 is INF:
        return p2
    if p2 is INF:
        return p1
    x1, y1 = p1
    x2, y2 = p2
    if x1 == x2:
        if (y1 + y2) % Q_MOD == 0:
            return INF
        lam = 3 * x1 * x1 * pow(2 * y1, -1, Q_MOD) % Q_MOD
    else:
        lam = (y2 - y1) * pow(x2 - x1, -1, Q_MOD) % Q_MOD
    x3 = (lam * lam - x1 - x2) % Q_MOD
    return (x3, (lam * (x1 - x3) - y1) % Q_MOD)


def mul(k, p):
    """k p by double-and-add, k any non-negative integer."""
    acc = INF
    while k:
        if k & 1:
            acc = add(acc, p)
        p = add(p, p)
        k >>= 1
    return acc


def in_subgroup(p):
    """Membership in the group of prime order r that Sec. 2.3 works in: on the curve and r p = O."""
    return on_curve(p) and mul(R_MOD, p) is INF


def generator(label, index):
    """The index-th generator of `label` (see the module docstring)."""
    tag = b"zkdl-mi355x/g1/" + bytes(label)
    ctr = 0
    while True:
        seed = tag + struct.pack(">II", index, ctr)
        x = int.from_bytes(hashlib.sha256(seed + b"\x00").digest() + hashlib.sha256(seed + b"\x01").digest(), "big") % Q_MOD
        rhs = (x * x * x + CURVE_B) % Q_MOD
        y = pow(rhs, (Q_MOD + 1) // 4, Q_MOD)          # q = 3 mod 4
        if y * y % Q_MOD == rhs:
            y = min(y, Q_MOD - y)
            p = mul(COFACTOR, (x, y))
            if p is not INF:
                return p
        ctr += 1


def generators(label, count):
    return [generator(label, i) for i in range(count)], generator(label, H_INDEX)


def commit(values, rho, gens, h):
    """rho H + sum_i S_i G_i  (Sec. 2.3); S_i signed integers or field elements, read mod r."""
    assert len(values) <= len(gens)
    acc = mul(int(rho) % R_MOD, h)
    for s, g in zip(values, gens):
        acc = add(acc, mul(int(s) % R_MOD, g))
    return acc


def matrix_shape(numel):
    m = ilog2(numel)
    return 1 << (m - m // 2), 1 << (m // 2)


def commit_rows(values, rhos, gens, h):
    """One commitment per row of the tensor laid out as R x C."""
    rows, cols = matrix_shape(len(values))
    assert len(rhos) == rows and len(gens) >= cols
    return [commit(values[j * cols:(j + 1) * cols], rhos[j], gens, h) for j in range(rows)]


def open_rows(values, rhos, point):
    """The prover's side of the proof of evaluation at `point` (row coordinates first):
    (T, rho*, y) with T = sum_j beta~(v_row, j) S[j, :], y = <T, beta~(v_col, .)> = S~(point)."""
    rows, cols = matrix_shape(len(values))
    lr = ilog2(rows)
    assert len(point) == lr + ilog2(cols)
    b_row, b_col = beta_table(point[:lr]), beta_table(point[lr:])
    t = [sum(int(b_row[j]) * (int(values[j * cols + c]) % R_MOD) for j in range(rows)) % R_MOD for c in range(cols)]
    rho_star = sum(int(b_row[j]) * (int(rhos[j]) % R_MOD) for j in range(rows)) % R_MOD
    y = sum(int(b_col[c]) * t[c] for c in range(cols)) % R_MOD
    return t, rho_star, y


def verify_opening(commitments, point, t, rho_star, y, gens, h):
    """C* = sum_j beta~(v_row, j) C_j; Commit(T; rho*) = C* and <T, beta~(v_col, .)> = y."""
    rows = len(commitments)
    cols = len(t)
    lr = ilog2(rows)
    assert len(point) == lr + ilog2(cols)
    b_row, b_col = beta_table(point[:lr]), beta_table(point[lr:])
    assert all(in_subgroup(c) for c in commitments), "a commitment is not an element of the group of order r"
    c_star = INF
    for j in range(rows):
        c_star = add(c_star, mul(int(b_row[j]), commitments[j]))
    assert commit(t, rho_star, gens, h) == c_star, "the opened row does not match the combined commitment"
    assert sum(int(b_col[c]) * int(t[c]) for c in range(cols)) % R_MOD == y % R_MOD, "wrong evaluation"
    return True


def point_to_bytes(p):
    """x || y, 48 bytes little-endian each; the identity as 96 zero bytes ((0, 0) is not on the curve)."""
    if p is INF:
        return bytes(96)
    return p[0].to_bytes(48, "little") + p[1].to_bytes(48, "little")


def point_from_bytes(b):
    b = bytes(b)
    assert len(b) == 96
    if b == bytes(96):
        return INF
    p = (int.from_bytes(b[:48], "little"), int.from_bytes(b[48:], "little"))
    assert p[0] < Q_MOD and p[1] < Q_MOD and on_curve(p)
    return p
