"""Pins for the commitment oracle (oracle/curve.py): what the curve, Sec. 2.3 and the mathematics fix."""
import numpy as np
import pytest

from oracle import curve as EC
from oracle.field import R_MOD
from oracle.mle import mle_eval

# the generator of G1 that the curve's specification publishes (draft-irtf-cfrg-pairing-friendly-curves, BLS12-381)
G1_X = 0x17F1D3A73197D7942695638C4FA9AC0FC3688C4F9774B905A14E3A3F171BAC586C55E83FF97A1AEFFB3AF00ADB22C6BB
G1_Y = 0x08B3F481E3AAA0F1A09E30ED741D8AE4FCF5E095D5D00AF600DB18CB2C04B3EDD03CC744A2888AE40CAA232946C5E7E1
G1 = (G1_X, G1_Y)


def test_curve_parameters():
    assert EC.Q_MOD % 4 == 3                                     # the square root used is a^((q+1)/4)
    assert EC.on_curve(G1)                                       # y^2 = x^3 + 4
    assert EC.mul(R_MOD, G1) is EC.INF                           # the subgroup has order r
    assert EC.mul(R_MOD - 1, G1) == EC.neg(G1)
    # the cofactor: the curve has h r points (Hasse: |q + 1 - h r| <= 2 sqrt(q))
    t = EC.Q_MOD + 1 - EC.COFACTOR * R_MOD
    assert t * t <= 4 * EC.Q_MOD


def test_group_law():
    p, q2, s = EC.mul(5, G1), EC.mul(11, G1), EC.mul(123456789, G1)
    assert EC.add(p, q2) == EC.mul(16, G1) == EC.add(q2, p)
    assert EC.add(EC.add(p, q2), s) == EC.add(p, EC.add(q2, s))
    assert EC.add(p, EC.neg(p)) is EC.INF and EC.add(p, EC.INF) == p and EC.add(EC.INF, p) == p
    assert EC.add(p, p) == EC.mul(2, p) and EC.on_curve(EC.add(p, p))
    assert EC.mul(7 * 13, G1) == EC.mul(7, EC.mul(13, G1))
    assert EC.mul(0, G1) is EC.INF


def test_generators_are_subgroup_points_and_distinct():
    gens, h = EC.generators(b"test", 6)
    pts = gens + [h]
    assert len({EC.point_to_bytes(p) for p in pts}) == 7
    for p in pts:
        assert p is not EC.INF and EC.on_curve(p) and EC.mul(R_MOD, p) is EC.INF
    assert EC.generators(b"test", 3)[0] == gens[:3]              # a function of (label, index) alone
    assert EC.generator(b"other", 0) != gens[0]
    for p in pts:
        assert EC.point_from_bytes(EC.point_to_bytes(p)) == p
    assert EC.point_from_bytes(bytes(96)) is EC.INF


def test_commitment_is_the_defining_sum_and_homomorphic():
    gens, h = EC.generators(b"test", 4)
    s1, s2 = [3, -7, 0, 2 ** 31 - 1], [-2 ** 31, 5, 1, -1]
    r1, r2 = 0x1234567890ABCDEF1234567890ABCDEF, R_MOD - 5
    c1, c2 = EC.commit(s1, r1, gens, h), EC.commit(s2, r2, gens, h)
    # brute force: repeated addition for the small entries, negation for negative ones
    by_hand = EC.mul(r1, h)
    for _ in range(3):
        by_hand = EC.add(by_hand, gens[0])
    for _ in range(7):
        by_hand = EC.add(by_hand, EC.neg(gens[1]))
    by_hand = EC.add(by_hand, EC.mul(2 ** 31 - 1, gens[3]))
    assert c1 == by_hand
    # Sec. 2.3: com(S1) com(S2) commits to S1 + S2 with randomness r1 + r2
    assert EC.add(c1, c2) == EC.commit([a + b for a, b in zip(s1, s2)], r1 + r2, gens, h)
    # a negative entry is the field element r - |x|
    assert EC.commit([-7], 0, gens, h) == EC.commit([R_MOD - 7], 0, gens, h)
    assert EC.commit([0, 0], 0, gens, h) is EC.INF


@pytest.mark.parametrize("numel", [1, 2, 8, 32])
def test_row_commitments_open_to_the_multilinear_extension(numel):
    rng = np.random.default_rng(numel)
    vals = [int(v) for v in rng.integers(-2 ** 31, 2 ** 31, numel)]
    rows, cols = EC.matrix_shape(numel)
    assert rows * cols == numel and rows in (cols, 2 * cols)
    gens, h = EC.generators(b"test", cols)
    rhos = [int(v) for v in rng.integers(1, 2 ** 62, rows)]
    coms = EC.commit_rows(vals, rhos, gens, h)
    m = numel.bit_length() - 1
    point = [int(v) for v in rng.integers(1, 2 ** 62, m)]
    t, rho_star, y = EC.open_rows(vals, rhos, point)
    assert y == mle_eval(np.array([v % R_MOD for v in vals], dtype=object), point)
    assert EC.verify_opening(coms, point, t, rho_star, y, gens, h)
    if numel > 1:
        with pytest.raises(AssertionError):
            EC.verify_opening(coms, point, t, rho_star, (y + 1) % R_MOD, gens, h)
        bad = list(t)
        bad[0] = (bad[0] + 1) % R_MOD
        with pytest.raises(AssertionError):
            EC.verify_opening(coms, point, bad, rho_star, y, gens, h)
        with pytest.raises(AssertionError):
            EC.verify_opening(coms, point, t, (rho_star + 1) % R_MOD, y, gens, h)
        other = list(vals)
        other[-1] += 1
        with pytest.raises(AssertionError):
            EC.verify_opening(EC.commit_rows(other, rhos, gens, h), point, t, rho_star, y, gens, h)


def _point_outside_the_subgroup(seed):
    """A point of the curve found by trying x = seed, seed + 1, ..: the curve has h r points, so one found this way
    lies in the subgroup of order r with probability 1 / h."""
    x = seed
    while True:
        rhs = (x * x * x + EC.CURVE_B) % EC.Q_MOD
        y = pow(rhs, (EC.Q_MOD + 1) // 4, EC.Q_MOD)
        if y * y % EC.Q_MOD == rhs and not EC.mul(R_MOD, (x, y)) is EC.INF:
            return (x, y)
        x += 1


def test_subgroup_membership_is_more_than_being_on_the_curve():
    """Sec. 2.3 works in a group of prime order: a verifier must not take a point of the curve for an element of it."""
    assert EC.in_subgroup(G1) and EC.in_subgroup(EC.INF) and EC.in_subgroup(EC.mul(987654321, G1))
    three_torsion = (0, 2)                                       # 2^2 = 0^3 + 4; a point with x = 0 has order 3
    assert EC.on_curve(three_torsion) and EC.mul(3, three_torsion) is EC.INF
    assert not EC.in_subgroup(three_torsion)
    p = _point_outside_the_subgroup(5)
    assert EC.on_curve(p) and not EC.in_subgroup(p)
    assert EC.in_subgroup(EC.mul(EC.COFACTOR, p))                # the cofactor takes it into the subgroup
    assert not EC.in_subgroup(EC.add(G1, three_torsion))         # a subgroup point moved by a torsion point
    assert not EC.in_subgroup((G1_X, G1_Y + 1))                  # not on the curve at all


def test_opening_is_refused_when_a_commitment_leaves_the_subgroup():
    rng = np.random.default_rng(5)
    vals = [int(v) for v in rng.integers(-100, 100, 16)]
    gens, h = EC.generators(b"sub", 4)
    rhos = [int(v) for v in rng.integers(1, 2 ** 60, 4)]
    coms = EC.commit_rows(vals, rhos, gens, h)
    point = [int(v) for v in rng.integers(1, 2 ** 60, 4)]
    t, rho_star, y = EC.open_rows(vals, rhos, point)
    assert EC.verify_opening(coms, point, t, rho_star, y, gens, h)
    # the same commitment moved by a point of order 3: still on the curve, no longer in the group
    moved = [EC.add(coms[0], (0, 2))] + coms[1:]
    with pytest.raises(AssertionError, match="group of order r"):
        EC.verify_opening(moved, point, t, rho_star, y, gens, h)
