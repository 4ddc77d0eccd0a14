"""Pins for the oracle's field, transcript and multilinear-extension code."""
import hashlib
import itertools
import struct

import numpy as np
import pytest

from oracle.field import R_MOD, fr, inv, to_le, from_le, fr_array
from oracle.mle import beta_eval, beta_table, mle_eval, partial_eval, fold
from oracle.transcript import Transcript

rng = np.random.default_rng(11)


def rand_fr(n):
    return [int.from_bytes(rng.bytes(40), "little") % R_MOD for _ in range(n)]


def test_modulus_is_the_bls12_381_scalar_field():
    # r = x^4 - x^2 + 1 for the BLS12-381 curve parameter x = -0xd201000000010000
    x = -0xD201000000010000
    assert R_MOD == x ** 4 - x ** 2 + 1
    assert R_MOD.bit_length() == 255
    assert R_MOD % (1 << 32) == 1          # 2^32-th roots of unity exist
    for a in (2, 3, 5, 7, 11):              # Fermat witnesses
        assert pow(a, R_MOD - 1, R_MOD) == 1


def test_field_basics():
    assert fr(-1) == R_MOD - 1
    assert fr(-1) * fr(-1) % R_MOD == 1
    for a in rand_fr(5):
        assert a * inv(a) % R_MOD == 1
        assert from_le(to_le(a)) == a
    assert to_le(1) == b"\x01" + b"\x00" * 31
    with pytest.raises(AssertionError):
        from_le(to_le(R_MOD - 1)[:-1] + b"\xff")


def test_transcript_format():
    # SHA-256 itself: NIST "abc" vector through the same library call
    assert hashlib.sha256(b"abc").hexdigest() == \
        "ba7816bf8f01cfea414140de5dae2223b00361a396177a9cb410ff61f20015ad"
    t = Transcript(9)
    s0 = hashlib.sha256(b"zkdl-mi355x/v1" + struct.pack("<Q", 9)).digest()
    assert t.digest() == s0
    t.absorb(b"g", b"\x01\x02")
    s1 = hashlib.sha256(s0 + b"\x01g" + struct.pack("<Q", 2) + b"\x01\x02").digest()
    assert t.digest() == s1
    c = t.challenge()
    z4 = struct.pack("<I", 0)
    wide = hashlib.sha256(s1 + b"\x00" + z4).digest() + hashlib.sha256(s1 + b"\x01" + z4).digest()
    assert c == int.from_bytes(wide, "little") % R_MOD
    s2 = hashlib.sha256(s1 + b"\x02").digest()
    assert t.digest() == s2
    assert t.challenge() != c
    # a vector draw: index-derived elements, one state update
    t2 = Transcript(9)
    t2.absorb(b"g", b"\x01\x02")
    vec = t2.challenges_vec(3)
    assert vec[0] == c and len(set(vec)) == 3 and t2.digest() == s2
    i2 = struct.pack("<I", 2)
    wide = hashlib.sha256(s1 + b"\x00" + i2).digest() + hashlib.sha256(s1 + b"\x01" + i2).digest()
    assert vec[2] == int.from_bytes(wide, "little") % R_MOD
    assert t2.challenges_vec(0) == [] and t2.digest() == s2


def test_beta_table_boolean_points_are_one_hot_msb_first():
    for m in (1, 2, 3, 5):
        for b in range(1 << m):
            u = [(b >> (m - 1 - k)) & 1 for k in range(m)]     # coordinate 0 = MSB
            tab = beta_table(u)
            assert [int(x) for x in tab] == [1 if k == b else 0 for k in range(1 << m)]
    assert [int(x) for x in beta_table([1, 0])] == [0, 0, 1, 0]


def test_beta_table_matches_product_formula_and_sums_to_one():
    for m in (1, 4, 7):
        u = rand_fr(m)
        tab = beta_table(u)
        assert int(np.sum(tab) % R_MOD) == 1
        for b in range(1 << m):
            assert tab[b] == beta_eval(u, b)
    # symmetric in its two arguments on Boolean inputs, multilinear in u
    u = rand_fr(3)
    u2 = list(u)
    u2[1] = (u[1] + 1) % R_MOD
    u3 = list(u)
    u3[1] = (u[1] + 2) % R_MOD
    for b in range(8):
        assert (beta_eval(u, b) + beta_eval(u3, b) - 2 * beta_eval(u2, b)) % R_MOD == 0


def test_mle_eval_definition_and_boolean_points():
    m = 5
    tab = fr_array(rand_fr(1 << m))
    u = rand_fr(m)
    brute = 0
    for bits in itertools.product((0, 1), repeat=m):
        idx = int("".join(map(str, bits)), 2)
        w = 1
        for uk, bk in zip(u, bits):
            w = w * (uk * bk + (1 - uk) * (1 - bk)) % R_MOD
        brute = (brute + tab[idx] * w) % R_MOD
    assert mle_eval(tab, u) == brute
    for idx in (0, 1, 13, 31):
        assert mle_eval(tab, [(idx >> (m - 1 - k)) & 1 for k in range(m)]) == tab[idx]


def test_fold_binds_the_most_significant_variable():
    m = 4
    tab = fr_array(rand_fr(1 << m))
    u = rand_fr(m)
    cur = tab
    for uk in u:
        cur = fold(cur, uk)
    assert cur.shape == (1,) and cur[0] == mle_eval(tab, u)
    assert [int(x) for x in fold(tab, 0)] == [int(x) for x in tab[:8]]
    assert [int(x) for x in fold(tab, 1)] == [int(x) for x in tab[8:]]


@pytest.mark.parametrize("axis", [0, 1, 2])
def test_partial_eval_each_axis(axis):
    shape = [4, 8, 2]
    n = 64
    tab = fr_array(rand_fr(n))
    pts = [rand_fr(2), rand_fr(3), rand_fr(1)]
    out, oshape = partial_eval(tab, shape, axis, axis + 1, pts[axis])
    assert oshape == shape[:axis] + shape[axis + 1:]
    # definition, entry by entry, from the 3-d array
    t3 = tab.reshape(shape)
    o3 = out.reshape(oshape)
    bt = beta_table(pts[axis])
    for idx in itertools.product(*[range(s) for s in oshape]):
        acc = 0
        for a in range(shape[axis]):
            full = list(idx)
            full.insert(axis, a)
            acc = (acc + bt[a] * t3[tuple(full)]) % R_MOD
        assert o3[idx] == acc
    # evaluating the remaining axes gives the full evaluation at the concatenated point
    rest = [p for k, p in enumerate(pts) if k != axis]
    assert mle_eval(out, rest[0] + rest[1]) == mle_eval(tab, pts[0] + pts[1] + pts[2])


def test_partial_eval_multi_axis_and_signed_inputs():
    vals = rng.integers(-2 ** 31, 2 ** 31, 32)
    tab = fr_array(vals)
    assert tab[0] == int(vals[0]) % R_MOD
    p = rand_fr(5)
    out, oshape = partial_eval(tab, [4, 2, 4], 0, 3, p)
    assert oshape == [] and out[0] == mle_eval(tab, p)
    out2, _ = partial_eval(tab, [4, 2, 4], 1, 3, p[2:])
    assert mle_eval(out2, p[:2]) == mle_eval(tab, p)
