"""Pins for the C tier of the oracle: byte-for-byte agreement with the Python-integer tier
(itself pinned against brute force and closed forms), and its field / hash primitives against
Python integers and hashlib."""
import hashlib

import numpy as np
import pytest

from oracle import c_oracle
from oracle import protocols as P
from oracle.field import R_MOD, fr_array_from_le, array_to_le
from oracle.mle import partial_eval
from oracle.transcript import Transcript
from workloads import uniform_fr_limbs


def test_field_product_against_python_integers():
    rng = np.random.default_rng(11)
    edge = [0, 1, 2, R_MOD - 1, R_MOD - 2, (R_MOD - 1) // 2, 1 << 254, (1 << 64) - 1, 1 << 64, (1 << 128) + 12345]
    vals = edge + [int.from_bytes(uniform_fr_limbs(rng, 1).tobytes(), "little") for _ in range(40)]
    for a in vals:
        for b in vals[:14]:
            assert c_oracle.fe_mul(a, b) == a * b % R_MOD


def test_sha256_against_hashlib():
    for n in (0, 1, 3, 55, 56, 63, 64, 65, 119, 120, 200, 1000):
        data = bytes((7 * i + n) & 0xFF for i in range(n))
        assert c_oracle.sha256(data) == hashlib.sha256(data).digest()


@pytest.mark.parametrize("k,d", [(1, 1), (2, 3), (3, 1), (3, 4), (3, 9), (2, 10)])
def test_product_sumcheck_matches_python_tier(k, d):
    n = 1 << d
    rng = np.random.default_rng(100 * k + d)
    raws = [uniform_fr_limbs(rng, n).tobytes() for _ in range(k)]
    proof, vs, digest = c_oracle.product_prove(raws, seed=31 + d)
    ts = Transcript(31 + d)
    buf, _, vs_py = P.product_prove([fr_array_from_le(r, n) for r in raws], ts)
    assert proof == buf
    assert vs == vs_py
    assert digest == ts.digest()


@pytest.mark.parametrize("outer,axis,inner", [(1, 8, 4), (3, 16, 1), (2, 1, 5), (1, 64, 32)])
def test_partial_eval_matches_python_tier(outer, axis, inner):
    rng = np.random.default_rng(outer * 1000 + axis)
    n = outer * axis * inner
    raw = uniform_fr_limbs(rng, n).tobytes()
    la = axis.bit_length() - 1
    point = [int.from_bytes(uniform_fr_limbs(rng, 1).tobytes(), "little") for _ in range(la)]
    got = c_oracle.partial_eval(raw, outer, axis, inner, point)
    expect, _ = partial_eval(fr_array_from_le(raw, n), [outer, axis, inner], 1, 2, point)
    assert got == array_to_le(expect)
