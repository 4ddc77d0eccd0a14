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


def test_field_sum_and_difference_against_python_integers():
    rng = np.random.default_rng(12)
    edge = [0, 1, 2, R_MOD - 1, R_MOD - 2, (R_MOD - 1) // 2, (R_MOD + 1) // 2, 1 << 254, (1 << 64) - 1, 1 << 64,
            (1 << 192) - 1, 1 << 192, R_MOD - (1 << 64), R_MOD - (1 << 192)]
    vals = edge + [int.from_bytes(uniform_fr_limbs(rng, 1).tobytes(), "little") for _ in range(30)]
    for a in vals:
        for b in vals:
            assert c_oracle.fe_add(a, b) == (a + b) % R_MOD
            assert c_oracle.fe_sub(a, b) == (a - b) % R_MOD


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


# --------------------------------------------------------------------------
# the protocol provers of the C tier against the Python tier, byte for byte
# --------------------------------------------------------------------------
def _same(cts, ts, got, buf):
    assert got == bytes(buf)
    assert cts.challenges == ts.challenges
    assert cts.digest() == ts.digest()


def _rand_point(rng, n):
    return [int.from_bytes(uniform_fr_limbs(rng, 1).tobytes(), "little") for _ in range(n)]


def test_transcript_object_matches_python_tier():
    ts, cts = Transcript(123), c_oracle.Transcript(123)
    for t in (ts, cts):
        t.absorb(b"label", b"\x01\x02\x03")
    assert cts.challenges_vec(3) == ts.challenges_vec(3)
    for t in (ts, cts):
        t.absorb(b"x" * 32, bytes(range(200)))
    assert cts.challenges_vec(0) == [] and ts.challenges_vec(0) == []
    assert cts.digest() == ts.digest()
    assert cts.challenges_vec(70) == ts.challenges_vec(70)
    assert cts.challenges == ts.challenges and cts.digest() == ts.digest()


@pytest.mark.parametrize("n,d1,d2,d3", [(1, 2, 4, 2), (4, 8, 16, 2), (2, 1, 2, 1), (8, 1, 1, 4), (1, 1, 1, 1), (2, 4, 32, 8)])
def test_matmul_matches_python_tier(n, d1, d2, d3):
    rng = np.random.default_rng(7 * n + d2)
    x0 = uniform_fr_limbs(rng, n * d1 * d2).tobytes()
    x1 = uniform_fr_limbs(rng, n * d2 * d3).tobytes()
    ts, cts = Transcript(3), c_oracle.Transcript(3)
    buf, _, _ = P.matmul_prove(fr_array_from_le(x0, n * d1 * d2), [n, d1, d2], fr_array_from_le(x1, n * d2 * d3), [n, d2, d3], ts)
    _same(cts, ts, c_oracle.matmul_prove(x0, [n, d1, d2], x1, [n, d2, d3], cts), buf)


@pytest.mark.parametrize("n,d1,d2,d3", [(1, 2, 4, 2), (4, 8, 16, 2), (2, 1, 2, 1), (8, 1, 1, 4), (1, 1, 1, 1), (16, 2, 8, 4)])
def test_matmul_ft_matches_python_tier(n, d1, d2, d3):
    rng = np.random.default_rng(11 * n + d2)
    x0 = uniform_fr_limbs(rng, n * d1 * d2).tobytes()
    x1 = uniform_fr_limbs(rng, n * d2 * d3).tobytes()
    ts, cts = Transcript(3), c_oracle.Transcript(3)
    buf, _ = P.matmul_ft_prove(fr_array_from_le(x0, n * d1 * d2), [n, d1, d2], fr_array_from_le(x1, n * d2 * d3), [n, d2, d3], ts)
    _same(cts, ts, c_oracle.matmul_ft_prove(x0, [n, d1, d2], x1, [n, d2, d3], cts), buf)


@pytest.mark.parametrize("d", [0, 1, 5, 9])
def test_hadamard_matches_python_tier(d):
    rng = np.random.default_rng(60 + d)
    x0 = uniform_fr_limbs(rng, 1 << d).tobytes()
    x1 = uniform_fr_limbs(rng, 1 << d).tobytes()
    ts, cts = Transcript(4), c_oracle.Transcript(4)
    buf, _, _ = P.hadamard_prove(fr_array_from_le(x0, 1 << d), fr_array_from_le(x1, 1 << d), ts)
    _same(cts, ts, c_oracle.hadamard_prove(x0, x1, cts), buf)


def _zk_inputs(rng, d_len, q, r):
    lim = 1 << (q + r - 1)
    z = [int(v) for v in rng.integers(-lim, lim, d_len, dtype=np.int64)] if q + r < 64 else \
        [int(v) for v in rng.integers(-2 ** 63, 2 ** 63 - 1, d_len, dtype=np.int64, endpoint=True)]
    g = list(reversed(z))
    edge = [0, -1, lim - 1, -lim, 1 << (r - 1), -(1 << (r - 1)), (1 << (r - 1)) - 1]
    for k, e in enumerate(edge[:d_len]):
        z[k] = e
        g[d_len - 1 - k] = e
    return z, g


@pytest.mark.parametrize("d_len,with_ga,q,r", [(1, True, 5, 3), (2, False, 5, 3), (8, True, 5, 3), (16, True, 32, 16),
                                               (4, True, 4, 4), (8, True, 48, 16), (8, False, 63, 1), (32, True, 10, 1)])
def test_zkrelu_matches_python_tier(d_len, with_ga, q, r):
    z, g = _zk_inputs(np.random.default_rng(d_len + q), d_len, q, r)
    ts, cts = Transcript(9), c_oracle.Transcript(9)
    buf, _ = P.zkrelu_prove(z, g if with_ga else None, q, r, ts)
    _same(cts, ts, c_oracle.zkrelu_prove(z, g if with_ga else None, q, r, cts), buf)


@pytest.mark.parametrize("bind", [True, False])
def test_zkrelu_at_given_points_matches_python_tier(bind):
    rng = np.random.default_rng(17)
    d_len, q, r = 8, 6, 2
    z, g = _zk_inputs(rng, d_len, q, r)
    pts = [_rand_point(rng, 3) for _ in range(4)]
    ts, cts = Transcript(10), c_oracle.Transcript(10)
    buf, _ = P.zkrelu_prove(z, g, q, r, ts, points=pts, bind_points=bind)
    _same(cts, ts, c_oracle.zkrelu_prove(z, g, q, r, cts, points=pts, bind_points=bind), buf)


def test_zkrelu_range_error_as_in_python_tier():
    with pytest.raises(ValueError):
        P.zkrelu_prove([0, 128, 0, 0], None, 5, 3, Transcript(1))
    with pytest.raises(c_oracle.OracleError) as e:
        c_oracle.zkrelu_prove([0, 128, 0, 0], None, 5, 3, c_oracle.Transcript(1))
    assert e.value.rc == -5
    with pytest.raises(c_oracle.OracleError):
        c_oracle.zkrelu_prove([0, 0, 0, 0], [0, 0, -129, 0], 5, 3, c_oracle.Transcript(1))
    c_oracle.zkrelu_prove([0, 127, -128, 0], None, 5, 3, c_oracle.Transcript(1))


@pytest.mark.parametrize("n,d,bind", [(4, 8, True), (8, 2, False), (1, 4, True), (16, 1, False)])
def test_reindex_matches_python_tier(n, d, bind):
    rng = np.random.default_rng(n * 31 + d)
    x = uniform_fr_limbs(rng, n * d).tobytes()
    maps = [list(range(n)), [j + 1 if j + 1 < n else -1 for j in range(n)], [0] * (2 * n)]
    pts = [_rand_point(rng, (len(m) - 1).bit_length()) for m in maps]
    u = _rand_point(rng, d.bit_length() - 1)
    ts, cts = Transcript(12), c_oracle.Transcript(12)
    buf, _ = P.reindex_prove(fr_array_from_le(x, n * d).reshape(n, d), n, d, maps, pts, u, ts, bind_statement=bind)
    _same(cts, ts, c_oracle.reindex_prove(x, n, d, maps, pts, u, cts, bind_statement=bind), buf)


@pytest.mark.parametrize("n,d,k,bind", [(4, 8, 2, True), (1, 8, 2, False), (8, 1, 3, True), (2, 2, 5, False), (4, 4, 1, True)])
def test_stack_merge_matches_python_tier(n, d, k, bind):
    rng = np.random.default_rng(n * 77 + d + k)
    x = uniform_fr_limbs(rng, n * d).tobytes()
    pts = [_rand_point(rng, (n * d).bit_length() - 1) for _ in range(k)]
    ts, cts = Transcript(13), c_oracle.Transcript(13)
    buf, _ = P.stack_merge_prove(fr_array_from_le(x, n * d), n, d, pts, ts, bind_statement=bind)
    _same(cts, ts, c_oracle.stack_merge_prove(x, n, d, pts, cts, bind_statement=bind), buf)


@pytest.mark.parametrize("d,q,r", [(1, 5, 3), (2, 4, 4), (8, 6, 4), (64, 10, 6), (256, 32, 30), (128, 33, 30)])
def test_update_matches_python_tier(d, q, r):
    rng = np.random.default_rng(d + q)
    lim = 1 << (q + r - 1)
    g = rng.integers(-lim + 1, lim, d, dtype=np.int64)
    half = 1 << (r - 1)
    for k, v in enumerate([half, -half, 0, lim - 1, -lim + 1]):
        if k < d:
            g[k] = v
    ts, cts = Transcript(16), c_oracle.Transcript(16)
    buf, _ = P.update_prove([int(x) for x in g], q, r, ts)
    _same(cts, ts, c_oracle.update_prove(g, q, r, cts), buf)


def test_update_range_error_as_in_python_tier():
    for g in ([1 << 9, 0], [-(1 << 9), 0]):
        with pytest.raises(ValueError):
            P.update_prove(g, 5, 5, Transcript(1))
        with pytest.raises(c_oracle.OracleError):
            c_oracle.update_prove(np.array(g, dtype=np.int64), 5, 5, c_oracle.Transcript(1))


@pytest.mark.parametrize("layers,width,batch,steps", [(2, 8, 4, 2), (4, 16, 2, 1), (1, 16, 2, 1), (2, 4, 2, 4), (8, 8, 4, 1)])
@pytest.mark.parametrize("linked", [False, True, "ft"])
def test_aggregate_matches_python_tier(layers, width, batch, steps, linked):
    from workloads import fcnn_window, CONFIG_SEED
    wit = fcnn_window(CONFIG_SEED + 50 + layers, layers, width, batch, steps)
    ts, cts = Transcript(14), c_oracle.Transcript(14)
    for t in (ts, cts):
        t.absorb(b"weights", b"\x07" * 32)       # a caller's binding of its tensors
    if linked == "ft":
        buf, _ = P.aggregate_ft_prove(wit, ts)
        got = c_oracle.aggregate_prove(wit, cts, ft=True)
    else:
        buf, _ = (P.aggregate_linked_prove if linked else P.aggregate_prove)(wit, ts)
        got = c_oracle.aggregate_prove(wit, cts, linked=linked)
    _same(cts, ts, got, buf)


@pytest.mark.parametrize("name", ["aggregate_l2_w4_b2_t2", "aggregate_linked_l2_w4_b2_t2", "zkrelu_d4_q5_r3", "matmul_n2_2x4x2"])
def test_c_tier_reproduces_stored_proofs(name):
    import json
    import os
    from oracle.field import fr_array
    from workloads import fcnn_window
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name + ".json")) as f:
        g = json.load(f)
    cts = c_oracle.Transcript(g["seed"])
    if g["protocol"] == "sumcheck_matmul":
        got = c_oracle.matmul_prove(array_to_le(fr_array(np.array(g["x0"]))), g["x0_shape"],
                                    array_to_le(fr_array(np.array(g["x1"]))), g["x1_shape"], cts)
    elif g["protocol"] == "zkrelu_prove":
        got = c_oracle.zkrelu_prove(g["Z"], g["GA"], g["Q"], g["R"], cts)
    else:
        got = c_oracle.aggregate_prove(fcnn_window(2307162730 + 90, 2, 4, 2, 2), cts,
                                       linked=g["protocol"] == "aggregate_prove_linked")
    assert got.hex() == g["proof_hex"]
    assert [hex(v) for v in cts.challenges] == g["challenges"]
    assert cts.digest().hex() == g["digest_hex"]


def test_thread_count_does_not_change_the_proof():
    from workloads import fcnn_window, CONFIG_SEED
    wit = fcnn_window(CONFIG_SEED + 3, 2, 8, 4, 1)
    before = c_oracle.threads()
    outs = []
    for nt in (1, 3, before):
        c_oracle.set_threads(nt)
        cts = c_oracle.Transcript(2)
        outs.append((c_oracle.aggregate_prove(wit, cts), cts.digest()))
    c_oracle.set_threads(before)
    assert outs[0] == outs[1] == outs[2]
