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


def _sha256_compress(h, block):
    """One application of the SHA-256 compression function (FIPS 180-4, Sec. 6.2.2)."""
    def rotr(x, n):
        return ((x >> n) | (x << (32 - n))) & 0xFFFFFFFF
    # round constants: fractional parts of the cube roots of the first 64 primes
    primes, c = [], 2
    while len(primes) < 64:
        if all(c % p for p in primes):
            primes.append(c)
        c += 1

    def icbrt(n):
        x = int(round(n ** (1.0 / 3)))
        while x ** 3 > n:
            x -= 1
        while (x + 1) ** 3 <= n:
            x += 1
        return x
    k = [icbrt(p << 96) & 0xFFFFFFFF for p in primes]
    w = list(struct.unpack(">16I", block))
    for t in range(16, 64):
        s0 = rotr(w[t - 15], 7) ^ rotr(w[t - 15], 18) ^ (w[t - 15] >> 3)
        s1 = rotr(w[t - 2], 17) ^ rotr(w[t - 2], 19) ^ (w[t - 2] >> 10)
        w.append((w[t - 16] + s0 + w[t - 7] + s1) & 0xFFFFFFFF)
    a, b, c_, d, e, f, g, hh = h
    for t in range(64):
        t1 = (hh + (rotr(e, 6) ^ rotr(e, 11) ^ rotr(e, 25)) + ((e & f) ^ (~e & g)) + k[t] + w[t]) & 0xFFFFFFFF
        t2 = ((rotr(a, 2) ^ rotr(a, 13) ^ rotr(a, 22)) + ((a & b) ^ (a & c_) ^ (b & c_))) & 0xFFFFFFFF
        a, b, c_, d, e, f, g, hh = (t1 + t2) & 0xFFFFFFFF, a, b, c_, (d + t1) & 0xFFFFFFFF, e, f, g
    return [(x + y) & 0xFFFFFFFF for x, y in zip(h, (a, b, c_, d, e, f, g, hh))]


_SHA256_IV = [0x6a09e667, 0xbb67ae85, 0x3c6ef372, 0xa54ff53a, 0x510e527f, 0x9b05688c, 0x1f83d9ab, 0x5be0cd19]


def test_transcript_format():
    # SHA-256 itself: NIST "abc" vector through the same library call
    assert hashlib.sha256(b"abc").hexdigest() == \
        "ba7816bf8f01cfea414140de5dae2223b00361a396177a9cb410ff61f20015ad"
    # every value is a one-shot hash of an explicitly written byte stream
    t = Transcript(9)
    stream = b"zkdl-mi355x/v3" + b"\0" * 42 + struct.pack("<Q", 9)
    assert len(stream) == 64 and t.digest() == hashlib.sha256(stream).digest()
    t.absorb(b"g", b"\x01\x02")
    stream += b"\x01g" + struct.pack("<Q", 2) + b"\x01\x02"
    assert len(stream) == 76 and t.digest() == hashlib.sha256(stream).digest()
    c = t.challenge()
    z4 = struct.pack("<I", 0)
    wide = hashlib.sha256(stream + b"\xf0" + z4).digest() + hashlib.sha256(stream + b"\xf1" + z4).digest()
    assert c == int.from_bytes(wide, "little") % R_MOD
    s1 = stream
    stream += b"\xf2" + b"\0" * 51      # a draw closes the block
    assert len(stream) == 128 and t.digest() == hashlib.sha256(stream).digest()
    assert t.challenge() != c
    # a vector draw: index-derived elements, one stream extension
    t2 = Transcript(9)
    t2.absorb(b"g", b"\x01\x02")
    vec = t2.challenges_vec(3)
    assert vec[0] == c and len(set(vec)) == 3 and t2.digest() == hashlib.sha256(stream).digest()
    i2 = struct.pack("<I", 2)
    wide = hashlib.sha256(s1 + b"\xf0" + i2).digest() + hashlib.sha256(s1 + b"\xf1" + i2).digest()
    assert vec[2] == int.from_bytes(wide, "little") % R_MOD
    assert t2.challenges_vec(0) == [] and t2.digest() == hashlib.sha256(stream).digest()
    # frames are appended without padding, whatever their length; a draw on an aligned stream
    # appends a whole block
    t3 = Transcript(1)
    s3 = b"zkdl-mi355x/v3" + b"\0" * 42 + struct.pack("<Q", 1)
    for label, data in ((b"f", bytes(range(96))), (b"x", bytes(54)), (b"y" * 32, bytes(200)), (b"", b"")):
        t3.absorb(label, data)
        s3 += bytes([len(label)]) + label + struct.pack("<Q", len(data)) + data
        assert t3.digest() == hashlib.sha256(s3).digest()
    t3.challenge()
    s3 += b"\xf2" + b"\0" * (-(len(s3) + 1) % 64)
    assert len(s3) % 64 == 0 and t3.digest() == hashlib.sha256(s3).digest()
    t3.challenge()
    s3 += b"\xf2" + b"\0" * 63
    assert t3.digest() == hashlib.sha256(s3).digest()


def test_transcript_round_step_is_two_compressions_deep():
    """The property the format is built for: after a draw the stream is block-aligned, so
    absorbing a round's 106-byte frame and drawing the challenge is one compression for the
    frame's first 64 bytes and then independent single compressions from that chaining value."""
    assert b"".join(struct.pack(">I", x) for x in _sha256_compress(
        _SHA256_IV, b"abc\x80" + b"\0" * 52 + struct.pack(">Q", 24))) == hashlib.sha256(b"abc").digest()
    t = Transcript(5)
    t.challenge()                      # leaves the stream aligned: 128 bytes
    t.absorb_fr(b"g", [3, 4, 5])
    head = b"zkdl-mi355x/v3" + b"\0" * 42 + struct.pack("<Q", 5) + b"\xf2" + b"\0" * 63
    frame = b"\x01g" + struct.pack("<Q", 96) + to_le(3) + to_le(4) + to_le(5)
    assert len(head) == 128 and len(frame) == 106
    h = _SHA256_IV
    for off in (0, 64):
        h = _sha256_compress(h, head[off:off + 64])
    h = _sha256_compress(h, frame[:64])                     # the one sequential compression
    rest = frame[64:]                                       # 42 bytes
    halves = []
    for tag in (0xF0, 0xF1):
        last = rest + bytes([tag]) + struct.pack("<I", 0) + b"\x80"
        last += b"\0" * (56 - len(last)) + struct.pack(">Q", 8 * (128 + 106 + 5))
        assert len(last) == 64
        halves.append(b"".join(struct.pack(">I", x) for x in _sha256_compress(h, last)))
    assert t.challenge() == int.from_bytes(halves[0] + halves[1], "little") % R_MOD
    h = _sha256_compress(h, rest + b"\xf2" + b"\0" * 21)
    fin = b"\x80" + b"\0" * 55 + struct.pack(">Q", 8 * 256)
    assert t.digest() == b"".join(struct.pack(">I", x) for x in _sha256_compress(h, fin))


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
