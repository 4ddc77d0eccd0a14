"""CPU-side checks of the HIP library: it loads, exports the declared ABI, and
its host-compiled field arithmetic and transcript agree with the oracle."""
import os
import re

import numpy as np
import pytest

import paper_2307_16273_amd as zk
from oracle.field import R_MOD
from oracle.transcript import Transcript as OracleTranscript

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = zk.load_library()
    header = open(os.path.join(ROOT, "include", "zkdl.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b([a-z_0-9]+)\s*\(", header)) - {"defined"}
    declared = {d for d in declared if d.startswith(("zkdl_", "fr_", "mle_", "sumcheck_", "zkrelu_",
                                                       "aggregate_", "reindex_", "claims_", "hyrax_", "update_"))}
    assert declared == set(zk.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name


def test_montgomery_constants_rederive():
    assert zk.selfcheck_constants() == 0
    assert zk.commit_selfcheck() == 0       # the base field of the commitments


def test_host_fr_mul_matches_python_integers():
    rng = np.random.default_rng(5)
    edge = [0, 1, 2, R_MOD - 1, R_MOD - 2, (1 << 255) % R_MOD, (1 << 32) - 1, 1 << 32,
            (1 << 254) + 12345, R_MOD // 2, R_MOD // 2 + 1]
    vals = edge + [int.from_bytes(rng.bytes(40), "little") % R_MOD for _ in range(40)]
    for a in vals[:16]:
        for b in vals:
            assert zk.host_fr_mul(a, b) == a * b % R_MOD
    # non-canonical inputs are reduced
    assert zk.host_fr_mul(R_MOD + 5, 3) == 15
    assert zk.host_fr_mul((1 << 256) - 1, (1 << 256) - 1) == ((1 << 256) - 1) ** 2 % R_MOD


def test_host_transcript_matches_oracle_format():
    for seed in (0, 1, 2 ** 63 + 5):
        a, b = zk.Transcript(seed), OracleTranscript(seed)
        assert a.digest() == b.digest()
        for label, data in ((b"g", b"\x01" * 128), (b"sumcheck_product", b"\x03\0\0\0\x18\0\0\0"),
                            (b"", b""), (b"x" * 32, bytes(range(200)))):
            a.absorb(label, data)
            b.absorb(label, data)
            assert a.digest() == b.digest()
            assert a.challenge() == b.challenge()
            assert a.digest() == b.digest()


def _host_transcript(seed):
    return zk.Transcript(seed)


def test_host_verifier_accepts_the_oracles_proofs_and_rejects_tampering():
    """The library's verifier (the program that also runs on the GPU), compiled for the host: it accepts the
    oracle's proofs of both forms, ends in the oracle's transcript state with the oracle's challenges,
    reports the claims the oracle's verifier returns, and refuses every flipped byte as the oracle does."""
    from oracle import protocols as P
    from workloads import fcnn_window, CONFIG_SEED
    for shape in ((2, 8, 4, 2), (1, 4, 2, 1), (4, 4, 2, 1)):
        wit = fcnn_window(CONFIG_SEED + 130, *shape)
        for ft in (False, True):
            ots = OracleTranscript(9)
            buf, _ = (P.aggregate_ft_prove if ft else P.aggregate_prove)(wit, ots)
            tr = _host_transcript(9)
            got = zk.aggregate_verify(None, buf, tr)
            assert got["verdict"] == 0
            assert got["points"] == ots.challenges
            assert tr.digest() == ots.digest()
            if not ft:
                res = P.aggregate_verify(buf, OracleTranscript(9))
                n = shape[0] * shape[3]
                names = {"fwd": ("Z", "A", "W"), "gradA": ("GA", "GZ_NEXT", "W_NEXT"), "gradW": ("GW", "A", "GZ")}
                k = 0
                for fam in ("fwd", "gradA", "gradW"):
                    proof, _ = res[fam]
                    assert got["claims_left"][k]["tensor"] == names[fam][0] and got["claims_left"][k]["value"] == proof.claim0
                    assert [c["value"] for c in got["claims_left"][k + 1:k + 3]] == proof.finals[1:]
                    k += 3
                assert [c["value"] for c in got["claims_left"][9:13]] == res["zkrelu"]["c_in"]
                assert got["claims_left"][13]["point"] == res["zkrelu"]["aux_claim"]["point"]
                assert got["claims_left"][13]["value"] == res["zkrelu"]["aux_claim"]["value"]
            # tampering: the library refuses a flip of ANY byte and leaves the transcript alone; where the byte
            # belongs to a field element (sampled; the oracle's parser is not hardened against broken size
            # words) the oracle's verifier refuses it as well
            for pos in range(len(buf)):
                bad = bytearray(buf)
                bad[pos] ^= 0x04
                tr2 = _host_transcript(9)
                before = tr2.digest()
                assert zk.aggregate_verify(None, bytes(bad), tr2)["verdict"] != 0, pos
                assert tr2.digest() == before
            first_element = 32 + (16 if not ft else 16)
            for pos in (first_element + 5, first_element + 32 + 7, len(buf) // 2 + 40, len(buf) - 70, len(buf) - 3):
                bad = bytearray(buf)
                bad[pos] ^= 0x04
                with pytest.raises(AssertionError):
                    (P.aggregate_ft_verify if ft else P.aggregate_verify)(bytes(bad), OracleTranscript(9))
            # a proof on the wrong transcript is refused too
            assert zk.aggregate_verify(None, buf, _host_transcript(10))["verdict"] != 0
            # truncated and extended proofs
            assert zk.aggregate_verify(None, buf[:-1], _host_transcript(9))["verdict"] != 0
            assert zk.aggregate_verify(None, buf + b"\x00", _host_transcript(9))["verdict"] != 0


def _flip_everything(buf, seed, step=1, draws=True):
    for pos in range(0, len(buf), step):
        bad = bytearray(buf)
        bad[pos] ^= 0x04
        tr2 = _host_transcript(seed)
        before = tr2.digest()
        assert zk.aggregate_verify(None, bytes(bad), tr2)["verdict"] != 0, pos
        assert tr2.digest() == before
    if draws:   # a proof without a single round uses no challenge: it holds on any transcript
        assert zk.aggregate_verify(None, buf, _host_transcript(seed + 1))["verdict"] != 0
    assert zk.aggregate_verify(None, buf[:-1], _host_transcript(seed))["verdict"] != 0
    assert zk.aggregate_verify(None, buf + b"\x00", _host_transcript(seed))["verdict"] != 0


def test_host_verifier_on_linked_windows():
    """The chained window ("ZKAL"): accepted with the oracle's challenges and transcript state; every link is
    checked (a flip of any byte is refused, also where only a link between two parts notices it)."""
    from oracle import protocols as P
    from workloads import fcnn_window, CONFIG_SEED
    for shape in ((2, 8, 4, 2), (1, 4, 2, 1), (4, 4, 2, 2)):
        wit = fcnn_window(CONFIG_SEED + 131, *shape)
        ots = OracleTranscript(11)
        buf, _ = P.aggregate_linked_prove(wit, ots)
        tr = _host_transcript(11)
        got = zk.aggregate_verify(None, buf, tr)
        assert got["verdict"] == 0, got["verdict"]
        assert got["points"] == ots.challenges
        assert tr.digest() == ots.digest()
        _flip_everything(buf, 11, step=1 if shape[0] == 1 else 3)


def test_host_verifier_on_update_proofs():
    from oracle import protocols as P
    import numpy as np
    for d, q, r in ((1, 5, 3), (8, 6, 4), (32, 32, 30)):
        rng = np.random.default_rng(d)
        lim = 1 << (q + r - 1)
        g = [int(x) for x in rng.integers(-lim + 1, lim, d)]
        ots = OracleTranscript(12)
        buf, _ = P.update_prove(g, q, r, ots)
        tr = _host_transcript(12)
        got = zk.aggregate_verify(None, buf, tr)
        assert got["verdict"] == 0, got["verdict"]
        assert got["points"] == ots.challenges
        assert tr.digest() == ots.digest()
        _flip_everything(buf, 12)


def test_host_verifier_on_general_form_proofs():
    from oracle import protocols as P
    from oracle.field import fr_array
    import numpy as np
    for n, d1, d2, d3 in ((2, 2, 4, 2), (1, 4, 8, 2), (4, 1, 2, 4), (4, 4, 1, 1), (1, 1, 1, 1)):
        rng = np.random.default_rng(n + d2)
        x0 = rng.integers(-100, 100, (n, d1, d2))
        x1 = rng.integers(-100, 100, (n, d2, d3))
        y = np.einsum("nij,njk->nik", x0, x1)
        ots = OracleTranscript(14)
        buf, _ = P.matmul_general_prove(fr_array(x0), [n, d1, d2], fr_array(x1), [n, d2, d3], fr_array(y), ots)
        tr = _host_transcript(14)
        got = zk.aggregate_verify(None, buf, tr)
        assert got["verdict"] == 0, got["verdict"]
        assert got["points"] == ots.challenges and tr.digest() == ots.digest()
        _flip_everything(buf, 14, draws=n * d1 * d2 * d3 > 1)


def test_host_scalar_split_is_the_division_by_z_squared():
    """hyrax_verify multiplies by k as a P + b (-phi(P)) with k = a + b z^2: the host's long division against
    Python's divmod, on the edge values of the quotient estimate and on random scalars."""
    zz = 0xd201000000010000 ** 2
    assert zz * zz - zz + 1 == R_MOD                              # r = z^4 - z^2 + 1
    rng = np.random.default_rng(17)
    ks = [0, 1, zz - 1, zz, zz + 1, R_MOD - 1, R_MOD, (1 << 128) * zz - 1, 3 * zz - 1, (zz - 1) * zz + zz - 1,
          (1 << 255) - 1, (1 << 192) - 1, 1 << 160, ((1 << 128) - 1) * zz]
    ks += [int.from_bytes(rng.bytes(32), "little") % R_MOD for _ in range(3000)]
    ks += [(int.from_bytes(rng.bytes(16), "little") >> 1) * zz + d for d in (0, 1, zz - 1) for _ in range(200)]
    ks += [int("".join(rng.choice(["00000000", "ffffffff"]) for _ in range(8)), 16) % ((1 << 128) * zz) for _ in range(500)]
    for k in ks:
        assert zk.host_scalar_split(k) == (k % zz, k // zz), hex(k)
    with pytest.raises(zk.ZkdlError):
        zk.host_scalar_split((1 << 128) * zz)                       # the quotient no longer fits 128 bits
    with pytest.raises(zk.ZkdlError):
        zk.host_scalar_split((1 << 256) - 1)
