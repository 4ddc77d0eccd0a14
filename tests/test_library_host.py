"""CPU-side checks of the HIP library: it loads, exports the declared ABI, and
its host-compiled field arithmetic and transcript agree with the oracle."""
import os
import re

import numpy as np

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
                                                       "aggregate_", "reindex_", "claims_", "hyrax_"))}
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
