"""GPU parity of the commitments: generators, row commitments and openings of the HIP library against the
Python-integer oracle (oracle/curve.py), byte for byte."""
import numpy as np
import pytest

from oracle import curve as EC
from oracle.field import R_MOD
from oracle.transcript import Transcript as OracleTranscript

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def test_generators_match_the_oracle(lib, ctx):
    say("commit key: generators")
    key = lib.CommitKey(ctx, b"parity", 16)
    got = key.generators(0, 17)
    gens, h = EC.generators(b"parity", 16)
    assert got == [EC.point_to_bytes(p) for p in gens + [h]]
    other = lib.CommitKey(ctx, b"", 2)
    assert other.generators(0, 3) == [EC.point_to_bytes(p) for p in
                                      EC.generators(b"", 2)[0] + [EC.generators(b"", 2)[1]]]


@pytest.mark.parametrize("numel,dtype,blinded", [(1, "i32", True), (2, "i32", False), (64, "i32", True), (256, "i64", True),
                                                 (2048, "i32", True), (512, "i64", False)])
@pytest.mark.parametrize("wbits", [8, 12])
def test_row_commitments_match_the_oracle(lib, ctx, numel, dtype, blinded, wbits):
    """Both widths of the fixed-base windows (the key picks one by table size; the commitments do not depend on it)."""
    import torch
    say(f"hyrax_commit numel={numel} {dtype} blinded={blinded} window bits={wbits}")
    rng = np.random.default_rng(numel + 7)
    if dtype == "i32":
        vals = rng.integers(-2 ** 31, 2 ** 31, numel, dtype=np.int64).astype(np.int32)
        edge = [0, -1, 2 ** 31 - 1, -2 ** 31, 1, 16, -16, 255, 4095, 4096, -4096, 2 ** 24 - 1, -2 ** 24, 256, 0xFFF000]
    else:
        vals = rng.integers(-2 ** 47, 2 ** 47, numel, dtype=np.int64)
        edge = [0, -1, 2 ** 63 - 1, -2 ** 63, 2 ** 47 - 1, -2 ** 47, 1 << 60, -(1 << 32), 4095, -4096, 1 << 36,
                (1 << 48) - 1, 0xFFF000FFF000]
    vals[:min(numel, len(edge))] = edge[:min(numel, len(edge))]
    rows, cols = EC.matrix_shape(numel)
    ctx.set_commit_window_bits(wbits)
    try:
        key = lib.CommitKey(ctx, b"rows", cols, 64 if dtype == "i64" else 32)
    finally:
        ctx.set_commit_window_bits(0)
    blind = [int(v) for v in rng.integers(1, 2 ** 62, rows)] if blinded else None
    if blinded:
        blind[0] = R_MOD - 1
    x = lib.tensor_wrap_int(ctx, torch.from_numpy(vals).cuda())
    got = lib.hyrax_commit(ctx, key, x, blind)
    gens, h = EC.generators(b"rows", cols)
    want = EC.commit_rows([int(v) for v in vals], blind if blinded else [0] * rows, gens, h)
    assert got == [EC.point_to_bytes(p) for p in want]


def test_opening_is_accepted_by_the_oracles_verifier(lib, ctx):
    import torch
    say("hyrax_open")
    rng = np.random.default_rng(3)
    numel = 128
    vals = rng.integers(-2 ** 31, 2 ** 31, numel, dtype=np.int64).astype(np.int32)
    rows, cols = EC.matrix_shape(numel)
    key = lib.CommitKey(ctx, b"open", cols)
    blind = [int(v) for v in rng.integers(1, 2 ** 62, rows)]
    x = lib.tensor_wrap_int(ctx, torch.from_numpy(vals).cuda())
    coms = [EC.point_from_bytes(c) for c in lib.hyrax_commit(ctx, key, x, blind)]
    point = [int(v) for v in rng.integers(1, 2 ** 62, 7)]
    t, rho_star, y = lib.hyrax_open(ctx, x, blind, point)
    assert (t, rho_star, y) == EC.open_rows([int(v) for v in vals], blind, point)
    gens, h = EC.generators(b"open", cols)
    assert EC.verify_opening(coms, point, t, rho_star, y, gens, h)


def _combined(coms, point, rows):
    lr = rows.bit_length() - 1
    from oracle.mle import beta_table
    b = beta_table(point[:lr])
    acc = EC.INF
    for j in range(rows):
        acc = EC.add(acc, EC.mul(int(b[j]), coms[j]))
    return acc


@pytest.mark.parametrize("numel,dtype,blinded", [(1, "i32", True), (2, "i32", True), (128, "i32", True), (256, "i64", False),
                                                 (2048, "i32", True)])
def test_library_verifies_openings_as_the_oracle_does(lib, ctx, numel, dtype, blinded):
    """hyrax_verify: the combined commitment equals the oracle's byte for byte; the library's opening is accepted;
    a changed row entry, blinding, value, commitment or point is refused with the verdict of the check that the
    oracle's verifier fails at."""
    import torch
    say(f"hyrax_verify numel={numel} {dtype} blinded={blinded}")
    rng = np.random.default_rng(numel + 11)
    if dtype == "i32":
        vals = rng.integers(-2 ** 31, 2 ** 31, numel, dtype=np.int64).astype(np.int32)
    else:
        vals = rng.integers(-2 ** 60, 2 ** 60, numel, dtype=np.int64)
    rows, cols = EC.matrix_shape(numel)
    key = lib.CommitKey(ctx, b"vfy", cols, 64 if dtype == "i64" else 32)
    blind = [int.from_bytes(rng.bytes(31), "little") for _ in range(rows)] if blinded else None
    x = lib.tensor_wrap_int(ctx, torch.from_numpy(vals).cuda())
    raw = lib.hyrax_commit(ctx, key, x, blind)
    m = numel.bit_length() - 1
    point = [int.from_bytes(rng.bytes(31), "little") for _ in range(m)]
    t, rho_star, y = lib.hyrax_open(ctx, x, blind, point)
    verdict, comb = lib.hyrax_verify(ctx, key, raw, point, t, rho_star if blinded else None, y)
    coms = [EC.point_from_bytes(c) for c in raw]
    assert comb == EC.point_to_bytes(_combined(coms, point, rows))
    assert verdict == 0
    # without the bytes of C* the two sums are compared as projective points
    assert lib.hyrax_verify(ctx, key, raw, point, t, rho_star if blinded else None, y, want_combined=False) == (0, None)
    gens, h = EC.generators(b"vfy", cols)
    assert EC.verify_opening(coms, point, t, rho_star if blinded else 0, y, gens, h)
    # tampering, with the oracle's verifier beside it
    def both(raw_, point_, t_, rho_, y_, want):
        v, _ = lib.hyrax_verify(ctx, key, raw_, point_, t_, rho_, y_)
        assert v == want
        assert lib.hyrax_verify(ctx, key, raw_, point_, t_, rho_, y_, want_combined=False) == (want, None)
        with pytest.raises(AssertionError):
            EC.verify_opening([EC.point_from_bytes(c) for c in raw_], point_, t_, rho_ or 0, y_, gens, h)
    rho_in = rho_star if blinded else None
    both(raw, point, t, rho_in, (y + 1) % R_MOD, 3)
    both(raw, point, [(t[0] + 1) % R_MOD] + t[1:], rho_in, y, 2)
    if blinded:
        both(raw, point, t, (rho_star + 1) % R_MOD, y, 2)
    if rows > 1:
        both([raw[1], raw[0]] + raw[2:], point, t, rho_in, y, 2)
        both(raw, [(point[0] + 1) % R_MOD] + point[1:], t, rho_in, y, 2)
    # a commitment moved by a point of order 3 is on the curve but no element of the group of order r
    both([EC.point_to_bytes(EC.add(coms[0], (0, 2)))] + raw[1:], point, t, rho_in, y, 1)
    # malformed inputs: a commitment off the curve, an element not below r
    off = bytearray(raw[0])
    off[0] ^= 1
    assert lib.hyrax_verify(ctx, key, [bytes(off)] + raw[1:], point, t, rho_in, y)[0] == 1
    assert lib.hyrax_verify(ctx, key, raw, point, [R_MOD] + t[1:], rho_in, y)[0] == 1


def test_library_verifies_the_full_size_opening(lib, ctx):
    """The 2^19 activation stack: 1024 row commitments combined and the 512-entry row recommitted on the GPU."""
    import torch
    from workloads import fcnn_window, CONFIG_SEED
    say("hyrax_verify on the 2^19 activation stack")
    wit = fcnn_window(CONFIG_SEED + 3, n_layers=8, width=1024, batch=64, steps=1)
    vals = np.ascontiguousarray(wit["A"]).reshape(-1)
    rows, cols = EC.matrix_shape(vals.size)
    rng = np.random.default_rng(12)
    blind = [int.from_bytes(rng.bytes(31), "little") for _ in range(rows)]
    key = lib.CommitKey(ctx, b"A", cols)
    x = lib.tensor_wrap_int(ctx, torch.from_numpy(vals).cuda())
    raw = lib.hyrax_commit(ctx, key, x, blind)
    point = [int.from_bytes(rng.bytes(31), "little") for _ in range(19)]
    t, rho_star, y = lib.hyrax_open(ctx, x, blind, point)
    assert lib.hyrax_verify(ctx, key, raw, point, t, rho_star, y)[0] == 0
    assert lib.hyrax_verify(ctx, key, raw, point, t, rho_star, (y + 1) % R_MOD)[0] == 3
    assert lib.hyrax_verify(ctx, key, raw[1:] + raw[:1], point, t, rho_star, y)[0] == 2


@pytest.mark.parametrize("dtype,zeros", [("i32", 0.0), ("i32", 0.9), ("i32", 0.995), ("i64", 0.5), ("i64", 0.97)])
def test_sparse_and_mixed_rows_agree_between_window_widths(lib, ctx, dtype, zeros):
    """Rows whose entries have anything from one to 31 (63) bits and are mostly zero: few digits, rows whose digit
    count is not a multiple of 64, empty rows.  Both window widths give the same commitments, and three rows
    (the first, an all-zero one, the last) equal the oracle's sums."""
    import torch
    say(f"hyrax_commit sparse rows {dtype} zeros={zeros}")
    rng = np.random.default_rng(int(zeros * 1000) + (7 if dtype == "i64" else 3))
    numel = 1 << 14
    top = 31 if dtype == "i32" else 63
    bits = rng.integers(1, top + 1, numel)
    vals = (rng.integers(0, 2 ** 62, numel, dtype=np.int64) >> (62 - bits)) * rng.choice([-1, 1], numel)
    vals[rng.random(numel) < zeros] = 0
    rows, cols = EC.matrix_shape(numel)
    vals[5 * cols:6 * cols] = 0                                     # a row without any digit
    vals = vals.astype(np.int32 if dtype == "i32" else np.int64)
    x = lib.tensor_wrap_int(ctx, torch.from_numpy(vals).cuda())
    blind = [int(v) for v in rng.integers(0, 2 ** 62, rows)]
    blind[5] = 0                                                    # ... and no blinding: the identity
    got = {}
    for wbits in (8, 12):
        ctx.set_commit_window_bits(wbits)
        try:
            key = lib.CommitKey(ctx, b"sparse", cols, 64 if dtype == "i64" else 32)
        finally:
            ctx.set_commit_window_bits(0)
        got[wbits] = lib.hyrax_commit(ctx, key, x, blind)
        key.close()
    assert got[8] == got[12]
    assert got[12][5] == bytes(96)
    gens, h = EC.generators(b"sparse", cols)
    for j in (0, 5, rows - 1):
        row = [int(v) for v in vals[j * cols:(j + 1) * cols]]
        assert EC.point_to_bytes(EC.commit(row, blind[j], gens, h)) == got[12][j]


def test_full_size_weight_stack_rows_and_opening(lib, ctx):
    """The weight stack of the 8 x 1024^2 window (2^23 int32, 4096 rows of 2048 columns; the key takes 12-bit
    windows, 2.4 GB of tables): two rows recomputed by the oracle from the definition, all 4096 commitments the
    same from a key with 8-bit windows, and the opening at a random point accepted by the library's verifier."""
    import torch
    from workloads import fcnn_window, CONFIG_SEED
    say("hyrax_commit on the 2^23 weight stack")
    wit = fcnn_window(CONFIG_SEED + 3, n_layers=8, width=1024, batch=64, steps=1)
    vals = np.ascontiguousarray(wit["W"]).reshape(-1)
    rows, cols = EC.matrix_shape(vals.size)
    assert (rows, cols) == (4096, 2048)
    rng = np.random.default_rng(13)
    blind = [int.from_bytes(rng.bytes(31), "little") for _ in range(rows)]
    x = lib.tensor_wrap_int(ctx, torch.from_numpy(vals).cuda())
    key = lib.CommitKey(ctx, b"W", cols)
    raw = lib.hyrax_commit(ctx, key, x, blind)
    ctx.set_commit_window_bits(8)
    try:
        key8 = lib.CommitKey(ctx, b"W", cols)
    finally:
        ctx.set_commit_window_bits(0)
    assert lib.hyrax_commit(ctx, key8, x, blind) == raw
    key8.close()
    say("  oracle: 2048 generators and two rows from the definition")
    gens, h = EC.generators(b"W", cols)
    for j in (0, rows - 3):
        row = [int(v) for v in vals[j * cols:(j + 1) * cols]]
        assert EC.point_to_bytes(EC.commit(row, blind[j], gens, h)) == raw[j]
    point = [int.from_bytes(rng.bytes(31), "little") for _ in range(23)]
    t, rho_star, y = lib.hyrax_open(ctx, x, blind, point)
    assert lib.hyrax_verify(ctx, key, raw, point, t, rho_star, y)[0] == 0
    assert lib.hyrax_verify(ctx, key, raw, point, t, rho_star, (y + 1) % R_MOD)[0] == 3
    key.close()


def test_claims_of_a_chained_window_open_against_the_commitments(lib, ctx):
    """Protocol zkdl end to end on one small window: the stacks A and W are committed, the chained window is
    proved, and the one claim it leaves on each of them is what the commitment opens to at the claim's point
    (proof of evaluation made and verified by the library, and by the oracle's verifier)."""
    import torch
    from workloads import fcnn_window, CONFIG_SEED
    say("commit -> prove -> open -> verify on a window")
    wit = fcnn_window(CONFIG_SEED + 140, n_layers=2, width=8, batch=4, steps=2)
    dw = {k: wit[k] for k in ("L", "B", "width", "T", "Q", "R")}
    for k in ("A", "W", "GZ", "Zr", "GA"):
        dw[k] = torch.from_numpy(np.ascontiguousarray(wit[k])).cuda()
    rng = np.random.default_rng(21)
    committed = {}
    for nm in ("A", "W"):
        flat = dw[nm].reshape(-1)
        rows, cols = EC.matrix_shape(flat.numel())
        key = lib.CommitKey(ctx, nm.encode(), cols)
        blind = [int.from_bytes(rng.bytes(31), "little") for _ in range(rows)]
        x = lib.tensor_wrap_int(ctx, flat)
        committed[nm] = (key, x, blind, lib.hyrax_commit(ctx, key, x, blind), cols)
    # the commitments go into the transcript before anything is drawn (Protocol zkdl: the prover commits first)
    tr = lib.Transcript(77)
    ots = OracleTranscript(77)
    for nm in ("A", "W"):
        tr.absorb(b"commit", b"".join(committed[nm][3]))
        ots.absorb(b"commit", b"".join(committed[nm][3]))
    got = lib.aggregate_prove(ctx, dw, tr, linked=True)
    from oracle import protocols as P
    P.aggregate_linked_verify(got["proof"], ots)             # the oracle's verifier on the same bound transcript
    assert ots.digest() == tr.digest()
    left = {c["tensor"]: c for c in got["claims_left"]}
    for nm in ("A", "W"):
        key, x, blind, coms, cols = committed[nm]
        claim = left[nm]
        t, rho_star, y = lib.hyrax_open(ctx, x, blind, claim["point"])
        assert y == claim["value"]
        assert lib.hyrax_verify(ctx, key, coms, claim["point"], t, rho_star, claim["value"])[0] == 0
        gens, h = EC.generators(nm.encode(), cols)
        assert EC.verify_opening([EC.point_from_bytes(c) for c in coms], claim["point"], t, rho_star, claim["value"], gens, h)
        assert lib.hyrax_verify(ctx, key, coms, claim["point"], t, rho_star, (claim["value"] + 1) % R_MOD)[0] == 3


def test_commitments_are_homomorphic(lib, ctx):
    """Sec. 2.3: the product of two commitments commits to the sum of the tensors."""
    import torch
    say("homomorphism")
    rng = np.random.default_rng(5)
    a = rng.integers(-2 ** 30, 2 ** 30, 32, dtype=np.int64).astype(np.int32)
    b = rng.integers(-2 ** 30, 2 ** 30, 32, dtype=np.int64).astype(np.int32)
    key = lib.CommitKey(ctx, b"hom", 4)
    ra, rb = [int(v) for v in rng.integers(1, 2 ** 60, 8)], [int(v) for v in rng.integers(1, 2 ** 60, 8)]
    ca = lib.hyrax_commit(ctx, key, lib.tensor_wrap_int(ctx, torch.from_numpy(a).cuda()), ra)
    cb = lib.hyrax_commit(ctx, key, lib.tensor_wrap_int(ctx, torch.from_numpy(b).cuda()), rb)
    cs = lib.hyrax_commit(ctx, key, lib.tensor_wrap_int(ctx, torch.from_numpy(a + b).cuda()), [x + y for x, y in zip(ra, rb)])
    for u, v, w in zip(ca, cb, cs):
        assert EC.add(EC.point_from_bytes(u), EC.point_from_bytes(v)) == EC.point_from_bytes(w)


def test_commit_rejects_bad_arguments(lib, ctx):
    import torch
    key = lib.CommitKey(ctx, b"args", 4)
    x64 = lib.tensor_wrap_int(ctx, torch.zeros(16, dtype=torch.int64).cuda())
    with pytest.raises(lib.ZkdlError):
        lib.hyrax_commit(ctx, key, x64)                      # a 32-bit key
    big = lib.tensor_wrap_int(ctx, torch.zeros(1024, dtype=torch.int32).cuda())
    with pytest.raises(lib.ZkdlError):
        lib.hyrax_commit(ctx, key, big)                      # 32 columns, the key has 4
    x = lib.tensor_wrap_int(ctx, torch.zeros(16, dtype=torch.int32).cuda())
    with pytest.raises(lib.ZkdlError):
        lib.hyrax_commit(ctx, key, x, [R_MOD] * 4)           # blinding not below r
    with pytest.raises(lib.ZkdlError):
        lib.CommitKey(ctx, b"x" * 17, 4)
    with pytest.raises(lib.ZkdlError):
        lib.CommitKey(ctx, b"x", 3)
    with pytest.raises(lib.ZkdlError):
        ctx.set_commit_window_bits(10)


def test_full_size_activation_stack_opens_correctly(lib, ctx):
    """The activation stack of the 8 x 1024^2, batch-64 window (2^19 int32, 1024 rows of 512 columns): the
    oracle cannot recompute 2^19 scalar multiplications in seconds, so the commitments are checked through
    the relation that holds at any size - the oracle's verifier combines the 1024 row commitments at a random
    point (the homomorphism of Sec. 2.3) and accepts the library's opening - and 16 sampled rows are
    recomputed from their definition."""
    import torch
    from workloads import fcnn_window, CONFIG_SEED
    say("hyrax_commit on the 2^19 activation stack")
    wit = fcnn_window(CONFIG_SEED + 3, n_layers=8, width=1024, batch=64, steps=1)
    vals = np.ascontiguousarray(wit["A"]).reshape(-1)
    rows, cols = EC.matrix_shape(vals.size)
    rng = np.random.default_rng(11)
    blind = [int.from_bytes(rng.bytes(31), "little") for _ in range(rows)]
    key = lib.CommitKey(ctx, b"A", cols)
    x = lib.tensor_wrap_int(ctx, torch.from_numpy(vals).cuda())
    raw = lib.hyrax_commit(ctx, key, x, blind)
    coms = [EC.point_from_bytes(c) for c in raw]
    gens = [EC.point_from_bytes(g) for g in key.generators(0, cols)]
    h = EC.point_from_bytes(key.generators(cols, 1)[0])
    for i in (0, 1, cols - 1):
        assert gens[i] == EC.generator(b"A", i)
    assert h == EC.generator(b"A", EC.H_INDEX)
    point = [int.from_bytes(rng.bytes(31), "little") for _ in range(19)]
    t, rho_star, y = lib.hyrax_open(ctx, x, blind, point)
    say("  oracle: verifying the opening")
    assert EC.verify_opening(coms, point, t, rho_star, y, gens, h)
    say("  oracle: sampled rows")
    for j in (0, 5, rows - 1):
        row = [int(v) for v in vals[j * cols:(j + 1) * cols]]
        assert EC.commit(row, blind[j], gens, h) == coms[j]
