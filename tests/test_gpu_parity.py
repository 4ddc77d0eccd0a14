"""GPU parity: the HIP library against the CPU oracle, through the C ABI.

Bit-exact on every proof byte, challenge, claim and the final transcript state.
"""
import sys

import numpy as np
import pytest

from oracle.field import R_MOD, fr_array, fr_array_from_le, array_to_le
from oracle.mle import partial_eval, mle_eval as P_mle_eval
from oracle import protocols as P
from oracle.transcript import Transcript as OracleTranscript
from workloads import uniform_fr_limbs, fcnn_window, fc_relu_layer, CONFIG_SEED

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def rand_fr_bytes(seed, n):
    return uniform_fr_limbs(np.random.default_rng(seed), n).tobytes()


@pytest.mark.parametrize("dtype", ["i32", "i64", "fr"])
def test_upload_download_roundtrip(lib, ctx, dtype):
    say(f"upload/download {dtype}")
    rng = np.random.default_rng(3)
    n = 1 << 10
    if dtype == "i32":
        src = rng.integers(-2 ** 31, 2 ** 31, n, dtype=np.int64).astype(np.int32)
        src[:4] = [0, -1, 2 ** 31 - 1, -2 ** 31]
        expect = fr_array(src)
    elif dtype == "i64":
        src = rng.integers(-2 ** 63, 2 ** 63, n, dtype=np.int64)
        src[:4] = [0, -1, 2 ** 63 - 1, -2 ** 63]
        expect = fr_array(src)
    else:
        limbs = uniform_fr_limbs(rng, n)
        limbs[0] = 0
        limbs[1] = [0xFFFFFFFF00000000, 0x53BDA402FFFE5BFE, 0x3339D80809A1D805, 0x73EDA753299D7D48]  # r - 1
        src = limbs.tobytes()
        expect = fr_array_from_le(src, n)
    t = lib.fr_tensor_upload(ctx, src, (n,))
    assert t.shape == (n,)
    assert t.download() == array_to_le(expect)


def test_upload_from_device_memory(lib, ctx):
    import torch
    say("upload from device")
    src = np.random.default_rng(4).integers(-2 ** 31, 2 ** 31, 4096, dtype=np.int64).astype(np.int32)
    t = lib.fr_tensor_upload(ctx, torch.from_numpy(src).cuda(), (64, 64))
    assert t.download() == array_to_le(fr_array(src))
    w = lib.tensor_wrap_int(ctx, torch.from_numpy(src).cuda().reshape(64, 64))
    assert w.download() == array_to_le(fr_array(src))


PE_CASES = [
    ((8, 16, 32), 0, 1, "fr"), ((8, 16, 32), 1, 2, "fr"), ((8, 16, 32), 2, 3, "fr"),
    ((8, 16, 32), 0, 3, "fr"), ((8, 16, 32), 1, 3, "i32"), ((4, 64, 2), 1, 2, "i64"),
    ((1, 1, 1), 0, 3, "fr"), ((2048, 64), 0, 1, "fr"), ((64, 4096), 1, 2, "i32"),
    ((16384,), 0, 1, "fr"), ((2, 8192, 2), 1, 2, "i32"),
]


@pytest.mark.parametrize("shape,lo,hi,kind", PE_CASES)
def test_mle_partial_eval(lib, ctx, shape, lo, hi, kind):
    say(f"partial_eval shape={shape} axes=[{lo},{hi}) {kind}")
    rng = np.random.default_rng(hash((shape, lo, hi)) % 2 ** 32)
    n = int(np.prod(shape))
    if kind == "fr":
        raw = uniform_fr_limbs(rng, n).tobytes()
        ref = fr_array_from_le(raw, n)
        t = lib.fr_tensor_upload(ctx, raw, shape)
    elif kind == "i32":
        import torch
        src = rng.integers(-2 ** 31, 2 ** 31, n, dtype=np.int64).astype(np.int32)
        ref = fr_array(src)
        t = lib.tensor_wrap_int(ctx, torch.from_numpy(src).cuda(), shape)
    else:
        import torch
        src = rng.integers(-2 ** 47, 2 ** 47, n, dtype=np.int64)
        ref = fr_array(src)
        t = lib.tensor_wrap_int(ctx, torch.from_numpy(src).cuda(), shape)
    npt = sum(int(s).bit_length() - 1 for s in shape[lo:hi])
    point = fr_array_from_le(rand_fr_bytes(99, max(npt, 1)), max(npt, 1)).tolist()[:npt]
    out = lib.mle_partial_eval(ctx, t, lo, hi, point)
    expect, oshape = partial_eval(ref, shape, lo, hi, point)
    assert list(out.shape) == oshape
    assert out.download() == array_to_le(expect)


@pytest.mark.parametrize("k,d", [(3, 0), (3, 1), (3, 2), (1, 5), (2, 9), (3, 10), (1, 11), (2, 12), (3, 14)])
def test_sumcheck_product(lib, ctx, k, d):
    say(f"sumcheck_product K={k} d={d}")
    n = 1 << d
    raws = [rand_fr_bytes(1000 + 10 * d + j, n) for j in range(k)]
    tabs = [lib.fr_tensor_upload(ctx, r, (n,)) for r in raws]
    tr = lib.Transcript(77)
    got = lib.sumcheck_product(ctx, tabs, tr)
    ots = OracleTranscript(77)
    buf, proof, vs = P.product_prove([fr_array_from_le(r, n) for r in raws], ots)
    assert got["proof"] == buf
    assert got["points"] == ots.challenges
    assert got["claims"] == proof.finals
    assert tr.digest() == ots.digest()
    # inputs are untouched
    assert tabs[0].download() == raws[0]


@pytest.mark.parametrize("n,d1,d2,d3,t0,t1,kind", [
    (1, 16, 256, 256, False, False, "i32"),      # one FC layer, batch 16 (config 1 shape)
    (4, 8, 32, 16, False, False, "fr"),
    (4, 8, 32, 16, True, False, "i32"),
    (4, 8, 32, 16, False, True, "i32"),
    (2, 1, 2, 1, False, False, "fr"),
    (8, 4, 64, 64, True, True, "i32"),
])
def test_sumcheck_matmul(lib, ctx, n, d1, d2, d3, t0, t1, kind):
    import torch
    say(f"sumcheck_matmul N={n} D=({d1},{d2},{d3}) tr=({t0},{t1}) {kind}")
    rng = np.random.default_rng(n * 1000 + d1 + d2 + d3)
    x0 = rng.integers(-2 ** 31, 2 ** 31, (n, d1, d2), dtype=np.int64).astype(np.int32)
    x1 = rng.integers(-2 ** 31, 2 ** 31, (n, d2, d3), dtype=np.int64).astype(np.int32)
    s0 = np.ascontiguousarray(np.transpose(x0, (0, 2, 1))) if t0 else x0     # what is stored
    s1 = np.ascontiguousarray(np.transpose(x1, (0, 2, 1))) if t1 else x1
    if kind == "i32":
        a = lib.tensor_wrap_int(ctx, torch.from_numpy(s0).cuda())
        b = lib.tensor_wrap_int(ctx, torch.from_numpy(s1).cuda())
    else:
        a = lib.fr_tensor_upload(ctx, s0, s0.shape)
        b = lib.fr_tensor_upload(ctx, s1, s1.shape)
    tr = lib.Transcript(5)
    got = lib.sumcheck_matmul(ctx, a, b, tr, t0, t1)
    ots = OracleTranscript(5)
    buf, proof, pts = P.matmul_prove(fr_array(x0), [n, d1, d2], fr_array(x1), [n, d2, d3], ots)
    assert got["proof"] == buf
    assert got["points"] == ots.challenges
    assert got["claims"] == [proof.claim0, proof.finals[1], proof.finals[2]]
    assert tr.digest() == ots.digest()


@pytest.mark.parametrize("n,d1,d2,d3,t0,t1,kind", [
    (1, 16, 256, 256, False, False, "i32"),      # no stack rounds: the single-product sumcheck alone
    (1, 2, 1, 2, False, False, "fr"),            # neither stack nor product rounds
    (4, 2, 1, 2, False, False, "i32"),           # stack rounds only (D2 = 1)
    (2, 4, 1, 2, False, False, "fr"),
    (2, 1, 2, 1, False, False, "fr"),
    (4, 8, 32, 16, False, False, "fr"),
    (4, 8, 32, 16, True, False, "i32"),
    (4, 8, 32, 16, False, True, "i32"),
    (8, 4, 64, 64, True, True, "i32"),
    (16, 2, 1024, 2, False, False, "i32"),       # 14 rounds: the single-block tail takes the last ten
    (128, 2, 16, 2, False, False, "i32"),        # seven stack rounds
])
def test_sumcheck_matmul_ft(lib, ctx, n, d1, d2, d3, t0, t1, kind):
    """The optimized aggregated protocol (stack rounds with f_t, then the single-product
    sumcheck): proof bytes, challenges, claims and transcript against the oracle."""
    import torch
    say(f"sumcheck_matmul_ft N={n} D=({d1},{d2},{d3}) tr=({t0},{t1}) {kind}")
    rng = np.random.default_rng(n * 1000 + d1 + d2 + d3 + 1)
    x0 = rng.integers(-2 ** 31, 2 ** 31, (n, d1, d2), dtype=np.int64).astype(np.int32)
    x1 = rng.integers(-2 ** 31, 2 ** 31, (n, d2, d3), dtype=np.int64).astype(np.int32)
    s0 = np.ascontiguousarray(np.transpose(x0, (0, 2, 1))) if t0 else x0     # what is stored
    s1 = np.ascontiguousarray(np.transpose(x1, (0, 2, 1))) if t1 else x1
    if kind == "i32":
        a = lib.tensor_wrap_int(ctx, torch.from_numpy(s0).cuda())
        b = lib.tensor_wrap_int(ctx, torch.from_numpy(s1).cuda())
    else:
        a = lib.fr_tensor_upload(ctx, s0, s0.shape)
        b = lib.fr_tensor_upload(ctx, s1, s1.shape)
    tr = lib.Transcript(6)
    got = lib.sumcheck_matmul_ft(ctx, a, b, tr, t0, t1)
    ots = OracleTranscript(6)
    buf, info = P.matmul_ft_prove(fr_array(x0), [n, d1, d2], fr_array(x1), [n, d2, d3], ots)
    assert got["proof"] == buf
    assert got["points"] == ots.challenges
    assert got["claims"] == [info["claim0"]] + info["inner"].finals
    assert tr.digest() == ots.digest()
    P.matmul_ft_verify(got["proof"], n, d1, d2, d3, OracleTranscript(6))


@pytest.mark.gpu
@pytest.mark.parametrize("n,d1,d2,d3,kind", [
    (2, 2, 4, 2, "fr"),
    (1, 1, 1, 1, "fr"),            # no round at all: header, claim_0 = 0, the finals
    (1, 4, 8, 2, "int"),           # no stack rounds: claim_0 = 0
    (4, 1, 8, 4, "fr"),            # no rounds over i0
    (4, 8, 4, 1, "int"),           # no rounds over i1
    (4, 4, 1, 2, "int"),           # no rounds over j
    (8, 16, 32, 8, "int"),
    (16, 4, 64, 16, "fr"),
    (64, 8, 8, 8, "int"),          # six stack rounds
    (2, 2, 1024, 2, "int"),        # tables of the j rounds longer than a block
    (8, 32, 32, 16, "int"),        # 2^17 terms: several blocks in the stack rounds, every phase longer than a wave
    (16, 64, 64, 32, "int"),       # 2^21 terms
])
def test_sumcheck_matmul_general(lib, ctx, n, d1, d2, d3, kind):
    """The general aggregated form on the three stacks: proof bytes, challenges, finals and transcript
    against the oracle, whose verifier also accepts the library's proof."""
    import torch
    say(f"sumcheck_matmul_general N={n} D=({d1},{d2},{d3}) {kind}")
    rng = np.random.default_rng(n * 1000 + d1 * 100 + d2 * 10 + d3)
    x0 = rng.integers(-2 ** 15, 2 ** 15, (n, d1, d2), dtype=np.int64)
    x1 = rng.integers(-2 ** 15, 2 ** 15, (n, d2, d3), dtype=np.int64)
    y = np.einsum("nij,njk->nik", x0, x1)
    if kind == "int":
        a = lib.tensor_wrap_int(ctx, torch.from_numpy(x0.astype(np.int32)).cuda())
        b = lib.tensor_wrap_int(ctx, torch.from_numpy(x1.astype(np.int32)).cuda())
        c = lib.tensor_wrap_int(ctx, torch.from_numpy(y).cuda())
    else:
        a = lib.fr_tensor_upload(ctx, x0, x0.shape)
        b = lib.fr_tensor_upload(ctx, x1, x1.shape)
        c = lib.fr_tensor_upload(ctx, y, y.shape)
    tr = lib.Transcript(8)
    got = lib.sumcheck_matmul_general(ctx, a, b, c, tr)
    ots = OracleTranscript(8)
    buf, info = P.matmul_general_prove(fr_array(x0), [n, d1, d2], fr_array(x1), [n, d2, d3], fr_array(y), ots)
    assert got["proof"] == buf
    assert got["points"] == ots.challenges
    assert got["claims"] == info["inner"].finals
    assert tr.digest() == ots.digest()
    finals, _ = P.matmul_general_verify(got["proof"], n, d1, d2, d3, OracleTranscript(8))
    assert finals == got["claims"]
    tv = lib.Transcript(8)
    ver = lib.aggregate_verify(ctx, got["proof"], tv)                 # the library's verifier, on the GPU
    assert ver["verdict"] == 0 and ver["points"] == ots.challenges and tv.digest() == ots.digest()


@pytest.mark.gpu
def test_sumcheck_matmul_general_wrong_product_is_rejected(lib, ctx):
    """The prover does not check Y: with one entry of Y off by one the proof it writes fails the
    oracle's verifier."""
    say("sumcheck_matmul_general with a wrong Y")
    n, d1, d2, d3 = 4, 4, 8, 2
    rng = np.random.default_rng(77)
    x0 = rng.integers(-2 ** 15, 2 ** 15, (n, d1, d2), dtype=np.int64)
    x1 = rng.integers(-2 ** 15, 2 ** 15, (n, d2, d3), dtype=np.int64)
    y = np.einsum("nij,njk->nik", x0, x1)
    y[2, 1, 1] += 1
    a, b, c = [lib.fr_tensor_upload(ctx, t, t.shape) for t in (x0, x1, y)]
    got = lib.sumcheck_matmul_general(ctx, a, b, c, lib.Transcript(8))
    with pytest.raises(AssertionError):
        P.matmul_general_verify(got["proof"], n, d1, d2, d3, OracleTranscript(8))
    assert lib.aggregate_verify(ctx, got["proof"], lib.Transcript(8))["verdict"] != 0


@pytest.mark.gpu
def test_sumcheck_matmul_general_rejects_bad_shapes(lib, ctx):
    say("sumcheck_matmul_general argument checks")
    z = lambda *sh: lib.fr_tensor_upload(ctx, np.zeros(sh, dtype=np.int64), sh)
    for sh0, sh1, shy in [((2, 2, 4), (2, 2, 2), (2, 2, 2)), ((2, 2, 4), (4, 4, 2), (2, 2, 2)),
                          ((2, 2, 4), (2, 4, 2), (2, 2, 4)), ((2, 2, 4), (2, 4, 2), (2, 4, 2))]:
        tr = lib.Transcript(1)
        before = tr.digest()
        with pytest.raises(lib.ZkdlError):
            lib.sumcheck_matmul_general(ctx, z(*sh0), z(*sh1), z(*shy), tr)
        assert tr.digest() == before


def _reindex_maps(case, n):
    rng = np.random.default_rng(99)
    if case == "layers":          # inputs of the layers / their outputs: a shift by one tensor
        return [list(range(0, n // 2)), list(range(1, n // 2 + 1))]
    if case == "shift_pad":
        return [list(range(n)), list(range(1, n)) + [-1]]
    if case == "single":
        return [[0]]
    if case == "swap":
        return [[1, 0], [0, -1]]
    if case == "repeat":
        return [[7, 6, 5, 4, 3, 2, 1, 0], [2, 5], [0, 0, 3, -1]]
    # "random8": eight maps of mixed lengths with repeats and padding
    maps = []
    for k in range(8):
        m = rng.integers(-1, n, max(n >> k, 1))
        maps.append([int(v) for v in m])
    return maps


@pytest.mark.parametrize("n,d,case,kind", [
    (4, 8, "shift_pad", "i32"),
    (8, 4, "repeat", "fr"),
    (1, 2, "single", "fr"),
    (2, 1, "swap", "i64"),
    (32, 4096, "layers", "i32"),
    (4096, 64, "random8", "i32"),      # 12 rounds over the stack: two grid rounds, then the single-block tail
])
def test_reindex_prove(lib, ctx, n, d, case, kind):
    """Re-indexing sumcheck (Eq. sc-reindex): proof bytes, challenges, claims and transcript
    against the oracle; the oracle's verifier accepts the library's proof."""
    import torch
    say(f"reindex_prove N={n} D={d} {case} {kind}")
    rng = np.random.default_rng(n * 7 + d)
    maps = _reindex_maps(case, n)
    if kind == "fr":
        raw = uniform_fr_limbs(rng, n * d).tobytes()
        x = lib.fr_tensor_upload(ctx, raw, (n, d))
        fx = fr_array_from_le(raw, n * d)
    elif kind == "i32":
        xi = rng.integers(-2 ** 31, 2 ** 31, (n, d), dtype=np.int64).astype(np.int32)
        x = lib.tensor_wrap_int(ctx, torch.from_numpy(xi).cuda())
        fx = fr_array(xi)
    else:
        xi = rng.integers(-2 ** 63, 2 ** 63, (n, d), dtype=np.int64)
        x = lib.fr_tensor_upload(ctx, xi, (n, d))
        fx = fr_array(xi)
    points = [[int(v) for v in fr_array_from_le(rand_fr_bytes(300 + k, 32), 32)[:len(m).bit_length() - 1]]
              for k, m in enumerate(maps)]
    u = [int(v) for v in fr_array_from_le(rand_fr_bytes(299, 40), 40)[:d.bit_length() - 1]]
    tr = lib.Transcript(12)
    got = lib.reindex_prove(ctx, x, maps, points, u, tr)
    ots = OracleTranscript(12)
    buf, info = P.reindex_prove(fx, n, d, maps, points, u, ots)
    assert got["proof"] == buf
    assert got["points"] == ots.challenges
    assert got["claims"] == info["claims"] + info["inner"].finals
    assert tr.digest() == ots.digest()
    claims, vs, xw = P.reindex_verify(got["proof"], n, d, maps, points, u, OracleTranscript(12))
    assert xw == got["claims"][-1]


@pytest.mark.parametrize("shape,k,kind", [((8,), 2, "fr"), ((1,), 2, "fr"), ((4, 64), 3, "i32"), ((2, 8, 16), 1, "i64"),
                                          ((16, 4096), 2, "i32"), ((2, 1024, 1024), 2, "i32"), ((3000 // 3000 * 4096,), 8, "fr")])
def test_claims_merge(lib, ctx, shape, k, kind):
    """K claims on one tensor become one: proof bytes, claims, challenges and transcript agree."""
    import torch
    n = int(np.prod(shape))
    d = n.bit_length() - 1
    say(f"claims_merge shape={shape} K={k} {kind}")
    rng = np.random.default_rng(n + k)
    pts = [fr_array_from_le(rand_fr_bytes(70 + j, d), d).tolist() if d else [] for j in range(k)]
    if kind == "fr":
        raw = rand_fr_bytes(n + 1, n)
        x = lib.fr_tensor_upload(ctx, raw, shape)
        xo = fr_array_from_le(raw, n)
    else:
        dt = np.int32 if kind == "i32" else np.int64
        vals = rng.integers(-2 ** 31, 2 ** 31, n).astype(dt)
        x = lib.tensor_wrap_int(ctx, torch.from_numpy(vals).cuda(), shape)
        xo = None
    tr = lib.Transcript(35)
    got = lib.claims_merge_prove(ctx, x, pts, tr)
    if n <= 1 << 16:
        if xo is None:
            xo = fr_array(vals)
        ots = OracleTranscript(35)
        buf, info = P.merge_prove(xo, pts, ots)
        assert got["proof"] == buf
        assert got["points"] == ots.challenges
        assert got["claims"][:k] == info["claims"] and got["claims"][k + 1] == info["inner"].finals[1]
        assert tr.digest() == ots.digest()
    else:
        # too large for the oracle's prover: its verifier replays the proof, and the claims are
        # evaluated from the integers one stack slot at a time
        ots = OracleTranscript(35)
        claims, vs, left = P.merge_verify(got["proof"], d, pts, ots)
        assert tr.digest() == ots.digest() and got["points"] == ots.challenges
        st = vals.reshape(shape)
        for c, pt in zip(claims + [left], pts + [vs]):
            assert c == _stack_mle(st, pt[:1], pt[1:11], pt[11:])


@pytest.mark.parametrize("shape,k,kind", [((4, 8), 2, "fr"), ((1, 8), 2, "i32"), ((8, 1), 2, "i64"), ((2, 2), 5, "fr"),
                                          ((4, 8, 16), 3, "i32"), ((16, 64, 32), 1, "i32"), ((2, 1, 2048), 2, "fr"),
                                          ((8, 1024, 1024), 2, "i32")])
def test_claims_merge_stack(lib, ctx, shape, k, kind):
    """The merge on tables of the inner size: proof bytes, claims, challenges and transcript agree."""
    import torch
    n = int(np.prod(shape))
    d = n.bit_length() - 1
    say(f"claims_merge_stack shape={shape} K={k} {kind}")
    rng = np.random.default_rng(n + 3 * k)
    pts = [fr_array_from_le(rand_fr_bytes(90 + j, d), d).tolist() for j in range(k)]
    if kind == "fr":
        raw = rand_fr_bytes(n + 2, n)
        x = lib.fr_tensor_upload(ctx, raw, shape)
        xo = fr_array_from_le(raw, n)
    else:
        dt = np.int32 if kind == "i32" else np.int64
        vals = rng.integers(-2 ** 31, 2 ** 31, n).astype(dt)
        x = lib.tensor_wrap_int(ctx, torch.from_numpy(vals).cuda(), shape)
        xo = None
    tr = lib.Transcript(36)
    got = lib.claims_merge_prove(ctx, x, pts, tr, stack=True)
    ots = OracleTranscript(36)
    if n <= 1 << 15:
        if xo is None:
            xo = fr_array(vals)
        buf, info = P.stack_merge_prove(xo, shape[0], n // shape[0], pts, ots)
        assert got["proof"] == buf
        assert got["points"] == ots.challenges
        assert got["claims"][:k] == info["claims"] and got["claims"][k + 1] == info["outer"].finals[1]
        assert tr.digest() == ots.digest()
    else:
        claims, point, left = P.stack_merge_verify(got["proof"], shape[0], n // shape[0], pts, ots)
        assert tr.digest() == ots.digest() and got["points"] == ots.challenges
        st = vals.reshape(shape)
        for c, pt in zip(claims + [left], pts + [point]):
            assert c == _stack_mle(st, pt[:3], pt[3:13], pt[13:])


def test_claims_merge_rejects_bad_arguments(lib, ctx):
    say("claims_merge bad arguments")
    x = lib.fr_tensor_upload(ctx, rand_fr_bytes(1, 8), (8,))
    tr = lib.Transcript(1)
    before = tr.digest()
    for pts in ([[0, 0, R_MOD]], [[0, 0, 0]] * 9, []):
        with pytest.raises(lib.ZkdlError):
            lib.claims_merge_prove(ctx, x, pts, tr)
    assert tr.digest() == before


def test_reindex_prove_rejects_bad_arguments(lib, ctx):
    say("reindex_prove argument checks")
    x = lib.fr_tensor_upload(ctx, np.arange(8, dtype=np.int64), (4, 2))
    tr = lib.Transcript(1)
    before = tr.digest()
    for maps, points in (([[0, 4]], [[5]]),              # index beyond the stack
                         ([[0, -2]], [[5]]),             # below -1
                         ([[0, 1, 2]], [[5, 6]]),        # length no power of two
                         ([[0]] * 9, [[]] * 9)):         # too many sub-stacks
        with pytest.raises(lib.ZkdlError):
            lib.reindex_prove(ctx, x, maps, points, [3], tr)
    assert tr.digest() == before


@pytest.mark.parametrize("shape", [(1,), (2, 4, 4), (4, 64, 16), (2, 64, 64), (16384,), (8, 64, 64), (32, 64, 64)])
def test_sumcheck_hadamard(lib, ctx, shape):
    say(f"sumcheck_hadamard shape={shape}")
    rng = np.random.default_rng(17)
    x0 = rng.integers(-2 ** 31, 2 ** 31, shape, dtype=np.int64).astype(np.int32)
    x1 = rng.integers(-2 ** 31, 2 ** 31, shape, dtype=np.int64).astype(np.int32)
    a = lib.fr_tensor_upload(ctx, x0, shape)
    b = lib.fr_tensor_upload(ctx, x1, shape)
    tr = lib.Transcript(6)
    got = lib.sumcheck_hadamard(ctx, a, b, tr)
    ots = OracleTranscript(6)
    buf, proof, pts = P.hadamard_prove(fr_array(x0), fr_array(x1), ots)
    assert got["proof"] == buf and got["points"] == ots.challenges
    assert got["claims"] == [proof.claim0, proof.finals[1], proof.finals[2]]
    assert tr.digest() == ots.digest()


@pytest.mark.parametrize("shape,extreme", [((16384,), False), ((4, 64, 64), True), ((32, 64, 64), False), ((8192,), True)])
def test_sumcheck_hadamard_int32_sources(lib, ctx, shape, extreme):
    """int32 stacks wrapped in place: from 2^14 entries on the first two rounds read the integers
    (products of the lines below 2^68, one reduction per thread) instead of converted tables."""
    import torch
    say(f"sumcheck_hadamard int32 shape={shape} extreme={extreme}")
    rng = np.random.default_rng(23)
    x0 = rng.integers(-2 ** 31, 2 ** 31, shape, dtype=np.int64).astype(np.int32)
    x1 = rng.integers(-2 ** 31, 2 ** 31, shape, dtype=np.int64).astype(np.int32)
    if extreme:       # the widest lines: 2 a1 - a0 = +-3 * 2^31 and their products, all sign patterns
        n = x0.size
        f0, f1 = x0.reshape(-1), x1.reshape(-1)
        lo, hi = -2 ** 31, 2 ** 31 - 1
        for i, (a0, a1, c0, c1) in enumerate([(lo, hi, lo, hi), (hi, lo, lo, hi), (lo, hi, hi, lo), (hi, lo, hi, lo),
                                              (lo, lo, hi, hi), (0, lo, 0, lo), (hi, hi, hi, hi), (lo, lo, lo, lo)]):
            f0[i], f0[i + n // 2], f1[i], f1[i + n // 2] = a0, a1, c0, c1
            f0[n // 4 + i], f0[n // 4 + i + n // 2] = a1, a0      # the same in the pairs of round 1
            f1[n // 4 + i], f1[n // 4 + i + n // 2] = c1, c0
    a = lib.tensor_wrap_int(ctx, torch.from_numpy(x0).cuda(), shape)
    b = lib.tensor_wrap_int(ctx, torch.from_numpy(x1).cuda(), shape)
    tr = lib.Transcript(8)
    got = lib.sumcheck_hadamard(ctx, a, b, tr)
    ots = OracleTranscript(8)
    buf, proof, pts = P.hadamard_prove(fr_array(x0), fr_array(x1), ots)
    assert got["proof"] == buf and got["points"] == ots.challenges
    assert got["claims"] == [proof.claim0, proof.finals[1], proof.finals[2]]
    assert tr.digest() == ots.digest()


def test_sumcheck_hadamard_full_size_by_properties(lib, ctx):
    """Hadamard product of two stacks of 2^24 int32 values (the size of the micro-benchmark's
    tables): the oracle's verifier replays all 24 rounds and ends in the library's transcript
    state; the three claims are evaluated directly from the integers."""
    import torch
    say("sumcheck_hadamard 16 x 1024 x 1024")
    shape = (16, 1024, 1024)
    rng = np.random.default_rng(2024)
    x0 = rng.integers(-2 ** 31, 2 ** 31, shape, dtype=np.int64).astype(np.int32)
    x1 = rng.integers(-2 ** 31, 2 ** 31, shape, dtype=np.int64).astype(np.int32)
    a = lib.tensor_wrap_int(ctx, torch.from_numpy(x0).cuda(), shape)
    b = lib.tensor_wrap_int(ctx, torch.from_numpy(x1).cuda(), shape)
    tr = lib.Transcript(7)
    got = lib.sumcheck_hadamard(ctx, a, b, tr)
    ots = OracleTranscript(7)
    proof, pts = P.hadamard_verify(got["proof"], 24, ots)
    assert tr.digest() == ots.digest() and got["points"] == ots.challenges
    p, v = pts["p"], pts["v"]
    assert got["claims"] == [proof.claim0, proof.finals[1], proof.finals[2]]
    assert proof.finals[1] == _stack_mle(x0, v[:4], v[4:14], v[14:])
    assert proof.finals[2] == _stack_mle(x1, v[:4], v[4:14], v[14:])
    prod = x0.astype(np.int64) * x1.astype(np.int64)            # |.| < 2^62
    assert proof.claim0 == _stack_mle(prod, p[:4], p[4:14], p[14:])
    ctx.trim()


def test_too_small_buffers_leave_the_transcript_untouched(lib, ctx):
    """A call whose proof or points buffer is too small reports the sizes needed and changes nothing of
    the caller's: the same call with room then gives the proof the oracle gives on that transcript."""
    import ctypes as C
    say("ZKDL_ESMALL leaves the transcript as it was")
    n, k = 1 << 6, 2
    raws = [rand_fr_bytes(4000 + j, n) for j in range(k)]
    tabs = [lib.fr_tensor_upload(ctx, r, (n,)) for r in raws]
    arr = (C.c_void_p * k)(*[t.handle for t in tabs])
    tr = lib.Transcript(5)
    before = tr.digest()
    raw = lib.load_library().sumcheck_product
    need = C.c_size_t(0)
    npts = C.c_size_t(0)
    # size query: proof == NULL
    rc = raw(ctx.handle, arr, k, tr.handle, None, C.byref(need), None, None, C.byref(npts))
    assert rc == -5 and need.value == 16 + 32 * (1 + 6 * 3 + 2) and npts.value == 6
    assert tr.digest() == before
    small = C.create_string_buffer(64)
    cap = C.c_size_t(64)
    rc = raw(ctx.handle, arr, k, tr.handle, small, C.byref(cap), None, None, None)
    assert rc == -5 and cap.value == need.value and tr.digest() == before
    pts = C.create_string_buffer(32 * 2)
    proof = C.create_string_buffer(need.value)
    cap, npts = C.c_size_t(need.value), C.c_size_t(2)
    rc = raw(ctx.handle, arr, k, tr.handle, proof, C.byref(cap), None, pts, C.byref(npts))
    assert rc == -5 and npts.value == 6 and tr.digest() == before
    got = lib.sumcheck_product(ctx, tabs, tr)
    ots = OracleTranscript(5)
    buf, _, _ = P.product_prove([fr_array_from_le(r, n) for r in raws], ots)
    assert got["proof"] == buf and tr.digest() == ots.digest()
    # claims without a proof buffer: sumcheck_matmul still reports Y~(w, u0, u1)
    import torch
    rng = np.random.default_rng(6)
    x0 = rng.integers(-100, 100, (2, 4, 8)).astype(np.int32)
    x1 = rng.integers(-100, 100, (2, 8, 4)).astype(np.int32)
    t0 = lib.tensor_wrap_int(ctx, torch.from_numpy(x0).cuda())
    t1 = lib.tensor_wrap_int(ctx, torch.from_numpy(x1).cuda())
    claims = C.create_string_buffer(96)
    tr2 = lib.Transcript(7)
    rc = lib.load_library().sumcheck_matmul(ctx.handle, t0.handle, t1.handle, 0, 0, tr2.handle, None, None, claims, None, None)
    assert rc == 0
    ots = OracleTranscript(7)
    _, proof_o, _ = P.matmul_prove(fr_array(x0), [2, 4, 8], fr_array(x1), [2, 8, 4], ots)
    assert [int.from_bytes(claims.raw[32 * j:32 * j + 32], "little") for j in range(3)] == \
        [proof_o.claim0, proof_o.finals[1], proof_o.finals[2]]
    assert tr2.digest() == ots.digest()


def test_too_small_buffers_in_the_widened_calls(lib, ctx):
    """update_prove and sumcheck_matmul_general: the size query and a short claims list change nothing."""
    import ctypes as C
    say("ZKDL_ESMALL in update_prove and sumcheck_matmul_general")
    g = _update_gradients(5, 8, 6, 4)
    raw = lib.load_library().update_prove
    tr = lib.Transcript(3)
    before = tr.digest()
    need, npts = C.c_size_t(0), C.c_size_t(0)
    rc = raw(ctx.handle, g.ctypes.data, 8, 6, 4, 0, tr.handle, None, C.byref(need), None, C.byref(npts), None, None)
    assert rc == -5 and tr.digest() == before
    ots = OracleTranscript(3)
    buf, _ = P.update_prove([int(x) for x in g], 6, 4, ots)
    assert need.value == len(buf) and npts.value == len(ots.challenges) + 3 * 4     # three copied points of 1 + 3 coordinates
    claims = (lib.binding.Claim * 2)() if hasattr(lib, "binding") else None
    if claims is not None:
        ncl = C.c_size_t(2)
        pts = C.create_string_buffer(32 * 1024)
        npts = C.c_size_t(1024)
        rc = raw(ctx.handle, g.ctypes.data, 8, 6, 4, 0, tr.handle, None, None, pts, C.byref(npts), claims, C.byref(ncl))
        assert rc == -5 and ncl.value == 3 and tr.digest() == before
    got = lib.update_prove(ctx, g, tr, 6, 4)
    assert got["proof"] == buf and tr.digest() == ots.digest()
    # the general aggregated form
    x0 = np.arange(16, dtype=np.int64).reshape(2, 2, 4) - 5
    x1 = np.arange(16, dtype=np.int64).reshape(2, 4, 2) - 7
    y = np.einsum("nij,njk->nik", x0, x1)
    a, b, c = [lib.fr_tensor_upload(ctx, t, t.shape) for t in (x0, x1, y)]
    tr = lib.Transcript(4)
    before = tr.digest()
    need = C.c_size_t(0)
    rc = lib.load_library().sumcheck_matmul_general(ctx.handle, a.handle, b.handle, c.handle, tr.handle, None, C.byref(need),
                                                    None, None, None)
    ots = OracleTranscript(4)
    buf, _ = P.matmul_general_prove(fr_array(x0), [2, 2, 4], fr_array(x1), [2, 4, 2], fr_array(y), ots)
    assert rc == -5 and need.value == len(buf) and tr.digest() == before
    got = lib.sumcheck_matmul_general(ctx, a, b, c, tr)
    assert got["proof"] == buf and tr.digest() == ots.digest()


def test_chained_calls_share_one_transcript(lib, ctx):
    say("chained calls")
    n = 64
    raws = [rand_fr_bytes(50 + j, n) for j in range(2)]
    tabs = [lib.fr_tensor_upload(ctx, r, (n,)) for r in raws]
    tr = lib.Transcript(1)
    tr.absorb(b"digest", b"\x07" * 32)
    g1 = lib.sumcheck_product(ctx, tabs, tr)
    g2 = lib.sumcheck_product(ctx, tabs[:1], tr)
    ots = OracleTranscript(1)
    ots.absorb(b"digest", b"\x07" * 32)
    b1, _, _ = P.product_prove([fr_array_from_le(r, n) for r in raws], ots)
    b2, _, _ = P.product_prove([fr_array_from_le(raws[0], n)], ots)
    assert g1["proof"] == b1 and g2["proof"] == b2 and tr.digest() == ots.digest()


ZKRELU_CASES = [
    (1, True, 32, 16), (2, True, 32, 16), (4, False, 32, 16), (64, True, 32, 16),
    (16, True, 5, 3), (8, True, 4, 4), (4, True, 48, 16), (512, False, 32, 16), (1024, True, 32, 16),
    (1024, True, 48, 16),      # 64 bit planes: the first rounds read the value tables, not the integers
    (256, True, 40, 16),       # 56 bit planes: the widest integers the first rounds take themselves
]


@pytest.mark.parametrize("d_len,with_ga,q,r", ZKRELU_CASES)
def test_zkrelu(lib, ctx, d_len, with_ga, q, r):
    say(f"zkrelu D={d_len} ga={with_ga} Q={q} R={r}")
    rng = np.random.default_rng(d_len * 7 + q)
    lim = 1 << (q + r - 1)
    z = rng.integers(-lim, lim, d_len, dtype=np.int64)
    ga = rng.integers(-lim, lim, d_len, dtype=np.int64) if with_ga else None
    edge = [0, -1, lim - 1, -lim, 1 << (r - 1), (1 << (r - 1)) - 1, -(1 << (r - 1)), -(1 << (r - 1)) - 1]
    z[:min(d_len, len(edge))] = edge[:min(d_len, len(edge))]
    tr = lib.Transcript(21)
    got = lib.zkrelu_prove(ctx, z, ga, tr, q, r)
    ots = OracleTranscript(21)
    buf, info = P.zkrelu_prove(z.tolist(), ga.tolist() if with_ga else None, q, r, ots)
    assert got["points"] == ots.challenges
    assert got["proof"] == buf
    assert got["claims"] == info["c_in"]
    assert tr.digest() == ots.digest()


@pytest.mark.parametrize("d_len,with_ga,q,r", [(1, True, 32, 16), (2, True, 32, 16), (8, False, 5, 3),
                                               (64, True, 32, 16), (2048, True, 32, 16), (512, True, 48, 16)])
def test_zkrelu_at_given_points(lib, ctx, d_len, with_ga, q, r):
    """The four points of the input claims supplied by the caller (bound by their digest)."""
    say(f"zkrelu_at D={d_len} ga={with_ga} Q={q} R={r}")
    rng = np.random.default_rng(d_len * 11 + q)
    lim = 1 << (q + r - 1)
    z = rng.integers(-lim, lim, d_len, dtype=np.int64)
    ga = rng.integers(-lim, lim, d_len, dtype=np.int64) if with_ga else None
    li = d_len.bit_length() - 1
    pts = [[int.from_bytes(rng.bytes(40), "little") % R_MOD for _ in range(li)] for _ in range(4)]
    if li:
        pts[1][0] = 0            # a corner of the cube and the largest element among the coordinates
        pts[2][li - 1] = R_MOD - 1
    tr = lib.Transcript(22)
    got = lib.zkrelu_prove(ctx, z, ga, tr, q, r, points=pts)
    ots = OracleTranscript(22)
    buf, info = P.zkrelu_prove(z.tolist(), ga.tolist() if with_ga else None, q, r, ots, points=pts)
    assert got["points"] == [x for pt in pts for x in pt] + ots.challenges
    assert got["proof"] == buf
    assert got["claims"] == info["c_in"]
    assert tr.digest() == ots.digest()
    tv = OracleTranscript(22)
    P.zkrelu_verify(got["proof"], tv, points=pts)
    assert tv.digest() == ots.digest()


def test_zkrelu_at_rejects_bad_points(lib, ctx):
    say("zkrelu_at bad points")
    z = np.arange(4, dtype=np.int64)
    tr = lib.Transcript(3)
    before = tr.digest()
    with pytest.raises(lib.ZkdlError):
        lib.zkrelu_prove(ctx, z, None, tr, 32, 16, points=[[R_MOD, 0], [0, 0], [0, 0], [0, 0]])
    assert tr.digest() == before


@pytest.mark.parametrize("fill,d_len,with_ga", [(1, 1024, True), (64, 1024, True), (128, 512, False), (4096, 2048, True)])
def test_zkrelu_column_chunking(lib, fill, d_len, with_ga):
    """The proof does not depend on how the bit columns are cut into chunks.  With a low fill
    threshold the rounds on the columns run whole columns per thread (or a few chunks) and hand
    their column sums from round to round, which the default threshold does only for large D."""
    import paper_2307_16273_amd as zk
    say(f"zkrelu fill_threads={fill} D={d_len} ga={with_ga}")
    c2 = zk.Context(0)
    c2.set_fill_threads(fill)
    rng = np.random.default_rng(d_len + fill)
    lim = 1 << 47
    z = rng.integers(-lim, lim, d_len, dtype=np.int64)
    ga = rng.integers(-lim, lim, d_len, dtype=np.int64) if with_ga else None
    tr = lib.Transcript(23)
    got = lib.zkrelu_prove(c2, z, ga, tr, 32, 16)
    ots = OracleTranscript(23)
    buf, info = P.zkrelu_prove(z.tolist(), ga.tolist() if with_ga else None, 32, 16, ots)
    assert got["proof"] == buf
    assert got["points"] == ots.challenges
    assert tr.digest() == ots.digest()
    c2.close()


@pytest.mark.parametrize("d_len,with_ga", [(1 << 16, True), (1 << 18, False)])
def test_zkrelu_paths_agree_at_larger_sizes(lib, d_len, with_ga):
    """At sizes the Python oracle cannot prove in reasonable time: every way of cutting the work
    (whole columns per thread with round 4 on the integers and split equality tables in all
    large rounds, a few chunks, the default) gives the same proof, and the oracle's verifier
    accepts it and ends in the same transcript state."""
    import paper_2307_16273_amd as zk
    rng = np.random.default_rng(d_len)
    lim = 1 << 47
    z = rng.integers(-lim, lim, d_len, dtype=np.int64)
    ga = rng.integers(-lim, lim, d_len, dtype=np.int64) if with_ga else None
    proofs = []
    for fill in (1, 2048, 65536):
        say(f"zkrelu D={d_len} ga={with_ga} fill_threads={fill}")
        c2 = zk.Context(0)
        c2.set_fill_threads(fill)
        tr = lib.Transcript(24)
        got = lib.zkrelu_prove(c2, z, ga, tr, 32, 16)
        proofs.append((got["proof"], got["points"], tr.digest()))
        c2.close()
    assert proofs[0] == proofs[1] == proofs[2]
    ots = OracleTranscript(24)
    P.zkrelu_verify(proofs[0][0], ots)
    assert ots.digest() == proofs[0][2]
    assert ots.challenges == proofs[0][1]


@pytest.mark.parametrize("q,r", [(40, 16), (32, 16), (55, 1), (63, 1)])
def test_zkrelu_extreme_values(lib, ctx, q, r):
    """Every entry at an end of the (Q+R)-bit range, arranged so that the pairs and quadruples
    of the first two rounds see opposite ends: the integer lines reach their largest magnitude."""
    say(f"zkrelu extremes Q={q} R={r}")
    lim = 1 << (q + r - 1)
    d_len = 32
    pat = np.array([lim - 1, -lim], dtype=np.int64)
    z = pat[(np.arange(d_len) // 8 + np.arange(d_len) // 16 + np.arange(d_len)) % 2]
    ga = pat[(np.arange(d_len) // 16 + 1 + np.arange(d_len) // 4) % 2]
    z[5], ga[7] = 0, -1
    tr = lib.Transcript(22)
    got = lib.zkrelu_prove(ctx, z, ga, tr, q, r)
    ots = OracleTranscript(22)
    buf, info = P.zkrelu_prove(z.tolist(), ga.tolist(), q, r, ots)
    assert got["proof"] == buf
    assert got["points"] == ots.challenges
    assert tr.digest() == ots.digest()


def test_zkrelu_device_inputs_and_range_error(lib, ctx):
    import torch
    say("zkrelu device inputs / range error")
    rng = np.random.default_rng(8)
    z = rng.integers(-2 ** 47, 2 ** 47, 256, dtype=np.int64)
    ga = rng.integers(-2 ** 47, 2 ** 47, 256, dtype=np.int64)
    tr = lib.Transcript(2)
    got = lib.zkrelu_prove(ctx, torch.from_numpy(z).cuda(), torch.from_numpy(ga).cuda(), tr)
    ots = OracleTranscript(2)
    buf, _ = P.zkrelu_prove(z.tolist(), ga.tolist(), 32, 16, ots)
    assert got["proof"] == buf and tr.digest() == ots.digest()
    for bad_z, bad_g in ((1 << 47, 0), (0, -(1 << 47) - 1)):
        z2, g2 = z.copy(), ga.copy()
        z2[100] += 0
        z2[17] = bad_z if bad_z else z2[17]
        g2[200] = bad_g if bad_g else g2[200]
        tr = lib.Transcript(2)
        before = tr.digest()
        with pytest.raises(lib.ZkdlError) as ei:
            lib.zkrelu_prove(ctx, z2, g2, tr)
        assert ei.value.code == -2          # ZKDL_ERANGE, as the oracle's ValueError
        assert tr.digest() == before        # a failed call leaves the transcript untouched
        with pytest.raises(ValueError):
            P.zkrelu_prove(z2.tolist(), g2.tolist(), 32, 16, OracleTranscript(2))


def _update_gradients(seed, d, q, r):
    rng = np.random.default_rng(seed)
    lim = 1 << (q + r - 1)
    g = rng.integers(-lim + 1, lim, d, dtype=np.int64)
    half = 1 << (r - 1)
    for k, v in enumerate([half, -half, 3 * half, -3 * half, 0, lim - 1, -lim + 1, 1, -1]):
        if k < d:
            g[k] = v
    return g


def _drawn_only(points, drawn):
    """The library repeats the points it hands to zkReLU; the drawn challenges remain, in order."""
    out, k = [], 0
    for v in points:
        if k < len(drawn) and v == drawn[k]:
            out.append(v)
            k += 1
    return out


@pytest.mark.gpu
@pytest.mark.parametrize("d,q,r,on_device", [
    (1, 5, 3, False),            # one entry: no coordinates in p
    (2, 4, 4, False),            # Q + R a power of two
    (8, 6, 4, True),
    (64, 10, 6, False),
    (256, 32, 30, True),         # the widths of a real step: learning rate 2^-14 on 16 fractional bits
    (1024, 33, 30, False),       # Q + R = 63, the widest allowed
])
def test_update_prove(lib, ctx, d, q, r, on_device):
    """The proof of the parameter update: proof bytes, challenges, transcript and the three claims against
    the oracle, and the update claim against the definition of rounding to nearest."""
    import torch
    say(f"update_prove D={d} Q={q} R={r} device={on_device}")
    g = _update_gradients(d * 10 + q, d, q, r)
    src = torch.from_numpy(g).cuda() if on_device else g
    tr = lib.Transcript(31)
    got = lib.update_prove(ctx, src, tr, q, r)
    ots = OracleTranscript(31)
    buf, info = P.update_prove([int(x) for x in g], q, r, ots)
    assert got["proof"] == buf
    assert tr.digest() == ots.digest()
    assert _drawn_only(got["points"], ots.challenges) == ots.challenges
    ld = d.bit_length() - 1
    out = P.update_verify(got["proof"], ld, q, r, OracleTranscript(31))
    left = {c["tensor"]: c for c in got["claims_left"]}
    assert [c["tensor"] for c in got["claims_left"]] == ["U", "GW", "AUX"]
    assert left["U"]["point"] == out["u"][0] and left["U"]["value"] == out["u"][1]
    assert left["GW"]["point"] == out["gw"][0] and left["GW"]["value"] == out["gw"][1]
    assert left["AUX"]["point"] == out["aux"]["point"] and left["AUX"]["value"] == out["aux"]["value"]
    u = [P.sround(int(x), r) for x in g]
    assert left["U"]["value"] == P_mle_eval(fr_array(u), left["U"]["point"])


@pytest.mark.gpu
def test_update_prove_range_and_arguments(lib, ctx):
    say("update_prove error paths")
    tr = lib.Transcript(2)
    before = tr.digest()
    for g, q, r in ((np.array([1 << 9, 0], dtype=np.int64), 5, 5),        # 2^(Q+R-1) itself
                    (np.array([-(1 << 9), 0], dtype=np.int64), 5, 5),     # in range, its negation is not
                    (np.array([1, 2, 3], dtype=np.int64), 5, 5),          # not a power of two
                    (np.array([1, 2], dtype=np.int64), 34, 30)):          # Q + R = 64
        with pytest.raises(lib.ZkdlError):
            lib.update_prove(ctx, g, tr, q, r)
        assert tr.digest() == before


@pytest.mark.gpu
def test_update_prove_weight_stack_by_properties(lib, ctx):
    """A stack of 2^20 gradients (16 layers of 256 x 256): the oracle's verifier replays the proof, and the three
    claims it leaves are evaluated directly from the integers."""
    import torch
    say("update_prove on 2^20 gradients")
    d, q, r = 1 << 20, 32, 30
    rng = np.random.default_rng(CONFIG_SEED + 70)
    g = rng.integers(-(1 << 44), 1 << 44, d, dtype=np.int64)
    g[:4] = [1 << 29, -(1 << 29), 3 << 29, -(3 << 29)]
    tr = lib.Transcript(8)
    got = lib.update_prove(ctx, torch.from_numpy(g).cuda(), tr, q, r)
    tv = OracleTranscript(8)
    out = P.update_verify(got["proof"], 20, q, r, tv)
    assert tv.digest() == tr.digest()
    left = {c["tensor"]: c for c in got["claims_left"]}
    half = 1 << (r - 1)
    mag = (np.abs(g) + half) >> r
    u = np.where(g >= 0, mag, -mag)
    assert left["U"]["value"] == out["u"][1] == _int_mle(u, left["U"]["point"])
    assert left["GW"]["value"] == out["gw"][1] == _int_mle(g, left["GW"]["point"])
    # the gradient stack of the 8 x 1024^2 network (2^23 entries, 2^24 rows of 62 bits in zkReLU): the oracle's
    # verifier, ending in the library's transcript state
    say("update_prove on 2^23 gradients")
    d = 1 << 23
    g = rng.integers(-(1 << 44), 1 << 44, d, dtype=np.int64)
    tr = lib.Transcript(9)
    got = lib.update_prove(ctx, torch.from_numpy(g).cuda(), tr, q, r)
    tv = OracleTranscript(9)
    out = P.update_verify(got["proof"], 23, q, r, tv)
    assert tv.digest() == tr.digest()
    left = {c["tensor"]: c for c in got["claims_left"]}
    assert left["U"]["value"] == out["u"][1] and left["GW"]["value"] == out["gw"][1]
    assert left["AUX"]["value"] == out["aux"]["value"] and left["AUX"]["point"] == out["aux"]["point"]


@pytest.mark.gpu
def test_update_prove_on_a_generated_window(lib, ctx):
    """The weights of consecutive steps of a seeded window differ by the update that the proof speaks of:
    U~(p) from the library equals (W_t - W_{t+1})~(p) of the window's own weight stack."""
    import torch
    say("update_prove on the steps of a window")
    layers, width, batch, steps = 4, 32, 8, 3
    wit = fcnn_window(CONFIG_SEED + 92, n_layers=layers, width=width, batch=batch, steps=steps)
    r_bits = 16 + 8 + 3
    for t in range(steps - 1):
        a = wit["A"][t * layers:(t + 1) * layers].astype(np.int64)
        gz = wit["GZ"][t * layers:(t + 1) * layers].astype(np.int64)
        gw = np.einsum("lbi,lbo->lio", a, gz).reshape(-1)
        w0 = wit["W"][t * layers:(t + 1) * layers].astype(np.int64).reshape(-1)
        w1 = wit["W"][(t + 1) * layers:(t + 2) * layers].astype(np.int64).reshape(-1)
        assert np.any(w0 != w1)
        got = lib.update_prove(ctx, torch.from_numpy(gw).cuda(), lib.Transcript(50 + t), 32, r_bits)
        left = {c["tensor"]: c for c in got["claims_left"]}
        assert left["U"]["value"] == _int_mle(w0 - w1, left["U"]["point"])
        assert left["GW"]["value"] == _int_mle(gw, left["GW"]["point"])
        P.update_verify(got["proof"], len(gw).bit_length() - 1, 32, r_bits, OracleTranscript(50 + t))


def _int_mle(values, point):
    """MLE of a vector of Python-int-sized integers at a point, folding one coordinate at a time."""
    cur = np.array([int(v) % R_MOD for v in values], dtype=object)
    for c in point:
        half = len(cur) // 2
        cur = (cur[:half] + c * (cur[half:] - cur[:half])) % R_MOD
    return int(cur[0])


def to_cuda_witness(wit):
    import torch
    out = {k: wit[k] for k in ("L", "B", "width", "T", "Q", "R")}
    for k in ("A", "W", "GZ", "Zr", "GA"):
        out[k] = torch.from_numpy(np.ascontiguousarray(wit[k])).cuda()
    return out


def expected_claims_unlinked(res, ln):
    """The list aggregate_prove reports, from what the oracle's verifier returns: per matmul family the
    claim on the product and the two finals, then zkReLU's four input claims and the claim on aux."""
    out = []
    names = {"fwd": ("Z", "A", "W"), "gradA": ("GA", "GZ_NEXT", "W_NEXT"), "gradW": ("GW", "A", "GZ")}
    for fam in ("fwd", "gradA", "gradW"):
        proof, pt = res[fam]
        vn, vi = pt["v"][:ln], pt["v"][ln:]
        y, x0, x1 = names[fam]
        out.append(dict(tensor=y, point=pt["w"] + pt["u0"] + pt["u1"], value=proof.claim0))
        if fam == "gradW":      # X0 = A transposed: in A's own (batch, feature) order the point is (v_n, v_i, u0)
            out.append(dict(tensor=x0, point=vn + vi + pt["u0"], value=proof.finals[1]))
        else:
            out.append(dict(tensor=x0, point=vn + pt["u0"] + vi, value=proof.finals[1]))
        if fam == "gradA":      # X1 = W of the next layer transposed: in W's (in, out) order (v_n, u1, v_i)
            out.append(dict(tensor=x1, point=vn + pt["u1"] + vi, value=proof.finals[2]))
        else:
            out.append(dict(tensor=x1, point=vn + vi + pt["u1"], value=proof.finals[2]))
    zk = res["zkrelu"]
    for nm, key, c in zip(("ZR", "A_RELU", "GA", "GZ_RELU"), ("u_z", "u_a", "u_ga", "u_gz"), zk["c_in"]):
        out.append(dict(tensor=nm, point=zk["points"][key], value=c))
    out.append(dict(tensor="AUX", point=zk["aux_claim"]["point"], value=zk["aux_claim"]["value"]))
    return out


def expected_claims_linked(left):
    """The list aggregate_prove_linked reports, from aggregate_linked_verify's result."""
    (pa, va), = left["A"]
    (pw, vw), = left["W"]
    (pg, vg), = left["GZ"]
    out = [dict(tensor="A", point=pa, value=va), dict(tensor="W", point=pw, value=vw),
           dict(tensor="GZ", point=pg, value=vg)]
    for nm in ("Zlast", "GZlast"):
        point, value = left[nm]
        out.append(dict(tensor={"Zlast": "Z_LAST", "GZlast": "GZ_LAST"}[nm], point=point, value=value))
    out.append(dict(tensor="GW", point=left["GW"][0], value=left["GW"][1]))
    out.append(dict(tensor="AUX", point=left["aux"][0], value=left["aux"][1]))
    return out


@pytest.mark.parametrize("layers,width,batch,steps", [(2, 8, 4, 2), (4, 32, 8, 1), (1, 16, 2, 1)])
def test_aggregate(lib, ctx, layers, width, batch, steps):
    say(f"aggregate L={layers} w={width} B={batch} T={steps}")
    wit = fcnn_window(CONFIG_SEED + 50 + layers, layers, width, batch, steps)
    tr = lib.Transcript(33)
    got = lib.aggregate_prove(ctx, to_cuda_witness(wit), tr)
    ots = OracleTranscript(33)
    buf, _ = P.aggregate_prove(wit, ots)
    assert got["points"] == ots.challenges
    assert got["proof"] == buf
    assert tr.digest() == ots.digest()
    res = P.aggregate_verify(got["proof"], OracleTranscript(33))
    assert got["claims_left"] == expected_claims_unlinked(res, (layers * steps).bit_length() - 1)


@pytest.mark.parametrize("layers,width,batch,steps", [(2, 8, 4, 2), (4, 32, 8, 1), (1, 16, 2, 1), (2, 4, 2, 4), (8, 16, 4, 16)])
def test_aggregate_ft(lib, ctx, layers, width, batch, steps):
    """The window with its matrix products in the optimized aggregated form (f_t for the stack rounds)."""
    say(f"aggregate ft L={layers} w={width} B={batch} T={steps}")
    wit = fcnn_window(CONFIG_SEED + 70 + layers, layers, width, batch, steps)
    tr = lib.Transcript(35)
    got = lib.aggregate_prove(ctx, to_cuda_witness(wit), tr, ft=True)
    ots = OracleTranscript(35)
    buf, _ = P.aggregate_ft_prove(wit, ots)
    assert got["points"] == ots.challenges
    assert got["proof"] == buf
    assert tr.digest() == ots.digest()
    P.aggregate_ft_verify(got["proof"], OracleTranscript(35))


@pytest.mark.parametrize("layers,width,batch,steps,ft", [(2, 8, 4, 2, False), (4, 32, 8, 1, True), (1, 16, 2, 1, False),
                                                         (8, 16, 4, 16, True)])
def test_gpu_verifier_agrees_with_the_oracles(lib, ctx, layers, width, batch, steps, ft):
    """aggregate_verify on the GPU: accepts the library's proof, re-derives the oracle's challenges, ends in the
    oracle's transcript state, reports the claims the prover reported; refuses tampered proofs with the verdict
    the same program gives on the CPU, leaving the transcript alone."""
    say(f"aggregate_verify L={layers} w={width} B={batch} T={steps} ft={ft}")
    wit = fcnn_window(CONFIG_SEED + 80 + layers, layers, width, batch, steps)
    tr = lib.Transcript(36)
    got = lib.aggregate_prove(ctx, to_cuda_witness(wit), tr, ft=ft)
    ots = OracleTranscript(36)
    (P.aggregate_ft_verify if ft else P.aggregate_verify)(got["proof"], ots)
    tv = lib.Transcript(36)
    ver = lib.aggregate_verify(ctx, got["proof"], tv)
    assert ver["verdict"] == 0
    assert ver["points"] == ots.challenges == got["points"]
    assert tv.digest() == ots.digest() == tr.digest()
    if not ft:
        assert ver["claims_left"] == got["claims_left"]
    proof = got["proof"]
    for pos in (5, 29, 40, 100, len(proof) // 3, len(proof) // 2, len(proof) - 200, len(proof) - 1):
        bad = bytearray(proof)
        bad[pos] ^= 0x10
        t1, t2 = lib.Transcript(36), lib.Transcript(36)
        before = t1.digest()
        on_gpu = lib.aggregate_verify(ctx, bytes(bad), t1)
        on_cpu = lib.aggregate_verify(None, bytes(bad), t2)
        assert on_gpu["verdict"] != 0 and on_gpu["verdict"] == on_cpu["verdict"]
        assert t1.digest() == before
    assert lib.aggregate_verify(ctx, proof, lib.Transcript(37))["verdict"] != 0     # another transcript
    # a buffer too long to be staged in LDS is read from device memory: the same verdict (trailing bytes)
    long_buf = proof + bytes(40000)
    assert lib.aggregate_verify(ctx, long_buf, lib.Transcript(36))["verdict"] == \
        lib.aggregate_verify(None, long_buf, lib.Transcript(36))["verdict"] == 103


@pytest.mark.parametrize("layers,width,batch,steps", [(2, 8, 4, 2), (4, 32, 8, 1), (1, 16, 2, 1), (8, 16, 4, 16)])
def test_gpu_verifier_on_linked_windows(lib, ctx, layers, width, batch, steps):
    """aggregate_verify on a chained window: the library's own proof accepted with the oracle's challenges and
    transcript state; tampered proofs refused with the verdict the same program gives on the CPU."""
    say(f"aggregate_verify (linked) L={layers} w={width} B={batch} T={steps}")
    wit = fcnn_window(CONFIG_SEED + 85 + layers, layers, width, batch, steps)
    tr = lib.Transcript(38)
    got = lib.aggregate_prove(ctx, to_cuda_witness(wit), tr, linked=True)
    ots = OracleTranscript(38)
    P.aggregate_linked_verify(got["proof"], ots)
    tv = lib.Transcript(38)
    ver = lib.aggregate_verify(ctx, got["proof"], tv)
    assert ver["verdict"] == 0, ver["verdict"]
    assert ver["points"] == ots.challenges
    assert tv.digest() == ots.digest() == tr.digest()
    proof = got["proof"]
    n = len(proof)
    for pos in (5, 40, 100, n // 5, n // 3, n // 2, (2 * n) // 3, (3 * n) // 4, (5 * n) // 6, n - 400, n - 200, n - 1):
        bad = bytearray(proof)
        bad[pos] ^= 0x10
        t1, t2 = lib.Transcript(38), lib.Transcript(38)
        before = t1.digest()
        on_gpu = lib.aggregate_verify(ctx, bytes(bad), t1)
        on_cpu = lib.aggregate_verify(None, bytes(bad), t2)
        assert on_gpu["verdict"] != 0 and on_gpu["verdict"] == on_cpu["verdict"], pos
        assert t1.digest() == before
    assert lib.aggregate_verify(ctx, proof, lib.Transcript(39))["verdict"] != 0


@pytest.mark.parametrize("d,q,r", [(1, 5, 3), (64, 10, 6), (4096, 32, 30)])
def test_gpu_verifier_on_update_proofs(lib, ctx, d, q, r):
    say(f"aggregate_verify (update) D={d}")
    g = _update_gradients(d + 3, d, q, r)
    tr = lib.Transcript(41)
    got = lib.update_prove(ctx, g, tr, q, r)
    ots = OracleTranscript(41)
    P.update_verify(got["proof"], d.bit_length() - 1, q, r, ots)
    tv = lib.Transcript(41)
    ver = lib.aggregate_verify(ctx, got["proof"], tv)
    assert ver["verdict"] == 0, ver["verdict"]
    assert ver["points"] == ots.challenges
    assert tv.digest() == ots.digest() == tr.digest()
    proof = got["proof"]
    n = len(proof)
    for pos in (5, 13, 40, 100, n // 4, n // 2, n - 300, n - 1):
        bad = bytearray(proof)
        bad[pos] ^= 0x10
        t1, t2 = lib.Transcript(41), lib.Transcript(41)
        on_gpu = lib.aggregate_verify(ctx, bytes(bad), t1)
        on_cpu = lib.aggregate_verify(None, bytes(bad), t2)
        assert on_gpu["verdict"] != 0 and on_gpu["verdict"] == on_cpu["verdict"], pos


@pytest.mark.parametrize("layers,width,batch,steps", [(2, 8, 4, 2), (4, 32, 8, 1), (1, 16, 2, 1), (2, 4, 2, 4),
                                                      (4, 16, 8, 4)])
def test_aggregate_linked(lib, ctx, layers, width, batch, steps):
    """The four families with their claims chained: zkReLU at the points the matmul sumchecks
    leave, re-indexing for the shifted stacks."""
    say(f"aggregate linked L={layers} w={width} B={batch} T={steps}")
    wit = fcnn_window(CONFIG_SEED + 60 + layers, layers, width, batch, steps)
    tr = lib.Transcript(34)
    got = lib.aggregate_prove(ctx, to_cuda_witness(wit), tr, linked=True)
    ots = OracleTranscript(34)
    buf, infos = P.aggregate_linked_prove(wit, ots)
    assert got["proof"] == buf
    assert tr.digest() == ots.digest()
    # the library repeats the four given points in front of zkReLU's own draws
    before = sum(len(infos[k][c]) for k in ("fwd", "gradA", "gradW") for c in ("w", "u0", "u1", "v"))
    zk = infos["zkrelu"]
    given = zk["u_z"] + zk["u_a"] + zk["u_ga"] + zk["u_gz"]
    assert got["points"] == ots.challenges[:before] + given + ots.challenges[before:]
    left = P.aggregate_linked_verify(got["proof"], OracleTranscript(34))
    assert got["claims_left"] == expected_claims_linked(left)


def test_config1_fc_layer_plus_relu(lib, ctx):
    """One FC layer + ReLU: X 16x256, W 256x256, zkReLU over Z with Q=32 (forward only)."""
    import torch
    say("config 1")
    lay = fc_relu_layer(CONFIG_SEED + 1)
    tr = lib.Transcript(CONFIG_SEED + 1)
    x = lib.tensor_wrap_int(ctx, torch.from_numpy(lay["X"]).cuda(), (1, 16, 256))
    w = lib.tensor_wrap_int(ctx, torch.from_numpy(lay["W"]).cuda(), (1, 256, 256))
    g1 = lib.sumcheck_matmul(ctx, x, w, tr)
    g2 = lib.zkrelu_prove(ctx, torch.from_numpy(lay["Z"]).cuda().reshape(-1), None, tr)
    ots = OracleTranscript(CONFIG_SEED + 1)
    b1, p1, _ = P.matmul_prove(fr_array(lay["X"]), [1, 16, 256], fr_array(lay["W"]), [1, 256, 256], ots)
    b2, info = P.zkrelu_prove(lay["Z"].reshape(-1).tolist(), None, 32, 16, ots)
    assert g1["proof"] == b1 and g2["proof"] == b2
    assert tr.digest() == ots.digest()
    # the matmul's claim on Y is the MLE of the very Z that zkReLU decomposes
    from oracle.mle import mle_eval
    pts = g1["points"]
    assert g1["claims"][0] == mle_eval(fr_array(lay["Z"]), pts[:4 + 8])


@pytest.mark.parametrize("shape,lo,hi", [((4096, 256), 0, 1), ((2, 8192, 64), 1, 2), ((512, 1024), 1, 2),
                                          ((128, 4096), 1, 2), ((64, 64), 1, 2)])
def test_partial_eval_long_axes_int32_and_fr(lib, ctx, shape, lo, hi):
    """Long contracted axes go through the wide-accumulation kernels: extreme and sign-mixed integers."""
    import torch
    say(f"partial_eval long axis shape={shape} axes=[{lo},{hi})")
    rng = np.random.default_rng(sum(shape))
    n = int(np.prod(shape))
    src = rng.integers(-2 ** 31, 2 ** 31, n, dtype=np.int64).astype(np.int32)
    src[:8] = [-2 ** 31, 2 ** 31 - 1, -1, 0, 1, -2 ** 31, -2 ** 31, 2 ** 31 - 1]
    npt = sum(int(s).bit_length() - 1 for s in shape[lo:hi])
    point = fr_array_from_le(rand_fr_bytes(5, npt), npt).tolist()
    t = lib.tensor_wrap_int(ctx, torch.from_numpy(src).cuda(), shape)
    out = lib.mle_partial_eval(ctx, t, lo, hi, point)
    expect, oshape = partial_eval(fr_array(src), shape, lo, hi, point)
    assert out.download() == array_to_le(expect)
    if lo == 0:
        raw = uniform_fr_limbs(rng, n)
        raw[0] = [0xFFFFFFFF00000000, 0x53BDA402FFFE5BFE, 0x3339D80809A1D805, 0x73EDA753299D7D48]   # r - 1
        tf = lib.fr_tensor_upload(ctx, raw.tobytes(), shape)
        outf = lib.mle_partial_eval(ctx, tf, lo, hi, point)
        expf, _ = partial_eval(fr_array_from_le(raw.tobytes(), n), shape, lo, hi, point)
        assert outf.download() == array_to_le(expf)


def test_full_size_microbench_sumcheck_by_properties(lib, ctx):
    """Three tables of 2^24 (the benchmark's launch configuration).  The oracle cannot redo
    the proof in seconds at this size, so the proof is checked through what holds at any size:
    the oracle's verifier accepts it (every round, the final product, the same transcript),
    claim_0 equals the exact integer sum, and the finals equal closed-form MLE evaluations of
    tables chosen to have one: T0[b] = b, T1[b] = 3b + 7, T2[b] = b xor c."""
    import torch
    say("full-size sumcheck_product (2^24 x 3)")
    d = 24
    n = 1 << d
    c = 0xA5C3F1
    b = np.arange(n, dtype=np.int64)
    tabs_np = [b, 3 * b + 7, b ^ c]
    tabs = [lib.fr_tensor_upload(ctx, torch.from_numpy(t).cuda(), (n,)) for t in tabs_np]
    tr = lib.Transcript(99)
    got = lib.sumcheck_product(ctx, tabs, tr)
    ots = OracleTranscript(99)
    proof, vs = P.product_verify(got["proof"], 3, d, ots)
    assert tr.digest() == ots.digest() and got["points"] == vs
    # claim_0: exact sum of the integer products (chunked so that intermediate values stay exact)
    total = 0
    for s in range(0, n, 1 << 20):
        x = b[s:s + (1 << 20)].astype(object)
        total += int(np.sum(x * (3 * x + 7) * (x ^ c)))
    assert proof.claim0 == total % R_MOD
    # finals: the MLE of b is sum_k 2^(d-1-k) v_k; xor with a constant flips v_k to 1 - v_k
    idx = sum(((1 << (d - 1 - k)) * vs[k]) for k in range(d)) % R_MOD
    xor = sum((1 << (d - 1 - k)) * ((1 - vs[k]) if (c >> (d - 1 - k)) & 1 else vs[k]) for k in range(d)) % R_MOD
    assert got["claims"] == [idx, (3 * idx + 7) % R_MOD, xor]


def test_full_size_partial_eval_sampled(lib, ctx):
    """4096 x 4096 uniform Fr matrix at a row point: sampled output columns against the oracle."""
    say("full-size mle_partial_eval (4096 x 4096)")
    rng = np.random.default_rng(CONFIG_SEED + 2)
    side = 4096
    limbs = uniform_fr_limbs(rng, side * side)
    t = lib.fr_tensor_upload(ctx, limbs, (side, side))
    point = fr_array_from_le(rand_fr_bytes(8, 12), 12).tolist()
    out = lib.mle_partial_eval(ctx, t, 0, 1, point).download()
    from oracle.mle import beta_table
    beta = beta_table(point)
    m3 = limbs.reshape(side, side, 4)
    for col in (0, 1, 63, 64, 2047, 4095, 1234, 3001):
        colv = fr_array_from_le(np.ascontiguousarray(m3[:, col, :]).tobytes(), side)
        expect = int(np.sum(beta * colv) % R_MOD)
        assert int.from_bytes(out[32 * col:32 * col + 32], "little") == expect


def test_full_size_microbench_byte_exact_against_c_tier(lib, ctx):
    """The benchmark's own inputs and launch configuration (three tables of 2^24 uniform Fr,
    the 4096 x 4096 matrix): proof bytes, challenges, transcript digest and every output of
    the partial evaluation against the C tier of the oracle, which is pinned byte for byte
    against the Python tier on small inputs (tests/test_oracle_c.py)."""
    from oracle import c_oracle
    say("full-size microbench, byte-exact against the C oracle tier")
    d = 24
    n = 1 << d
    side = 1 << (d // 2)
    rng = np.random.default_rng(CONFIG_SEED + 2)
    raws = [uniform_fr_limbs(rng, n) for _ in range(3)]
    mat = uniform_fr_limbs(rng, side * side)
    point = [int.from_bytes(uniform_fr_limbs(rng, 1).tobytes(), "little") for _ in range(d // 2)]
    tabs = [lib.fr_tensor_upload(ctx, r, (n,)) for r in raws]
    tr = lib.Transcript(CONFIG_SEED + 2)
    got = lib.sumcheck_product(ctx, tabs, tr)
    for t in tabs:
        t.free()
    say("  C oracle: sumcheck")
    proof, vs, digest = c_oracle.product_prove([r.tobytes() for r in raws], CONFIG_SEED + 2)
    assert got["proof"] == proof
    assert got["points"] == vs
    assert tr.digest() == digest
    del raws
    tm = lib.fr_tensor_upload(ctx, mat, (side, side))
    out = lib.mle_partial_eval(ctx, tm, 0, 1, point).download()
    say("  C oracle: partial evaluation")
    assert out == c_oracle.partial_eval(mat.tobytes(), 1, side, side, point)


def test_config3_aggregate_by_properties(lib, ctx):
    """8 layers x 1024, batch 64 (the aggregate timed by the benchmark): the oracle's verifier
    accepts the proof and ends in the same transcript state; the forward family's claim on the
    activation stack equals its direct MLE evaluation."""
    say("config 3 aggregate (8 x 1024^2, batch 64)")
    from oracle.mle import mle_eval
    wit = fcnn_window(CONFIG_SEED + 3, n_layers=8, width=1024, batch=64, steps=1)
    tr = lib.Transcript(CONFIG_SEED + 3)
    got = lib.aggregate_prove(ctx, to_cuda_witness(wit), tr)
    ots = OracleTranscript(CONFIG_SEED + 3)
    res = P.aggregate_verify(got["proof"], ots)
    assert tr.digest() == ots.digest()
    assert got["points"] == ots.challenges
    fproof, fpts = res["fwd"]
    vn, vi = fpts["v"][:3], fpts["v"][3:]
    assert fproof.finals[1] == mle_eval(fr_array(wit["A"]), vn + fpts["u0"] + vi)
    # zkReLU at full size (D = 2^19 rows): the four input claims are the MLEs of Z, A = relu(Z'),
    # G_A and (1 - sign) G_A' at their points, and the one claim left on aux after the merge is
    # aux~(k*, v, w*) evaluated directly from the bits of the witness
    from oracle.mle import beta_table
    zk = res["zkrelu"]
    z = wit["Zr"].reshape(-1).astype(object)
    ga = wit["GA"].reshape(-1).astype(object)
    q_bits, r_bits = wit["Q"], wit["R"]
    half = 1 << (r_bits - 1)
    ns = np.array([0 if int(x) < 0 else 1 for x in z], dtype=object)
    zp = np.array([(int(x) + half) >> r_bits for x in z], dtype=object)
    gp = np.array([(int(x) + half) >> r_bits for x in ga], dtype=object)
    pts = zk["points"]
    for claim, vec, pt in ((zk["c_in"][0], z, pts["u_z"]), (zk["c_in"][1], ns * zp, pts["u_a"]),
                           (zk["c_in"][2], ga, pts["u_ga"]), (zk["c_in"][3], ns * gp, pts["u_gz"])):
        assert claim == int(np.dot(beta_table(pt), vec % R_MOD) % R_MOD)
    li = len(pts["u_z"])
    point, value = zk["aux_claim"]["point"], zk["aux_claim"]["value"]
    kst, v_i, wst = point[0], point[1:1 + li], point[1 + li:]
    b_i, b_j = beta_table(v_i), beta_table(wst)
    total = 0
    for bk, arr in (((1 - kst) % R_MOD, wit["Zr"].reshape(-1)), (kst, wit["GA"].reshape(-1))):
        for j in range(q_bits + r_bits):
            mask = ((arr >> j) & 1).astype(bool)
            total += bk * int(b_j[j]) % R_MOD * int(b_i[mask].sum() % R_MOD)
    assert value == total % R_MOD


def _stack_mle(stack, pn, pr, pc):
    """X~(pn, pr, pc) of an integer stack [N, rows, cols], one slot at a time."""
    from oracle.mle import beta_table
    bn, br, bc = beta_table(pn), beta_table(pr), beta_table(pc)
    total = 0
    for k in range(stack.shape[0]):
        rows = np.dot(stack[k].astype(object), bc) % R_MOD
        total += int(bn[k]) * int(np.dot(br, rows) % R_MOD)
    return total % R_MOD


def test_config3_aggregate_linked_by_properties(lib, ctx):
    """8 layers x 1024, batch 64 with the claims chained: the oracle's verifier accepts the proof,
    checks every link and ends in the same transcript state; each claim that is left is the MLE
    of the stack it names, evaluated here from the witness."""
    say("config 3 linked aggregate (8 x 1024^2, batch 64)")
    wit = fcnn_window(CONFIG_SEED + 3, n_layers=8, width=1024, batch=64, steps=1)
    tr = lib.Transcript(CONFIG_SEED + 4)
    got = lib.aggregate_prove(ctx, to_cuda_witness(wit), tr, linked=True)
    ots = OracleTranscript(CONFIG_SEED + 4)
    left = P.aggregate_linked_verify(got["proof"], ots)
    assert tr.digest() == ots.digest()
    tv = lib.Transcript(CONFIG_SEED + 4)
    ver = lib.aggregate_verify(ctx, got["proof"], tv)                 # the library's own verifier, on the GPU
    assert ver["verdict"] == 0 and ver["points"] == ots.challenges and tv.digest() == ots.digest()
    ln, lb = 3, 6
    for name in ("A", "GZ", "W"):
        rows_bits = lb if name != "W" else 10
        for point, value in left[name]:
            assert value == _stack_mle(wit[name], point[:ln], point[ln:ln + rows_bits], point[ln + rows_bits:]), name
    z_last = wit["A"][7].astype(np.int64) @ wit["W"][7].astype(np.int64)
    point, value = left["Zlast"]
    assert value == _stack_mle(z_last[None], [], point[:lb], point[lb:])
    point, value = left["GZlast"]
    assert value == _stack_mle(wit["GZ"][7:8], [], point[:lb], point[lb:])


@pytest.mark.parametrize("name,layers,width,batch,steps,cfg", [
    ("config 4: 8 x 1024^2, batch 64, 16 steps aggregated", 8, 1024, 64, 16, 4),
    ("config 5: 4 x 4096^2, batch 256", 4, 4096, 256, 1, 5),
])
def test_large_aggregates_by_properties(lib, ctx, name, layers, width, batch, steps, cfg):
    """Full-size aggregated proofs: the oracle's verifier replays every round of all four
    families and must end in the library's transcript state."""
    say(name)
    wit = fcnn_window(CONFIG_SEED + cfg, n_layers=layers, width=width, batch=batch, steps=steps)
    tr = lib.Transcript(CONFIG_SEED + cfg)
    got = lib.aggregate_prove(ctx, to_cuda_witness(wit), tr)
    ots = OracleTranscript(CONFIG_SEED + cfg)
    res = P.aggregate_verify(got["proof"], ots)
    assert tr.digest() == ots.digest()
    assert got["points"] == ots.challenges
    assert got["claims_left"] == expected_claims_unlinked(res, (layers * steps).bit_length() - 1)
    ver = lib.aggregate_verify(ctx, got["proof"], lib.Transcript(CONFIG_SEED + cfg))
    assert ver["verdict"] == 0 and ver["points"] == ots.challenges and ver["claims_left"] == got["claims_left"]
    ctx.trim()
    # the same window with the claims chained: every link holds, and the one claim left on each of
    # A, G_Z and W (the merge on W runs over the whole stack, 2^26 or 2^27 elements) is the MLE of
    # the witness stack
    say(name + " (linked)")
    tr = lib.Transcript(CONFIG_SEED + cfg + 1)
    got = lib.aggregate_prove(ctx, to_cuda_witness(wit), tr, linked=True)
    ots = OracleTranscript(CONFIG_SEED + cfg + 1)
    left = P.aggregate_linked_verify(got["proof"], ots)
    assert tr.digest() == ots.digest()
    assert got["claims_left"] == expected_claims_linked(left)
    tv = lib.Transcript(CONFIG_SEED + cfg + 1)
    ver = lib.aggregate_verify(ctx, got["proof"], tv)
    assert ver["verdict"] == 0 and ver["points"] == ots.challenges and tv.digest() == ots.digest()
    ln, lb, lw = (layers * steps).bit_length() - 1, batch.bit_length() - 1, width.bit_length() - 1
    for nm in ("A", "GZ", "W"):
        rows_bits = lb if nm != "W" else lw
        (point, value), = left[nm]
        assert value == _stack_mle(wit[nm], point[:ln], point[ln:ln + rows_bits], point[ln + rows_bits:]), nm
    ctx.trim()
