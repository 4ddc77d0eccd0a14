"""The entry point that allocates nothing (sumcheck_product_noalloc) against sumcheck_product:
same proof bytes, challenges, finals and transcript, on two calls in a row, the second with a
smaller input (the static work memory still holds the first call's tables)."""
import numpy as np
import pytest

from workloads import uniform_fr_limbs

pytestmark = pytest.mark.gpu


def _tables(lib, ctx, seed, k, d):
    n = 1 << d
    return [lib.fr_tensor_upload(ctx, uniform_fr_limbs(np.random.default_rng(seed + j), n).tobytes(), (n,))
            for j in range(k)]


def _both(lib, ctx, tabs, seed):
    tr_a, tr_b = lib.Transcript(seed), lib.Transcript(seed)
    want = lib.sumcheck_product(ctx, tabs, tr_a)
    got = lib.sumcheck_product(ctx, tabs, tr_b, noalloc=True)
    assert got["proof"] == want["proof"]
    assert got["points"] == want["points"]
    assert got["claims"] == want["claims"]
    assert tr_b.digest() == tr_a.digest()


def test_noalloc_matches_sumcheck_product_twice_in_a_row(lib, ctx):
    big = _tables(lib, ctx, 9100, 3, 16)      # several blocks per round, then the single-block tail
    small = _tables(lib, ctx, 9200, 3, 9)     # the single-block tail only, on a used work array
    # the reference proofs first, so that the two calls under test follow each other directly
    refs = []
    for tabs, seed in ((big, 1), (small, 2)):
        tr = lib.Transcript(seed)
        refs.append((lib.sumcheck_product(ctx, tabs, tr), tr.digest()))
    for (tabs, seed), (want, digest) in zip(((big, 1), (small, 2)), refs):
        tr = lib.Transcript(seed)
        got = lib.sumcheck_product(ctx, tabs, tr, noalloc=True)
        assert got["proof"] == want["proof"] and got["points"] == want["points"]
        assert got["claims"] == want["claims"] and tr.digest() == digest


@pytest.mark.parametrize("k,d", [(1, 0), (2, 1), (3, 2), (2, 12), (3, 18), (1, 5)])
def test_noalloc_shapes(lib, ctx, k, d):
    _both(lib, ctx, _tables(lib, ctx, 9300 + 10 * d, k, d), 40 + d)


def test_noalloc_limits(lib, ctx):
    import torch
    tabs = _tables(lib, ctx, 9400, 1, 19)
    tr = lib.Transcript(3)
    before = tr.digest()
    with pytest.raises(lib.ZkdlError) as e:
        lib.sumcheck_product(ctx, tabs, tr, noalloc=True)
    assert e.value.code == -6 and tr.digest() == before        # ZKDL_ETOOBIG, nothing consumed
    ints = lib.tensor_wrap_int(ctx, torch.arange(64, dtype=torch.int32).cuda())
    with pytest.raises(lib.ZkdlError) as e:
        lib.sumcheck_product(ctx, [ints], tr, noalloc=True)
    assert e.value.code == -1 and tr.digest() == before
    # a second context on the same device shares the array; calls one after the other agree
    other = lib.Context(0)
    small = _tables(lib, other, 9500, 2, 8)
    _both(lib, other, small, 77)
    other.close()
