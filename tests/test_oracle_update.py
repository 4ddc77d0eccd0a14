"""Pins for the oracle's proof of the parameter update (Sec. 5, Example FCNN, last item; the rounding is
proved by zkReLU, Sec. 3.1 and App. A)."""
import numpy as np
import pytest

from oracle.field import R_MOD, fr_array
from oracle.mle import mle_eval, ilog2
from oracle import protocols as P
from oracle.transcript import Transcript
from workloads import fcnn_window, CONFIG_SEED


def nearest_away(g, r_bits):
    """g / 2^r to the nearest integer, halves away from zero, from exact rationals."""
    from fractions import Fraction
    x = Fraction(int(g), 1 << r_bits)
    lo = x.numerator // x.denominator          # floor
    frac = x - lo
    if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and x > 0):
        return lo + 1
    return lo


def test_sround_is_nearest_with_halves_away_from_zero():
    for r_bits in (1, 3, 4, 16):
        half = 1 << (r_bits - 1)
        vals = list(range(-5 * half - 3, 5 * half + 4)) + [3 * half, -3 * half, (1 << 40) + half, -(1 << 40) - half]
        for g in vals:
            assert P.sround(g, r_bits) == nearest_away(g, r_bits)
            assert P.sround(-g, r_bits) == -P.sround(g, r_bits)
    # differs from zkReLU's own rescaling (round half up) exactly at the negative ties
    assert P.sround(-8, 4) == -1 and (-8 + 8) >> 4 == 0
    assert P.sround(8, 4) == 1 and (8 + 8) >> 4 == 1


def test_update_is_the_difference_of_two_relus():
    # U = ReLU(rescale(G)) - ReLU(rescale(-G)) with rescale = round half up: the identity the proof rests on
    for r_bits in (1, 2, 5):
        half = 1 << (r_bits - 1)
        for g in range(-6 * half - 2, 6 * half + 3):
            up = lambda x: (x + half) >> r_bits
            assert max(0, up(g)) - max(0, up(-g)) == P.sround(g, r_bits)


def gradients(seed, d, q, r_bits):
    rng = np.random.default_rng(seed)
    lim = 1 << (q + r_bits - 1)
    g = [int(x) for x in rng.integers(-lim + 1, lim, d)]
    half = 1 << (r_bits - 1)
    for k, v in enumerate([half, -half, 3 * half, -3 * half, 0, lim - 1, -lim + 1, 1, -1]):
        if k < d:
            g[k] = v
    return g


@pytest.mark.parametrize("d,q,r_bits", [(1, 5, 3), (2, 4, 4), (8, 6, 4), (16, 10, 6), (4, 32, 30), (4, 33, 30)])
def test_update_claims_are_the_definitions(d, q, r_bits):
    g = gradients(d * 100 + q, d, q, r_bits)
    ts = Transcript(21)
    buf, info = P.update_prove(g, q, r_bits, ts)
    ld = ilog2(d)
    tv = Transcript(21)
    out = P.update_verify(buf, ld, q, r_bits, tv)
    assert tv.digest() == ts.digest() and tv.challenges == ts.challenges
    u = [nearest_away(x, r_bits) for x in g]
    p, u_val = out["u"]
    assert p == info["p"] and len(p) == ld
    assert u_val == mle_eval(fr_array(u), p)                      # the update itself, from the definition
    pt, g_val = out["gw"]
    assert g_val == mle_eval(fr_array(g), pt)                     # the claim left on the gradients
    # the two halves of Au and the claim left on the bits
    assert info["a"][0] == mle_eval(fr_array([max(0, x) for x in u]), p)
    assert info["a"][1] == mle_eval(fr_array([max(0, -x) for x in u]), p)
    zu = g + [-x for x in g]
    wit = P.zkrelu_witness(zu, [0] * (2 * d), q, r_bits)
    aux = np.concatenate([fr_array(wit["aux0"]), fr_array(wit["aux1"])])
    assert out["aux"]["value"] == mle_eval(aux, out["aux"]["point"])
    # the two claims lie on a line in the stack coordinate: the one claim zkReLU starts from is Au~(rho, p)
    au = [max(0, x) for x in u] + [max(0, -x) for x in u]
    assert info["zkrelu"]["c_in"][1] == mle_eval(fr_array(au), [info["rho"]] + p)
    assert info["zkrelu"]["c_in"][1] == ((1 - info["rho"]) * info["a"][0] + info["rho"] * info["a"][1]) % R_MOD
    # proof size: header, the two claims, zkReLU on 2 D rows
    lj = ilog2(wit["j_pad"])
    zk = 32 + 128 + (16 + 32 + (1 + ld + lj) * 128 + 96) + (16 + 32 + (1 + lj) * 96 + 64)
    assert len(buf) == 32 + 64 + zk


def test_update_closes_a_step_of_sgd():
    # W_next = W - U entry by entry, so W_next~(p) = W~(p) - U~(p) for the proof's p: what the verifier
    # checks against two openings
    rng = np.random.default_rng(5)
    d, q, r_bits = 16, 12, 8
    w = [int(x) for x in rng.integers(-2000, 2000, d)]
    g = gradients(77, d, q, r_bits)
    w_next = [a - nearest_away(b, r_bits) for a, b in zip(w, g)]
    buf, info = P.update_prove(g, q, r_bits, Transcript(3))
    out = P.update_verify(buf, 4, q, r_bits, Transcript(3))
    p, u_val = out["u"]
    assert (mle_eval(fr_array(w), p) - mle_eval(fr_array(w_next), p)) % R_MOD == u_val
    # a step with another rounding (half up) is not what the proof says
    w_bad = [a - ((b + (1 << (r_bits - 1))) >> r_bits) for a, b in zip(w, g)]
    assert w_bad != w_next
    assert (mle_eval(fr_array(w), p) - mle_eval(fr_array(w_bad), p)) % R_MOD != u_val


def test_update_rejects_out_of_range_and_tampering():
    with pytest.raises(ValueError):
        P.update_prove([1 << 9, 0], 5, 5, Transcript(1))         # 2^(Q+R-1) itself
    with pytest.raises(ValueError):
        P.update_prove([-(1 << 9), 0], 5, 5, Transcript(1))      # in range, but its negation is not
    g = gradients(9, 4, 5, 3)
    buf, _ = P.update_prove(g, 5, 3, Transcript(2))
    P.update_verify(buf, 2, 5, 3, Transcript(2))
    rng = np.random.default_rng(0)
    elems = [32, 64] + [o for o in range(96 + 32, len(buf) - 31, 32)]
    for off in rng.choice(elems, 24, replace=False):
        bad = bytearray(buf)
        bad[off + 3] ^= 0x10
        with pytest.raises(AssertionError):
            P.update_verify(bytes(bad), 2, 5, 3, Transcript(2))
    with pytest.raises(AssertionError):
        P.update_verify(buf, 2, 5, 3, Transcript(4))             # another transcript
    with pytest.raises(AssertionError):
        P.update_verify(buf + b"\x00" * 32, 2, 5, 3, Transcript(2))


def window_gradients(wit, t):
    """G_W = A^T G_Z of every layer of step t, and the weights before and after the step."""
    n_layers = wit["L"]
    a = wit["A"][t * n_layers:(t + 1) * n_layers].astype(np.int64)
    gz = wit["GZ"][t * n_layers:(t + 1) * n_layers].astype(np.int64)
    gw = np.einsum("lbi,lbo->lio", a, gz)
    return gw, wit["W"][t * n_layers:(t + 1) * n_layers].astype(np.int64), \
        wit["W"][(t + 1) * n_layers:(t + 2) * n_layers].astype(np.int64)


def test_update_of_a_generated_window():
    # the weights of consecutive steps of a seeded window differ by the update the proof speaks of
    wit = fcnn_window(CONFIG_SEED + 91, n_layers=2, width=4, batch=2, steps=3)
    r_bits = 16 + 8 + 1          # the generator's learning-rate shift for batch 2
    for t in range(2):
        gw, w0, w1 = window_gradients(wit, t)
        g = [int(x) for x in gw.reshape(-1)]
        buf, _ = P.update_prove(g, 32, r_bits, Transcript(40 + t))
        out = P.update_verify(buf, ilog2(len(g)), 32, r_bits, Transcript(40 + t))
        p, u_val = out["u"]
        diff = [int(x) for x in (w0 - w1).reshape(-1)]
        assert u_val == mle_eval(fr_array(diff), p)
