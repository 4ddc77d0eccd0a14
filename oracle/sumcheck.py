"""Textbook sumcheck prover and verifier (Sec. 2.2; App. B round structure).

The claim is  sum_{b in {0,1}^d} F(b)  with  F = sum_terms coef * prod_k T_k,
every T_k a table of length 2^d read as a multilinear polynomial.  In round t
the prover sends g_t(x) = sum over the remaining hypercube of F(v_0..v_{t-1},
x, b') as its values at x = 0..deg, the verifier checks
g_t(0) + g_t(1) = previous claim, draws v_t, and the next claim is g_t(v_t).

Reading adopted where the paper leaves a choice: the equality-polynomial
factor beta~(w, .) is an ordinary table of the product and is folded like the
others, so the prover sends g_t itself (not the beta-free f_t of the optimized
protocol in App. B); both reach the same final evaluation claims.
Test infrastructure; not used by the product.
"""
import struct

import numpy as np

from .field import R_MOD, inv, to_le, from_le
from .mle import ilog2

SC_MAGIC = 0x43534B5A   # bytes "ZKSC"


def lagrange_eval(ys, v):
    """Value at v of the polynomial of degree < len(ys) through (k, ys[k])."""
    n = len(ys)
    acc = 0
    for k in range(n):
        num, den = 1, 1
        for j in range(n):
            if j != k:
                num = num * (v - j) % R_MOD
                den = den * (k - j) % R_MOD
        acc = (acc + ys[k] * num % R_MOD * inv(den)) % R_MOD
    return acc


def hypercube_sum(tables, terms):
    total = 0
    for coef, idx in terms:
        prod = tables[idx[0]]
        for k in idx[1:]:
            prod = prod * tables[k] % R_MOD
        total = (total + coef * int(np.sum(prod) % R_MOD)) % R_MOD
    return total


class SumcheckProof:
    """One sumcheck: claim_0, the round evaluations, the final table values."""

    def __init__(self, n_finals, degree, claim0, rounds, finals):
        self.n_finals = n_finals
        self.degree = degree
        self.claim0 = claim0
        self.rounds = rounds          # list of lists of degree+1 elements
        self.finals = finals          # list of n_finals elements

    def to_bytes(self):
        out = [struct.pack("<IIII", SC_MAGIC, self.n_finals, self.degree, len(self.rounds))]
        out.append(to_le(self.claim0))
        for g in self.rounds:
            assert len(g) == self.degree + 1
            out.extend(to_le(x) for x in g)
        out.extend(to_le(x) for x in self.finals)
        return b"".join(out)

    @staticmethod
    def from_bytes(buf, off=0):
        magic, k, deg, rounds = struct.unpack_from("<IIII", buf, off)
        assert magic == SC_MAGIC
        off += 16

        def take():
            nonlocal off
            x = from_le(buf[off:off + 32])
            off += 32
            return x
        claim0 = take()
        rs = [[take() for _ in range(deg + 1)] for _ in range(rounds)]
        finals = [take() for _ in range(k)]
        return SumcheckProof(k, deg, claim0, rs, finals), off


def round_message(g):
    """What a round binds into the transcript: g_t(0), g_t(2), ..., g_t(deg).

    g_t(1) is left out: the round check g_t(0) + g_t(1) = claim (Sec. 2.2) fixes it,
    and the claim is a function of what the transcript already holds.  The proof
    bytes still carry all deg + 1 evaluations.
    """
    return [g[0]] + list(g[2:])


def prove(tables, terms, degree, ts, absorb_claim=True, report=None):
    """Run the prover.  `tables`: list of equal-length object arrays (2^d);
    `terms`: list of (coef, [table ids]); returns (SumcheckProof, challenges).

    Every table is folded with every challenge.  `report` maps the list of all
    tables' final values to the list that is sent (default: all, in order).
    """
    tables = [np.asarray(t, dtype=object).reshape(-1) % R_MOD for t in tables]
    n = tables[0].shape[0]
    d = ilog2(n)
    assert all(t.shape[0] == n for t in tables)
    claim = hypercube_sum(tables, terms)
    claim0 = claim
    if absorb_claim:
        ts.absorb_fr(b"c", [claim0])
    rounds, vs = [], []
    for _ in range(d):
        half = tables[0].shape[0] // 2
        lo = [t[:half] for t in tables]
        hi = [t[half:] for t in tables]
        g = []
        for x in range(degree + 1):
            at_x = [(l + x * (h - l)) % R_MOD for l, h in zip(lo, hi)]
            g.append(hypercube_sum(at_x, terms))
        assert (g[0] + g[1]) % R_MOD == claim, "round invariant broken"
        ts.absorb_fr(b"g", round_message(g))
        v = ts.challenge()
        tables = [(l + v * (h - l)) % R_MOD for l, h in zip(lo, hi)]
        claim = lagrange_eval(g, v)
        rounds.append(g)
        vs.append(v)
    finals_all = [int(t[0]) for t in tables]
    finals = list(finals_all) if report is None else [x % R_MOD for x in report(finals_all)]
    ts.absorb_fr(b"f", finals)
    assert hypercube_sum([np.array([f], dtype=object) for f in finals_all], terms) == claim
    return SumcheckProof(len(finals), degree, claim0, rounds, finals), vs


def verify_rounds(proof, ts, absorb_claim=True, expected_claim0=None):
    """Replay the rounds: check every g_t(0)+g_t(1), re-derive the challenges.

    Returns (final claim, challenges).  The caller checks the final claim
    against the expression in the reported finals and absorbs nothing more.
    Raises AssertionError on any failed check.
    """
    claim = proof.claim0
    if expected_claim0 is not None:
        assert claim == expected_claim0 % R_MOD, "claim_0 mismatch"
    if absorb_claim:
        ts.absorb_fr(b"c", [claim])
    vs = []
    for g in proof.rounds:
        assert len(g) == proof.degree + 1
        assert (g[0] + g[1]) % R_MOD == claim, "g(0)+g(1) != claim"
        ts.absorb_fr(b"g", round_message(g))
        v = ts.challenge()
        claim = lagrange_eval(g, v)
        vs.append(v)
    ts.absorb_fr(b"f", proof.finals)
    return claim, vs
