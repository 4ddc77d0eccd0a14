"""Multilinear extensions (Eq. multilinear-extension, Sec. 2.2).

Index/variable convention (the paper only says an index is identified with its
binary string): tensors are row-major; a point is the concatenation of one
vector per axis, leading axis first; inside an axis coordinate 0 is the most
significant bit of that axis' index.  So variable 0 is the most significant bit
of the flat row-major index, and binding it pairs T[b] with T[b + len/2].
Test infrastructure; not used by the product.
"""
import numpy as np

from .field import R_MOD


def ilog2(n):
    n = int(n)
    assert n >= 1 and (n & (n - 1)) == 0, f"{n} is not a power of two"
    return n.bit_length() - 1


def beta_eval(u, b):
    """beta~(u, b) for a Boolean index b: prod_k (u_k b_k + (1-u_k)(1-b_k)).

    The unique multilinear polynomial that is the indicator of u == b on
    Boolean inputs (Sec. 2.2); bit k of b, counted from the most significant of
    len(u) bits, pairs with u_k.
    """
    m = len(u)
    acc = 1
    for k in range(m):
        bit = (b >> (m - 1 - k)) & 1
        acc = acc * (u[k] if bit else (1 - u[k])) % R_MOD
    return acc


def beta_table(u):
    """All 2^m values beta~(u, b), b = 0..2^m-1, by doubling."""
    eq = [1]
    for uk in u:
        nxt = [0] * (2 * len(eq))
        for i, e in enumerate(eq):
            nxt[2 * i] = e * (1 - uk) % R_MOD
            nxt[2 * i + 1] = e * uk % R_MOD
        eq = nxt
    out = np.empty(len(eq), dtype=object)
    out[:] = eq
    return out


def mle_eval(table, u):
    """S~(u) = sum_b S(b) beta~(u, b)  (Eq. multilinear-extension)."""
    table = np.asarray(table, dtype=object).reshape(-1)
    assert table.shape[0] == 1 << len(u)
    return int(np.sum(table * beta_table(u)) % R_MOD)


def partial_eval(table, shape, axis_lo, axis_hi, point):
    """Bind the variables of axes [axis_lo, axis_hi) to `point`.

    out[o, i] = sum_a beta~(point, a) * T[o, a, i] over the view
    (outer, contracted axes, inner).  Returns (flat object array, new shape).
    """
    shape = [int(s) for s in shape]
    outer = int(np.prod(shape[:axis_lo], dtype=object)) if axis_lo > 0 else 1
    mid = int(np.prod(shape[axis_lo:axis_hi], dtype=object)) if axis_hi > axis_lo else 1
    inner = int(np.prod(shape[axis_hi:], dtype=object)) if axis_hi < len(shape) else 1
    assert len(point) == sum(ilog2(s) for s in shape[axis_lo:axis_hi])
    t = np.asarray(table, dtype=object).reshape(outer, mid, inner)
    beta = beta_table(point).reshape(1, mid, 1)
    out = np.sum(t * beta, axis=1) % R_MOD
    return out.reshape(-1), shape[:axis_lo] + shape[axis_hi:]


def fold(table, v):
    """Bind variable 0 to v: T'[b] = T[b] + v (T[b + len/2] - T[b])."""
    table = np.asarray(table, dtype=object).reshape(-1)
    half = table.shape[0] // 2
    lo, hi = table[:half], table[half:]
    return (lo + v * (hi - lo)) % R_MOD
