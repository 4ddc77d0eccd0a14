"""Arithmetic in F = Z/rZ, r the BLS12-381 scalar-field prime (Sec. 2.4, Sec. 6).

Elements are Python ints in [0, r).  A signed integer x (a quantised real,
Sec. 2.2) maps to x mod r, so negatives appear as r - |x|.
Test infrastructure; not used by the product.
"""
import numpy as np

R_MOD = 0x73EDA753299D7D483339D80809A1D80553BDA402FFFE5BFEFFFFFFFF00000001
FR_BYTES = 32


def fr(x):
    """Signed or unsigned integer -> canonical representative in [0, r)."""
    return int(x) % R_MOD


def inv(x):
    x = int(x) % R_MOD
    if x == 0:
        raise ZeroDivisionError("0 has no inverse in F")
    return pow(x, -1, R_MOD)


def to_le(x):
    """Canonical 32-byte little-endian encoding of a reduced element."""
    x = int(x)
    assert 0 <= x < R_MOD
    return x.to_bytes(FR_BYTES, "little")


def from_le(b):
    x = int.from_bytes(bytes(b), "little")
    assert x < R_MOD, "non-canonical field element"
    return x


def fr_array(values):
    """Flat object array of canonical field elements from any integer array."""
    flat = np.asarray(values).reshape(-1)
    out = np.empty(flat.shape[0], dtype=object)
    for k, x in enumerate(flat.tolist()):
        out[k] = int(x) % R_MOD
    return out


def fr_array_from_le(buf, count):
    """`count` canonical 32-byte little-endian elements -> object array."""
    buf = bytes(buf)
    assert len(buf) == count * FR_BYTES
    out = np.empty(count, dtype=object)
    for k in range(count):
        out[k] = from_le(buf[k * FR_BYTES:(k + 1) * FR_BYTES])
    return out


def array_to_le(arr):
    return b"".join(to_le(x) for x in np.asarray(arr, dtype=object).reshape(-1).tolist())
