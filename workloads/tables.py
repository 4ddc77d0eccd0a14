"""Uniformly random elements of the BLS12-381 scalar field as 4 x u64 limbs.

Drawn by rejection: 255 uniform bits per candidate (PCG64), candidates not below
the modulus are redrawn.  The output is canonical little-endian, so
`arr.tobytes()` is the 32-byte-per-element encoding both provers accept.
No modular arithmetic is done here.
"""
import numpy as np

CONFIG_SEED = 2307162730          # + config index (+ step index inside a window)

# the modulus as four little-endian 64-bit limbs (public constant of the curve)
_R_LIMBS = np.array([0xFFFFFFFF00000001, 0x53BDA402FFFE5BFE,
                     0x3339D80809A1D805, 0x73EDA753299D7D48], dtype=np.uint64)


def _below_modulus(x):
    """Row-wise x < r for an [n,4] little-endian limb array."""
    lt = np.zeros(x.shape[0], dtype=bool)
    eq = np.ones(x.shape[0], dtype=bool)
    for k in (3, 2, 1, 0):
        lt |= eq & (x[:, k] < _R_LIMBS[k])
        eq &= x[:, k] == _R_LIMBS[k]
    return lt


def uniform_fr_limbs(rng, n):
    """[n,4] uint64, each row a uniform element of [0, r), little-endian limbs."""
    out = rng.integers(0, 1 << 64, size=(n, 4), dtype=np.uint64, endpoint=False)
    out[:, 3] &= np.uint64((1 << 63) - 1)
    bad = np.flatnonzero(~_below_modulus(out))
    while bad.size:
        redo = rng.integers(0, 1 << 64, size=(bad.size, 4), dtype=np.uint64, endpoint=False)
        redo[:, 3] &= np.uint64((1 << 63) - 1)
        out[bad] = redo
        bad = bad[~_below_modulus(redo)]
    return out
