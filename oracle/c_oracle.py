"""Loader for the C tier of the CPU oracle (oracle/c/zkdl_oracle.c).

The C tier computes the product sumcheck (Sec. 2.2) and the partial evaluation of a
multilinear extension (Eq. multilinear-extension) for inputs too large for the
Python-integer tier; it is pinned byte for byte against that tier on small inputs.
Test infrastructure; not used by the product.
"""
import ctypes as C
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "c", "zkdl_oracle.c")
LIB = os.path.join(HERE, "c", "libzkdl_oracle.so")
_lib = None


def build(force=False):
    """gcc -O2 -fopenmp -shared; rebuilt when the source is newer than the library."""
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", LIB, SRC])
    return LIB


def load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.zko_threads.restype = C.c_int
    return _lib


def threads():
    return int(load().zko_threads())


def fe_mul(a, b):
    out = C.create_string_buffer(32)
    load().zko_fe_mul(int(a).to_bytes(32, "little"), int(b).to_bytes(32, "little"), out)
    return int.from_bytes(out.raw, "little")


def sha256(data):
    out = C.create_string_buffer(32)
    load().zko_sha256(bytes(data), C.c_uint64(len(data)), out)
    return out.raw


def partial_eval(src_le, outer, axis, inner, point):
    """src_le: outer*axis*inner canonical 32-byte elements; point: log2(axis) integers.
    Returns outer*inner elements as bytes."""
    out = C.create_string_buffer(32 * outer * inner)
    pt = b"".join(int(v).to_bytes(32, "little") for v in point)
    rc = load().zko_partial_eval(bytes(src_le) if not isinstance(src_le, (bytes, bytearray)) else src_le,
                                 C.c_uint64(outer), C.c_uint64(axis), C.c_uint64(inner), pt, out)
    assert rc == 0, rc
    return out.raw


def product_prove(tables_le, seed):
    """tables_le: K byte strings of n canonical 32-byte elements.  Returns
    (proof bytes, challenges as integers, transcript digest)."""
    k = len(tables_le)
    n = len(tables_le[0]) // 32
    d = n.bit_length() - 1
    assert n == 1 << d and all(len(t) == 32 * n for t in tables_le)
    keep = [C.create_string_buffer(bytes(t), len(t)) if not isinstance(t, bytes) else t for t in tables_le]
    arr = (C.c_char_p * k)(*[C.cast(C.c_char_p(t) if isinstance(t, bytes) else t, C.c_char_p) for t in keep])
    proof = C.create_string_buffer(16 + 32 * (1 + d * (k + 1) + k))
    chal = C.create_string_buffer(max(32 * d, 1))
    digest = C.create_string_buffer(32)
    rc = load().zko_product_prove(arr, C.c_int(k), C.c_uint64(n), C.c_uint64(seed), proof, chal, digest)
    assert rc == 0, f"C oracle: product sumcheck failed its own check ({rc})"
    vs = [int.from_bytes(chal.raw[32 * i:32 * i + 32], "little") for i in range(d)]
    return proof.raw, vs, digest.raw
