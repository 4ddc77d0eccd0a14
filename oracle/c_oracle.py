"""Loader for the C tier of the CPU oracle (oracle/c/zkdl_oracle.c).

The C tier redoes, for inputs too large for the Python-integer tier, the product sumcheck
(Sec. 2.2), the partial evaluation of a multilinear extension (Eq. multilinear-extension) and
the provers of the matrix product (Eq. exm-matmul-batched), the Hadamard product
(Eq. exm-hadamard-batched), zkReLU (App. A), re-indexing (Eq. sc-reindex), the merge of claims
on a stack and the aggregated window (Sec. 5, Protocol zkdl); it is pinned byte for byte against
the Python tier on small inputs.
Test infrastructure; not used by the product.
"""
import ctypes as C
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "c", "zkdl_oracle.c")
LIB = os.path.join(HERE, "c", "libzkdl_oracle.so")
_lib = None

ERRORS = {-1: "bad argument", -2: "out of memory", -3: "a consistency check of the prover failed",
          -4: "proof buffer too small", -5: "a zkReLU input is not a (Q+R)-bit signed integer"}


def build(force=False):
    """gcc -O3 -fopenmp -shared; rebuilt when the source is newer than the library."""
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.check_call(["gcc", "-O3", "-fopenmp", "-shared", "-fPIC", "-o", LIB, SRC])
    return LIB


class _Witness(C.Structure):
    _fields_ = [("L", C.c_uint32), ("B", C.c_uint32), ("width", C.c_uint32), ("T", C.c_uint32),
                ("Q", C.c_uint32), ("R", C.c_uint32),
                ("A", C.c_void_p), ("W", C.c_void_p), ("GZ", C.c_void_p), ("Zr", C.c_void_p), ("GA", C.c_void_p)]


PROGRESS_FN = C.CFUNCTYPE(None, C.c_char_p, C.c_int, C.c_int)


def load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.zko_threads.restype = C.c_int
        _lib.zko_set_threads.restype = C.c_int
        _lib.zko_ts_new.restype = C.c_void_p
        _lib.zko_ts_new.argtypes = [C.c_uint64]
        _lib.zko_ts_free.argtypes = [C.c_void_p]
        _lib.zko_ts_absorb.argtypes = [C.c_void_p, C.c_char_p, C.c_char_p, C.c_uint64]
        _lib.zko_ts_draw.argtypes = [C.c_void_p, C.c_int, C.c_char_p]
        _lib.zko_ts_digest.argtypes = [C.c_void_p, C.c_char_p]
        _lib.zko_ts_nchal.restype = C.c_uint64
        _lib.zko_ts_nchal.argtypes = [C.c_void_p]
        _lib.zko_ts_challenges.argtypes = [C.c_void_p, C.c_char_p]
        _lib.zko_set_progress.argtypes = [C.c_void_p]
    return _lib


def threads():
    return int(load().zko_threads())


def set_threads(n):
    """Number of OpenMP threads for the calls that follow; returns the value in force."""
    return int(load().zko_set_threads(C.c_int(n)))


_progress_keep = None


def set_progress(fn):
    """fn(what: str, round: int, rounds: int) is called at the start of every sumcheck round
    (None switches it off)."""
    global _progress_keep
    if fn is None:
        _progress_keep = None
        load().zko_set_progress(None)
        return
    _progress_keep = PROGRESS_FN(lambda what, t, d: fn(what.decode(), t, d))
    load().zko_set_progress(C.cast(_progress_keep, C.c_void_p))


def fe_mul(a, b):
    out = C.create_string_buffer(32)
    load().zko_fe_mul(int(a).to_bytes(32, "little"), int(b).to_bytes(32, "little"), out)
    return int.from_bytes(out.raw, "little")


def fe_add(a, b):
    out = C.create_string_buffer(32)
    load().zko_fe_add(int(a).to_bytes(32, "little"), int(b).to_bytes(32, "little"), out)
    return int.from_bytes(out.raw, "little")


def fe_sub(a, b):
    out = C.create_string_buffer(32)
    load().zko_fe_sub(int(a).to_bytes(32, "little"), int(b).to_bytes(32, "little"), out)
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


class Transcript:
    """The C tier's transcript object (same stream format as oracle.transcript.Transcript)."""

    def __init__(self, seed=0):
        self._lib = load()
        self._h = self._lib.zko_ts_new(C.c_uint64(seed))
        assert self._h

    def __del__(self):
        if getattr(self, "_h", None):
            self._lib.zko_ts_free(self._h)
            self._h = None

    def absorb(self, label, data):
        data = bytes(data)
        rc = self._lib.zko_ts_absorb(self._h, bytes(label), data, C.c_uint64(len(data)))
        assert rc == 0, ERRORS.get(rc, rc)

    def challenges_vec(self, n):
        out = C.create_string_buffer(max(32 * n, 1))
        rc = self._lib.zko_ts_draw(self._h, C.c_int(n), out)
        assert rc == 0, ERRORS.get(rc, rc)
        return [int.from_bytes(out.raw[32 * i:32 * i + 32], "little") for i in range(n)]

    def digest(self):
        out = C.create_string_buffer(32)
        self._lib.zko_ts_digest(self._h, out)
        return out.raw

    @property
    def challenges(self):
        """Every challenge drawn so far, in order."""
        n = int(self._lib.zko_ts_nchal(self._h))
        out = C.create_string_buffer(max(32 * n, 1))
        self._lib.zko_ts_challenges(self._h, out)
        return [int.from_bytes(out.raw[32 * i:32 * i + 32], "little") for i in range(n)]


class OracleError(Exception):
    def __init__(self, rc):
        super().__init__(f"C oracle: {ERRORS.get(rc, rc)}")
        self.rc = rc


def _run(fn, *args, cap=1 << 20):
    proof = C.create_string_buffer(cap)
    plen = C.c_uint64(0)
    rc = fn(*args, proof, C.c_uint64(cap), C.byref(plen))
    if rc != 0:
        raise OracleError(rc)
    return proof.raw[:plen.value]


def _le(values):
    return b"".join(int(v).to_bytes(32, "little") for v in values)


def matmul_prove(x0_le, shape0, x1_le, shape1, ts):
    """x0_le [N,D1,D2], x1_le [N,D2,D3] as canonical 32-byte elements.  Returns the proof bytes."""
    n, d1, d2 = shape0
    n_, d2_, d3 = shape1
    assert n == n_ and d2 == d2_
    return _run(load().zko_matmul_prove, bytes(x0_le), bytes(x1_le), C.c_uint64(n), C.c_uint64(d1),
                C.c_uint64(d2), C.c_uint64(d3), C.c_void_p(ts._h))


def matmul_ft_prove(x0_le, shape0, x1_le, shape1, ts):
    """The same product with the messages of the optimized aggregated protocol (App. B)."""
    n, d1, d2 = shape0
    n_, d2_, d3 = shape1
    assert n == n_ and d2 == d2_
    return _run(load().zko_matmul_ft_prove, bytes(x0_le), bytes(x1_le), C.c_uint64(n), C.c_uint64(d1),
                C.c_uint64(d2), C.c_uint64(d3), C.c_void_p(ts._h))


def hadamard_prove(x0_le, x1_le, ts):
    n = len(x0_le) // 32
    d = n.bit_length() - 1
    assert n == 1 << d and len(x1_le) == len(x0_le)
    return _run(load().zko_hadamard_prove, bytes(x0_le), bytes(x1_le), C.c_int(d), C.c_void_p(ts._h))


def _i64(values):
    return np.ascontiguousarray(np.asarray(values, dtype=np.int64).reshape(-1))


def zkrelu_prove(z, ga, q, r_bits, ts, points=None, bind_points=True):
    """z, ga: integer arrays (ga None: forward only); points: None or the four points as lists of
    integers.  Returns the proof bytes; OracleError(-5) on a value out of range."""
    zz = _i64(z)
    gg = _i64(ga) if ga is not None else None
    pts = _le([x for pt in points for x in pt]) if points is not None else None
    return _run(load().zko_zkrelu_prove, zz.ctypes.data_as(C.c_void_p),
                gg.ctypes.data_as(C.c_void_p) if gg is not None else None, C.c_uint64(zz.shape[0]),
                C.c_int(q), C.c_int(r_bits), pts, C.c_int(1 if bind_points else 0), C.c_void_p(ts._h))


def update_prove(gw, q, r_bits, ts):
    """gw: integer array, a power of two of entries.  Returns the proof bytes (oracle.protocols.update_prove)."""
    gg = _i64(gw)
    return _run(load().zko_update_prove, gg.ctypes.data_as(C.c_void_p), C.c_uint64(gg.shape[0]), C.c_int(q),
                C.c_int(r_bits), C.c_void_p(ts._h))


def reindex_prove(x_le, n, d, maps, points, u, ts, bind_statement=True):
    k = len(maps)
    marr = [np.ascontiguousarray(np.asarray(m, dtype=np.int32)) for m in maps]
    mp = (C.c_void_p * k)(*[m.ctypes.data for m in marr])
    ml = (C.c_uint64 * k)(*[len(m) for m in maps])
    pbytes = [C.create_string_buffer(_le(pt), max(32 * len(pt), 1)) for pt in points]
    pp = (C.c_void_p * k)(*[C.addressof(b) for b in pbytes])
    ub = C.create_string_buffer(_le(u), max(32 * len(u), 1))
    return _run(load().zko_reindex_prove, bytes(x_le), C.c_uint64(n), C.c_uint64(d), C.c_int(k), mp, ml, pp, ub,
                C.c_int(1 if bind_statement else 0), C.c_void_p(ts._h))


def stack_merge_prove(x_le, n, d, points, ts, bind_statement=True):
    k = len(points)
    pbytes = [C.create_string_buffer(_le(pt), max(32 * len(pt), 1)) for pt in points]
    pp = (C.c_void_p * k)(*[C.addressof(b) for b in pbytes])
    return _run(load().zko_stack_merge_prove, bytes(x_le), C.c_uint64(n), C.c_uint64(d), C.c_int(k), pp,
                C.c_int(1 if bind_statement else 0), C.c_void_p(ts._h))


def _witness(wit):
    keep = dict(A=np.ascontiguousarray(wit["A"], dtype=np.int32), W=np.ascontiguousarray(wit["W"], dtype=np.int32),
                GZ=np.ascontiguousarray(wit["GZ"], dtype=np.int32), Zr=np.ascontiguousarray(wit["Zr"], dtype=np.int64),
                GA=np.ascontiguousarray(wit["GA"], dtype=np.int64))
    w = _Witness(wit["L"], wit["B"], wit["width"], wit["T"], wit["Q"], wit["R"],
                 *[keep[k].ctypes.data for k in ("A", "W", "GZ", "Zr", "GA")])
    return w, keep


def aggregate_prove(wit, ts, linked=False, ft=False):
    """wit as oracle.protocols.aggregate_prove takes it (integer stacks).  Returns the proof bytes.
    linked: aggregate_linked_prove; ft: aggregate_ft_prove."""
    assert not (linked and ft)
    w, keep = _witness(wit)
    fn = load().zko_aggregate_linked_prove if linked else load().zko_aggregate_ft_prove if ft else load().zko_aggregate_prove
    out = _run(fn, C.byref(w), C.c_void_p(ts._h))
    del keep
    return out
