"""ctypes binding of libzkdl.so; argument marshalling only."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

ZKDL_I32, ZKDL_I64, ZKDL_FR_LE = 0, 1, 2
ERRORS = {0: "ok", -1: "ZKDL_EINVAL", -2: "ZKDL_ERANGE", -3: "ZKDL_ENOMEM", -4: "ZKDL_EHIP",
          -5: "ZKDL_ESMALL", -6: "ZKDL_ETOOBIG"}

EXPORTED_SYMBOLS = [
    "zkdl_ctx_create", "zkdl_ctx_destroy", "zkdl_last_hip_error", "zkdl_strerror", "zkdl_ctx_trim",
    "zkdl_ctx_set_fill_threads", "zkdl_ctx_set_commit_window_bits",
    "zkdl_transcript_create", "zkdl_transcript_destroy", "zkdl_transcript_absorb",
    "zkdl_transcript_challenge", "zkdl_transcript_digest",
    "fr_tensor_upload", "zkdl_tensor_wrap_int", "zkdl_tensor_ndim", "zkdl_tensor_dim",
    "zkdl_tensor_numel", "zkdl_tensor_download", "zkdl_tensor_free",
    "mle_partial_eval", "sumcheck_product", "sumcheck_product_noalloc", "sumcheck_matmul", "sumcheck_matmul_ft", "sumcheck_matmul_general", "update_prove", "hyrax_verify", "sumcheck_hadamard",
    "reindex_prove", "claims_merge_prove", "claims_merge_stack_prove", "zkrelu_prove", "zkrelu_prove_at", "aggregate_prove", "aggregate_prove_linked", "aggregate_prove_ft", "zkdl_host_fr_mul", "zkdl_selfcheck_constants", "zkdl_host_scalar_split",
    "zkdl_ctx_profile_enable", "zkdl_ctx_profile_reset", "zkdl_ctx_profile_read", "zkdl_selfbench",
    "zkdl_commit_key_create", "zkdl_commit_key_destroy", "zkdl_commit_key_generators", "hyrax_commit", "hyrax_open",
    "zkdl_commit_selfcheck", "aggregate_verify", "zkdl_host_aggregate_verify",
]

PROF_CLASSES = {"sc_round_fused": 0, "sc_round_first": 1, "partial_eval": 2, "zk_bin": 3, "zk_lin": 4,
                "finalise": 5}


class ZkdlError(RuntimeError):
    def __init__(self, code, where, hip=0):
        self.code = code
        self.hip = hip
        super().__init__(f"{where}: {ERRORS.get(code, code)}" + (f" (hip error {hip})" if hip else ""))


class FcnnWitness(C.Structure):
    _fields_ = [("L", C.c_uint32), ("B", C.c_uint32), ("width", C.c_uint32), ("T", C.c_uint32),
                ("Q", C.c_uint32), ("R", C.c_uint32),
                ("A", C.c_void_p), ("W", C.c_void_p), ("GZ", C.c_void_p), ("Zr", C.c_void_p),
                ("GA", C.c_void_p)]


class Claim(C.Structure):
    _fields_ = [("tensor", C.c_uint32), ("nseg", C.c_uint32), ("seg_off", C.c_uint32 * 4),
                ("seg_len", C.c_uint32 * 4), ("value", C.c_uint8 * 32)]


CLAIM_TENSORS = ["A", "W", "GZ", "Z", "ZR", "GA", "GW", "A_RELU", "GZ_RELU", "GZ_NEXT", "W_NEXT", "AUX",
                 "Z_LAST", "GZ_LAST", "U"]


def library_path():
    return os.path.join(_HERE, "libzkdl.so")


def load_library():
    """Loads libzkdl.so; raises if it has not been built (there is no fallback)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "or `python paper_2307_16273_amd/build.py`")
    lib = C.CDLL(path)
    vp, i, u64, sz = C.c_void_p, C.c_int, C.c_uint64, C.c_size_t
    pp = C.POINTER(vp)
    psz = C.POINTER(sz)
    sig = {
        "zkdl_ctx_create": [pp, i, vp], "zkdl_ctx_destroy": [vp], "zkdl_last_hip_error": [vp],
        "zkdl_ctx_trim": [vp], "zkdl_ctx_set_fill_threads": [vp, u64],
        "zkdl_ctx_set_commit_window_bits": [vp, i],
        "zkdl_transcript_create": [pp, u64], "zkdl_transcript_destroy": [vp],
        "zkdl_transcript_absorb": [vp, C.c_char_p, vp, sz], "zkdl_transcript_challenge": [vp, vp],
        "zkdl_transcript_digest": [vp, vp],
        "fr_tensor_upload": [vp, vp, i, i, C.POINTER(u64), i, pp],
        "zkdl_tensor_wrap_int": [vp, vp, i, C.POINTER(u64), i, pp],
        "zkdl_tensor_ndim": [vp], "zkdl_tensor_download": [vp, vp, vp], "zkdl_tensor_free": [vp, vp],
        "mle_partial_eval": [vp, vp, i, i, vp, sz, pp],
        "sumcheck_product": [vp, pp, i, vp, vp, psz, vp, vp, psz],
        "sumcheck_product_noalloc": [vp, pp, i, vp, vp, psz, vp, vp, psz],
        "sumcheck_matmul": [vp, vp, vp, i, i, vp, vp, psz, vp, vp, psz],
        "sumcheck_matmul_ft": [vp, vp, vp, i, i, vp, vp, psz, vp, vp, psz],
        "sumcheck_matmul_general": [vp, vp, vp, vp, vp, vp, psz, vp, vp, psz],
        "sumcheck_hadamard": [vp, vp, vp, vp, vp, psz, vp, vp, psz],
        "reindex_prove": [vp, vp, i, pp, C.POINTER(u64), pp, vp, vp, vp, psz, vp, vp, psz],
        "claims_merge_prove": [vp, vp, i, pp, vp, vp, psz, vp, vp, psz],
        "claims_merge_stack_prove": [vp, vp, i, pp, vp, vp, psz, vp, vp, psz],
        "zkrelu_prove": [vp, vp, vp, u64, i, i, i, vp, vp, psz, vp, vp, psz],
        "zkrelu_prove_at": [vp, vp, vp, u64, i, i, i, vp, vp, vp, psz, vp, vp, psz],
        "aggregate_prove": [vp, C.POINTER(FcnnWitness), vp, vp, psz, vp, psz, vp, psz],
        "update_prove": [vp, vp, u64, i, i, i, vp, vp, psz, vp, psz, vp, psz],
        "aggregate_prove_linked": [vp, C.POINTER(FcnnWitness), vp, vp, psz, vp, psz, vp, psz],
        "aggregate_prove_ft": [vp, C.POINTER(FcnnWitness), vp, vp, psz, vp, psz],
        "zkdl_host_fr_mul": [vp, vp, vp], "zkdl_selfcheck_constants": [],
        "zkdl_host_scalar_split": [vp, vp],
        "zkdl_ctx_profile_enable": [vp, i], "zkdl_ctx_profile_reset": [vp],
        "zkdl_ctx_profile_read": [vp, i, C.POINTER(u64), C.POINTER(C.c_double), C.POINTER(C.c_double)],
        "zkdl_selfbench": [vp, i, u64, C.POINTER(C.c_double), C.POINTER(C.c_double)],
        "zkdl_commit_key_create": [vp, C.c_char_p, u64, i, pp], "zkdl_commit_key_destroy": [vp, vp],
        "zkdl_commit_key_generators": [vp, vp, u64, u64, vp],
        "hyrax_commit": [vp, vp, vp, vp, vp, psz], "hyrax_open": [vp, vp, vp, vp, sz, vp, vp, vp],
        "hyrax_verify": [vp, vp, vp, sz, vp, sz, vp, vp, vp, vp, vp],
        "zkdl_commit_selfcheck": [],
        "aggregate_verify": [vp, vp, sz, vp, C.POINTER(i), vp, psz, vp, psz],
        "zkdl_host_aggregate_verify": [vp, sz, vp, C.POINTER(i), vp, psz, vp, psz],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = i
    lib.zkdl_strerror.argtypes = [i]
    lib.zkdl_strerror.restype = C.c_char_p
    lib.zkdl_tensor_dim.argtypes = [vp, i]
    lib.zkdl_tensor_dim.restype = u64
    lib.zkdl_tensor_numel.argtypes = [vp]
    lib.zkdl_tensor_numel.restype = u64
    _LIB = lib
    return lib


def _check(rc, where, ctx=None):
    if rc != 0:
        hip = load_library().zkdl_last_hip_error(ctx.handle) if (ctx is not None and rc == -4) else 0
        raise ZkdlError(rc, where, hip)


PROOF_CAP = 1 << 17
POINTS_CAP = 1024


class Context:
    """Device context on the current PyTorch stream of `device`."""

    def __init__(self, device=0, stream=None):
        import torch
        lib = load_library()
        if stream is None:
            stream = torch.cuda.current_stream(device).cuda_stream
        self.handle = C.c_void_p()
        self.device = device
        _check(lib.zkdl_ctx_create(C.byref(self.handle), device, C.c_void_p(stream)), "zkdl_ctx_create")

    def profile(self, on=True, reset=True):
        """Per-kernel-class HIP-event timing on this context's stream."""
        lib = load_library()
        if reset:
            _check(lib.zkdl_ctx_profile_reset(self.handle), "zkdl_ctx_profile_reset", self)
        _check(lib.zkdl_ctx_profile_enable(self.handle, int(on)), "zkdl_ctx_profile_enable", self)

    def profile_read(self):
        lib = load_library()
        out = {}
        for name, cls in PROF_CLASSES.items():
            n, ms, by = C.c_uint64(), C.c_double(), C.c_double()
            _check(lib.zkdl_ctx_profile_read(self.handle, cls, C.byref(n), C.byref(ms), C.byref(by)),
                   "zkdl_ctx_profile_read", self)
            out[name] = dict(launches=n.value, ms=ms.value, bytes=by.value)
        return out

    def selfbench(self, what, work):
        """One machine probe ("copy": bytes, "mad" / "modmul": loop count); returns units per second."""
        units, secs = C.c_double(), C.c_double()
        code = {"copy": 0, "mad": 1, "modmul": 2}[what]
        _check(load_library().zkdl_selfbench(self.handle, code, int(work), C.byref(units), C.byref(secs)),
               "zkdl_selfbench", self)
        return units.value / secs.value

    def trim(self):
        _check(load_library().zkdl_ctx_trim(self.handle), "zkdl_ctx_trim", self)

    def set_fill_threads(self, threads):
        _check(load_library().zkdl_ctx_set_fill_threads(self.handle, int(threads)), "zkdl_ctx_set_fill_threads", self)

    def set_commit_window_bits(self, bits):
        _check(load_library().zkdl_ctx_set_commit_window_bits(self.handle, int(bits)),
               "zkdl_ctx_set_commit_window_bits", self)

    def close(self):
        if self.handle:
            load_library().zkdl_ctx_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Transcript:
    def __init__(self, seed=0):
        self.handle = C.c_void_p()
        _check(load_library().zkdl_transcript_create(C.byref(self.handle), seed), "zkdl_transcript_create")

    def absorb(self, label, data):
        data = bytes(data)
        buf = C.create_string_buffer(data, len(data))
        _check(load_library().zkdl_transcript_absorb(self.handle, bytes(label), buf, len(data)),
               "zkdl_transcript_absorb")

    def challenge(self):
        out = C.create_string_buffer(32)
        _check(load_library().zkdl_transcript_challenge(self.handle, out), "zkdl_transcript_challenge")
        return int.from_bytes(out.raw, "little")

    def digest(self):
        out = C.create_string_buffer(32)
        _check(load_library().zkdl_transcript_digest(self.handle, out), "zkdl_transcript_digest")
        return out.raw

    def __del__(self):
        try:
            if self.handle:
                load_library().zkdl_transcript_destroy(self.handle)
                self.handle = C.c_void_p()
        except Exception:
            pass


class FrTensor:
    def __init__(self, ctx, handle, keepalive=None):
        self.ctx = ctx
        self.handle = handle
        self._keepalive = keepalive

    @property
    def shape(self):
        lib = load_library()
        return tuple(int(lib.zkdl_tensor_dim(self.handle, a)) for a in range(lib.zkdl_tensor_ndim(self.handle)))

    @property
    def numel(self):
        return int(load_library().zkdl_tensor_numel(self.handle))

    def download(self):
        """Canonical little-endian bytes, numel x 32."""
        out = np.empty(self.numel * 32, dtype=np.uint8)
        _check(load_library().zkdl_tensor_download(self.ctx.handle, self.handle, out.ctypes.data),
               "zkdl_tensor_download", self.ctx)
        return out.tobytes()

    def free(self):
        if self.handle:
            load_library().zkdl_tensor_free(self.ctx.handle, self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def _shape_arr(shape):
    return (C.c_uint64 * len(shape))(*[int(s) for s in shape]), len(shape)


def _src_pointer(src):
    """(pointer, on_device, dtype code, keepalive) for a numpy array, bytes or torch tensor."""
    try:
        import torch
        is_torch = isinstance(src, torch.Tensor)
    except ImportError:
        is_torch = False
    if is_torch:
        import torch
        assert src.is_contiguous()
        code = {torch.int32: ZKDL_I32, torch.int64: ZKDL_I64, torch.uint8: ZKDL_FR_LE}[src.dtype]
        return src.data_ptr(), 1 if src.is_cuda else 0, code, src
    if isinstance(src, (bytes, bytearray)):
        arr = np.frombuffer(bytes(src), dtype=np.uint8)
        return arr.ctypes.data, 0, ZKDL_FR_LE, arr
    arr = np.ascontiguousarray(src)
    code = {np.dtype(np.int32): ZKDL_I32, np.dtype(np.int64): ZKDL_I64, np.dtype(np.uint8): ZKDL_FR_LE,
            np.dtype(np.uint64): ZKDL_FR_LE}[arr.dtype]
    return arr.ctypes.data, 0, code, arr


def fr_tensor_upload(ctx, src, shape):
    """int32 / int64 (signed, x mod r) or raw 32-byte little-endian elements
    (uint8 / uint64 arrays, bytes) -> Fr tensor on the device."""
    ptr, on_dev, code, keep = _src_pointer(src)
    sh, nd = _shape_arr(shape)
    out = C.c_void_p()
    _check(load_library().fr_tensor_upload(ctx.handle, ptr, code, on_dev, sh, nd, C.byref(out)),
           "fr_tensor_upload", ctx)
    return FrTensor(ctx, out)


def tensor_wrap_int(ctx, torch_tensor, shape=None):
    """A no-copy view of an int32/int64 CUDA tensor (kept alive by the result)."""
    ptr, on_dev, code, keep = _src_pointer(torch_tensor)
    assert on_dev and code in (ZKDL_I32, ZKDL_I64)
    sh, nd = _shape_arr(shape if shape is not None else tuple(torch_tensor.shape))
    out = C.c_void_p()
    _check(load_library().zkdl_tensor_wrap_int(ctx.handle, ptr, code, sh, nd, C.byref(out)),
           "zkdl_tensor_wrap_int", ctx)
    return FrTensor(ctx, out, keepalive=keep)


def _fr_bytes(values):
    return b"".join(int(v).to_bytes(32, "little") for v in values)


def _split_fr(buf, n):
    return [int.from_bytes(buf[32 * k:32 * k + 32], "little") for k in range(n)]


def mle_partial_eval(ctx, t, axis_lo, axis_hi, point):
    pb = _fr_bytes(point)
    buf = C.create_string_buffer(pb, max(len(pb), 1))
    out = C.c_void_p()
    _check(load_library().mle_partial_eval(ctx.handle, t.handle, axis_lo, axis_hi, buf, len(point),
                                           C.byref(out)), "mle_partial_eval", ctx)
    return FrTensor(ctx, out)


class _Outputs:
    """Output buffers of one call.  The two large ones belong to the context and are reused from call to call
    (result() copies what the call wrote out of them before the next call can run)."""

    def __init__(self, ctx, n_claims):
        if getattr(ctx, "_out_bufs", None) is None:
            ctx._out_bufs = (C.create_string_buffer(PROOF_CAP), C.create_string_buffer(32 * POINTS_CAP))
        self.proof, self.points = ctx._out_bufs
        self.proof_len = C.c_size_t(PROOF_CAP)
        self.claims = C.create_string_buffer(32 * max(n_claims, 1))
        self.npoints = C.c_size_t(POINTS_CAP)
        self.n_claims = n_claims

    def result(self):
        return dict(proof=C.string_at(self.proof, self.proof_len.value),
                    claims=_split_fr(self.claims.raw, self.n_claims),
                    points=_split_fr(C.string_at(self.points, 32 * self.npoints.value), self.npoints.value))


def sumcheck_product(ctx, tables, tr, noalloc=False):
    """noalloc: the entry point that allocates nothing (Fr tables of at most 2^18 entries)."""
    k = len(tables)
    arr = (C.c_void_p * k)(*[t.handle for t in tables])
    o = _Outputs(ctx, k)
    name = "sumcheck_product_noalloc" if noalloc else "sumcheck_product"
    _check(getattr(load_library(), name)(ctx.handle, arr, k, tr.handle, o.proof, C.byref(o.proof_len),
                                         o.claims, o.points, C.byref(o.npoints)), name, ctx)
    return o.result()


def sumcheck_matmul(ctx, x0, x1, tr, transpose_x0=False, transpose_x1=False):
    o = _Outputs(ctx, 3)
    _check(load_library().sumcheck_matmul(ctx.handle, x0.handle, x1.handle, int(transpose_x0),
                                          int(transpose_x1), tr.handle, o.proof, C.byref(o.proof_len),
                                          o.claims, o.points, C.byref(o.npoints)), "sumcheck_matmul", ctx)
    return o.result()


def sumcheck_matmul_ft(ctx, x0, x1, tr, transpose_x0=False, transpose_x1=False):
    o = _Outputs(ctx, 3)
    _check(load_library().sumcheck_matmul_ft(ctx.handle, x0.handle, x1.handle, int(transpose_x0),
                                             int(transpose_x1), tr.handle, o.proof, C.byref(o.proof_len),
                                             o.claims, o.points, C.byref(o.npoints)), "sumcheck_matmul_ft", ctx)
    return o.result()


def sumcheck_matmul_general(ctx, x0, x1, y, tr):
    """claims: Y~, X0~, X1~ at the final points (the general aggregated form takes Y as a stack)."""
    o = _Outputs(ctx, 3)
    _check(load_library().sumcheck_matmul_general(ctx.handle, x0.handle, x1.handle, y.handle, tr.handle, o.proof,
                                                  C.byref(o.proof_len), o.claims, o.points, C.byref(o.npoints)),
           "sumcheck_matmul_general", ctx)
    return o.result()


def sumcheck_hadamard(ctx, x0, x1, tr):
    o = _Outputs(ctx, 3)
    _check(load_library().sumcheck_hadamard(ctx.handle, x0.handle, x1.handle, tr.handle, o.proof,
                                            C.byref(o.proof_len), o.claims, o.points, C.byref(o.npoints)),
           "sumcheck_hadamard", ctx)
    return o.result()


def reindex_prove(ctx, x, maps, points, u, tr):
    """x: tensor handle of the stack [N, ...]; maps: K sequences of stack indices (-1 = zero
    tensor); points: K lists of field elements (log2 len(maps[k]) each); u: log2(numel / N)."""
    k = len(maps)
    arrs = [np.ascontiguousarray(np.asarray(m, dtype=np.int32)) for m in maps]
    map_ptrs = (C.c_void_p * k)(*[a.ctypes.data for a in arrs])
    lens = (C.c_uint64 * k)(*[a.size for a in arrs])
    pbufs = [C.create_string_buffer(_fr_bytes(p), max(32 * len(p), 1)) for p in points]
    pt_ptrs = (C.c_void_p * k)(*[C.addressof(b) for b in pbufs])
    ub = C.create_string_buffer(_fr_bytes(u), max(32 * len(u), 1))
    o = _Outputs(ctx, k + 2)
    _check(load_library().reindex_prove(ctx.handle, x.handle, k, map_ptrs, lens, pt_ptrs, ub, tr.handle, o.proof,
                                        C.byref(o.proof_len), o.claims, o.points, C.byref(o.npoints)),
           "reindex_prove", ctx)
    return o.result()


def claims_merge_prove(ctx, x, points, tr, stack=False):
    """x: tensor handle (2^d elements); points: K lists of d field elements.  Returns the K claims,
    P~(v) and X~(v) in `claims`.  stack: x is a stack [N, ...] and the merge runs on tables of the
    inner size (claims_merge_stack_prove)."""
    k = len(points)
    name = "claims_merge_stack_prove" if stack else "claims_merge_prove"
    pbufs = [C.create_string_buffer(_fr_bytes(p), max(32 * len(p), 1)) for p in points]
    pt_ptrs = (C.c_void_p * k)(*[C.addressof(b) for b in pbufs])
    o = _Outputs(ctx, k + 2)
    _check(getattr(load_library(), name)(ctx.handle, x.handle, k, pt_ptrs, tr.handle, o.proof,
                                         C.byref(o.proof_len), o.claims, o.points, C.byref(o.npoints)),
           name, ctx)
    return o.result()


def zkrelu_prove(ctx, z, ga, tr, q=32, r=16, points=None):
    """z, ga: int64 numpy arrays (host) or int64 CUDA tensors; ga may be None.
    points: None, or the four points (u_Z, u_A, u_GA, u_GZ) as lists of field elements
    (zkrelu_prove_at)."""
    zp, z_dev, zc, zk_ = _src_pointer(z)
    assert zc == ZKDL_I64
    d = int(np.prod(z.shape))
    gp = None
    if ga is not None:
        gp, g_dev, gc, gk_ = _src_pointer(ga)
        assert gc == ZKDL_I64 and g_dev == z_dev
    o = _Outputs(ctx, 4)
    if points is not None:
        assert len(points) == 4
        flat = [x for pt in points for x in pt]
        pb = C.create_string_buffer(_fr_bytes(flat), max(32 * len(flat), 1))
        _check(load_library().zkrelu_prove_at(ctx.handle, zp, gp, d, q, r, z_dev, pb, tr.handle, o.proof,
                                              C.byref(o.proof_len), o.claims, o.points, C.byref(o.npoints)),
               "zkrelu_prove_at", ctx)
        return o.result()
    _check(load_library().zkrelu_prove(ctx.handle, zp, gp, d, q, r, z_dev, tr.handle, o.proof,
                                       C.byref(o.proof_len), o.claims, o.points, C.byref(o.npoints)),
           "zkrelu_prove", ctx)
    return o.result()


def update_prove(ctx, gw, tr, q=32, r=30):
    """gw: int64 numpy array (host) or int64 CUDA tensor, a power of two of entries.  Returns proof, points and
    claims_left (U at p, GW, AUX)."""
    gp, g_dev, gc, keep = _src_pointer(gw)
    assert gc == ZKDL_I64
    d = int(np.prod(gw.shape))
    o = _Outputs(ctx, 0)
    claims = (Claim * 4)()
    nclaims = C.c_size_t(4)
    _check(load_library().update_prove(ctx.handle, gp, d, q, r, g_dev, tr.handle, o.proof, C.byref(o.proof_len),
                                       o.points, C.byref(o.npoints), claims, C.byref(nclaims)), "update_prove", ctx)
    out = o.result()
    pts = out["points"]
    out["claims_left"] = [
        dict(tensor=CLAIM_TENSORS[c.tensor],
             point=[x for s in range(c.nseg) for x in pts[c.seg_off[s]:c.seg_off[s] + c.seg_len[s]]],
             value=int.from_bytes(bytes(c.value), "little"))
        for c in claims[:nclaims.value]]
    return out


def aggregate_prove(ctx, wit, tr, linked=False, ft=False):
    """wit: dict with L, B, width, T, Q, R and CUDA tensors A, W, GZ (int32), Zr, GA (int64).
    linked: the claims of the four families chained (aggregate_prove_linked); ft: the matrix-product
    families in the optimized aggregated form (aggregate_prove_ft)."""
    import torch
    for k, dt in (("A", torch.int32), ("W", torch.int32), ("GZ", torch.int32), ("Zr", torch.int64),
                  ("GA", torch.int64)):
        assert wit[k].is_cuda and wit[k].dtype == dt and wit[k].is_contiguous()
    n = wit["L"] * wit["T"]
    assert wit["A"].numel() == n * wit["B"] * wit["width"] == wit["GZ"].numel() == wit["Zr"].numel() \
        == wit["GA"].numel() and wit["W"].numel() == n * wit["width"] ** 2
    w = FcnnWitness(wit["L"], wit["B"], wit["width"], wit["T"], wit["Q"], wit["R"],
                    wit["A"].data_ptr(), wit["W"].data_ptr(), wit["GZ"].data_ptr(), wit["Zr"].data_ptr(),
                    wit["GA"].data_ptr())
    o = _Outputs(ctx, 0)
    if ft:
        assert not linked
        _check(load_library().aggregate_prove_ft(ctx.handle, C.byref(w), tr.handle, o.proof, C.byref(o.proof_len),
                                                 o.points, C.byref(o.npoints)), "aggregate_prove_ft", ctx)
        return o.result()
    name = "aggregate_prove_linked" if linked else "aggregate_prove"
    claims = (Claim * 16)()
    nclaims = C.c_size_t(16)
    _check(getattr(load_library(), name)(ctx.handle, C.byref(w), tr.handle, o.proof, C.byref(o.proof_len),
                                         o.points, C.byref(o.npoints), claims, C.byref(nclaims)), name, ctx)
    out = o.result()
    pts = out["points"]
    out["claims_left"] = [
        dict(tensor=CLAIM_TENSORS[c.tensor],
             point=[x for s in range(c.nseg) for x in pts[c.seg_off[s]:c.seg_off[s] + c.seg_len[s]]],
             value=int.from_bytes(bytes(c.value), "little"))
        for c in claims[:nclaims.value]]
    return out


def host_fr_mul(a, b):
    out = C.create_string_buffer(32)
    _check(load_library().zkdl_host_fr_mul(C.create_string_buffer(int(a).to_bytes(32, "little"), 32),
                                           C.create_string_buffer(int(b).to_bytes(32, "little"), 32), out),
           "zkdl_host_fr_mul")
    return int.from_bytes(out.raw, "little")


def host_scalar_split(k):
    """(a, b) with k = a + b z^2, a < z^2 (the split hyrax_verify uses), by the library's host code."""
    out = C.create_string_buffer(32)
    _check(load_library().zkdl_host_scalar_split(C.create_string_buffer(int(k).to_bytes(32, "little"), 32), out),
           "zkdl_host_scalar_split")
    return int.from_bytes(out.raw[:16], "little"), int.from_bytes(out.raw[16:], "little")


def selfcheck_constants():
    return load_library().zkdl_selfcheck_constants()


class CommitKey:
    """Generators and window tables of the row-wise Pedersen commitment (device memory)."""

    def __init__(self, ctx, label, ncols, max_bits=32):
        self.ctx = ctx
        self.ncols = ncols
        self.handle = C.c_void_p()
        _check(load_library().zkdl_commit_key_create(ctx.handle, bytes(label), ncols, max_bits, C.byref(self.handle)),
               "zkdl_commit_key_create", ctx)

    def generators(self, first, count):
        """`count` generators from index `first` (index ncols is H), 96 bytes each."""
        out = C.create_string_buffer(96 * count)
        _check(load_library().zkdl_commit_key_generators(self.ctx.handle, self.handle, first, count, out),
               "zkdl_commit_key_generators", self.ctx)
        return [out.raw[96 * k:96 * k + 96] for k in range(count)]

    def close(self):
        if self.handle:
            load_library().zkdl_commit_key_destroy(self.ctx.handle, self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def hyrax_commit(ctx, key, x, blind=None):
    """x: an int32 / int64 tensor view; blind: None or one field element per row.  Returns the row
    commitments, 96 bytes each."""
    m = x.numel.bit_length() - 1
    rows = 1 << (m - m // 2)
    out = C.create_string_buffer(96 * rows)
    n = C.c_size_t(rows)
    bb = C.create_string_buffer(_fr_bytes(blind), 32 * rows) if blind is not None else None
    _check(load_library().hyrax_commit(ctx.handle, key.handle, x.handle, bb, out, C.byref(n)), "hyrax_commit", ctx)
    raw = out.raw   # one copy of the buffer, not one per row
    return [raw[96 * k:96 * k + 96] for k in range(n.value)]


def hyrax_open(ctx, x, blind, point):
    """Returns (T, rho*, y) as integers."""
    m = x.numel.bit_length() - 1
    rows, cols = 1 << (m - m // 2), 1 << (m // 2)
    t = C.create_string_buffer(32 * cols)
    rho, y = C.create_string_buffer(32), C.create_string_buffer(32)
    bb = C.create_string_buffer(_fr_bytes(blind), 32 * rows) if blind is not None else None
    pb = C.create_string_buffer(_fr_bytes(point), max(32 * len(point), 1))
    _check(load_library().hyrax_open(ctx.handle, x.handle, bb, pb, len(point), t, rho, y), "hyrax_open", ctx)
    return _split_fr(t.raw, cols), int.from_bytes(rho.raw, "little"), int.from_bytes(y.raw, "little")


def hyrax_verify(ctx, key, commitments, point, t, rho, y, want_combined=True):
    """commitments: list of 96-byte strings; t: the opened row; rho: rho* or None.  Returns (verdict, combined
    commitment bytes, or None if not asked for); verdict 0 = accepted."""
    rows = len(commitments)
    cb = C.create_string_buffer(b"".join(commitments), 96 * rows)
    pb = C.create_string_buffer(_fr_bytes(point), max(32 * len(point), 1))
    tb = C.create_string_buffer(_fr_bytes(t), 32 * len(t))
    rb = C.create_string_buffer(_fr_bytes([rho]), 32) if rho is not None else None
    yb = C.create_string_buffer(_fr_bytes([y]), 32)
    verdict = C.c_int(-1)
    comb = C.create_string_buffer(96) if want_combined else None
    _check(load_library().hyrax_verify(ctx.handle, key.handle, cb, rows, pb, len(point), tb, rb, yb, C.byref(verdict), comb),
           "hyrax_verify", ctx)
    return verdict.value, (comb.raw if want_combined else None)


def commit_selfcheck():
    return load_library().zkdl_commit_selfcheck()


def aggregate_verify(ctx, proof, tr):
    """The library's verifier: on the GPU, or (ctx None) the same program on the CPU.  Returns a dict with
    verdict (0 = accepted), points and claims_left; the transcript advances only if the proof is accepted."""
    proof = bytes(proof)
    buf = C.create_string_buffer(proof, len(proof))
    verdict = C.c_int(-1)
    pts = C.create_string_buffer(32 * POINTS_CAP)
    npts = C.c_size_t(POINTS_CAP)
    claims = (Claim * 16)()
    ncl = C.c_size_t(16)
    if ctx is None:
        _check(load_library().zkdl_host_aggregate_verify(buf, len(proof), tr.handle, C.byref(verdict), pts, C.byref(npts),
                                                         claims, C.byref(ncl)), "zkdl_host_aggregate_verify")
    else:
        _check(load_library().aggregate_verify(ctx.handle, buf, len(proof), tr.handle, C.byref(verdict), pts, C.byref(npts),
                                               claims, C.byref(ncl)), "aggregate_verify", ctx)
    out = dict(verdict=verdict.value, points=[], claims_left=[])
    if verdict.value == 0:
        out["points"] = _split_fr(pts.raw, npts.value)
        p = out["points"]
        out["claims_left"] = [
            dict(tensor=CLAIM_TENSORS[c.tensor],
                 point=[x for s in range(c.nseg) for x in p[c.seg_off[s]:c.seg_off[s] + c.seg_len[s]]],
                 value=int.from_bytes(bytes(c.value), "little"))
            for c in claims[:ncl.value]]
    return out
