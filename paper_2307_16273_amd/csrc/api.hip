// C ABI of the library: contexts, transcripts, tensors and the host-side
// orchestration of each proof (which kernels run, in which order, on the
// context's stream).  See include/zkdl.h for the contract of every entry point.
#include <string.h>
#include <initializer_list>
#include <mutex>
#include <new>
#include <utility>

#include "zkdl_internal.h"

// ---------------------------------------------------------------------------
// scratch allocator: hipMalloc with a cache of freed blocks.  All work of a
// context is on one stream, so a block may be handed out again as soon as the
// host has released it: the kernels that used it are ahead in the stream.
// ---------------------------------------------------------------------------
void* zk_alloc(zkdl_ctx* ctx, size_t bytes) {
    if (bytes == 0) bytes = 256;
    bytes = (bytes + 255) & ~(size_t)255;
    auto it = ctx->free_blocks.lower_bound(bytes);
    if (it != ctx->free_blocks.end() && it->first <= bytes * 2) {
        void* p = it->second;
        ctx->live_blocks[p] = it->first;
        ctx->free_blocks.erase(it);
        return p;
    }
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) {
        // give cached memory back and retry once
        zkdl_ctx_trim(ctx);
        e = hipMalloc(&p, bytes);
        if (e != hipSuccess) {
            ctx->last_hip = (int)e;
            (void)hipGetLastError();
            return nullptr;
        }
    }
    ctx->live_blocks[p] = bytes;
    return p;
}

void zk_free(zkdl_ctx* ctx, void* p) {
    if (!p) return;
    auto it = ctx->live_blocks.find(p);
    if (it == ctx->live_blocks.end()) return;
    ctx->free_blocks.insert({it->second, p});
    ctx->live_blocks.erase(it);
}

extern "C" int zkdl_ctx_trim(zkdl_ctx* ctx) {
    if (!ctx) return ZKDL_EINVAL;
    (void)hipStreamSynchronize(ctx->stream);
    for (auto& kv : ctx->free_blocks) (void)hipFree(kv.second);
    ctx->free_blocks.clear();
    return ZKDL_OK;
}

// ---------------------------------------------------------------------------
// Work memory of sumcheck_product_noalloc: the folded tables of a product sumcheck of up to three
// tables of 2^ZKDL_NOALLOC_MAX_LOG2 entries (zk_sumcheck_work_bytes).  Every GPU the library runs on
// holds its own copy at its own address for the life of the process; the name below is only a handle
// for hipGetSymbolAddress, the address it yields is what kernels and copies are given.
// ---------------------------------------------------------------------------
constexpr size_t ZK_NOALLOC_SCRATCH_BYTES = (size_t)3 * ((size_t)1 << (ZKDL_NOALLOC_MAX_LOG2 - 1)) * 36;
static __device__ __align__(256) unsigned char scratch[ZK_NOALLOC_SCRATCH_BYTES];

constexpr int ZK_MAX_DEVICES = 64;
static void* g_scratch_addr[ZK_MAX_DEVICES];   // per device, set once under g_scratch_lock
static std::mutex g_scratch_lock;

// the address of `scratch` on `device`, which must be the current device
static hipError_t static_scratch_address(int device, void** out) {
    if (device < 0 || device >= ZK_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_addr[device]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_addr[device] = p;
    }
    *out = g_scratch_addr[device];
    return hipSuccess;
}

// ---------------------------------------------------------------------------
// constants
// ---------------------------------------------------------------------------
static Fr host_double_mod(const Fr& a) { return fr_add(a, a); }

extern "C" int zkdl_selfcheck_constants(void) {
    // 2^261, 2^522, 2^778 mod r by repeated doubling of 1
    Fr x = fr_zero();
    x.v[0] = 1;
    for (int i = 0; i < 261; ++i) x = host_double_mod(x);
    if (!fr_eq(x, fr_const(frc::ONE))) return ZKDL_EINVAL;
    for (int i = 0; i < 261; ++i) x = host_double_mod(x);
    if (!fr_eq(x, fr_const(frc::R2))) return ZKDL_EINVAL;
    for (int i = 0; i < 256; ++i) x = host_double_mod(x);
    if (!fr_eq(x, fr_const(frc::W3))) return ZKDL_EINVAL;
    // the 29-bit limbs of the modulus are its 32-bit limbs repacked
    F9 m9 = fr_unpack(fr_const(frc::MOD));
    for (int i = 0; i < 9; ++i)
        if (m9.v[i] != frc::MOD9[i]) return ZKDL_EINVAL;
    // the modulus is 1 mod 2^29, which the reduction step of f9_mul relies on
    if (frc::MOD9[0] != 1u) return ZKDL_EINVAL;
    return ZKDL_OK;
}

static Fr host_inverse(const Fr& a_mont) {
    uint32_t e[8];
    for (int i = 0; i < 8; ++i) e[i] = frc::MOD[i];
    // exponent r - 2 (Fermat); r[0] = 1, so the subtraction borrows from the next limb
    e[0] = 0xffffffffu;
    int k = 1;
    while (e[k] == 0) {
        e[k] = 0xffffffffu;
        ++k;
    }
    e[k] -= 1;
    return fr_pow(a_mont, e);
}

extern "C" int zkdl_host_fr_mul(const zkdl_fr* a, const zkdl_fr* b, zkdl_fr* out) {
    if (!a || !b || !out) return ZKDL_EINVAL;
    Fr x, y;
    memcpy(x.v, a->le, 32);
    memcpy(y.v, b->le, 32);
    Fr p = fr_mul(fr_to_mont(x), fr_to_mont(y));
    Fr plain = fr_from_mont(p);
    memcpy(out->le, plain.v, 32);
    return ZKDL_OK;
}

// ---------------------------------------------------------------------------
// context
// ---------------------------------------------------------------------------
extern "C" const char* zkdl_strerror(int err) {
    switch (err) {
        case ZKDL_OK: return "ok";
        case ZKDL_EINVAL: return "invalid argument";
        case ZKDL_ERANGE: return "zkReLU input outside the (Q+R)-bit range";
        case ZKDL_ENOMEM: return "out of memory";
        case ZKDL_EHIP: return "HIP runtime error";
        case ZKDL_ESMALL: return "output buffer too small";
        case ZKDL_ETOOBIG: return "input larger than the allocation-free entry point's static work memory";
        default: return "unknown error";
    }
}

extern "C" int zkdl_ctx_create(zkdl_ctx** out, int device, void* hip_stream) {
    if (!out) return ZKDL_EINVAL;
    *out = nullptr;
    if (zkdl_selfcheck_constants() != ZKDL_OK) return ZKDL_EINVAL;
    zkdl_ctx* ctx = new (std::nothrow) zkdl_ctx();
    if (!ctx) return ZKDL_ENOMEM;
    ctx->device = device;
    ctx->stream = (hipStream_t)hip_stream;
    ctx->last_hip = 0;
    ctx->dev = nullptr;
    ctx->host_stage = nullptr;
    ctx->partials = nullptr;
    ctx->n_chal = 0;
    ctx->proof_len = 0;
    ctx->prof_on = false;
    ctx->commit_wbits = 0;
    ctx->zk_fill_threads = 65536;    // one wave on each of the 1024 SIMDs; measured best on the 8 x 1024^2 network
    ctx->prof_used = 0;
    for (int i = 0; i < ZKDL_PROF_CLASSES; ++i) {
        ctx->prof_ms[i] = ctx->prof_bytes[i] = 0.0;
        ctx->prof_launches[i] = 0;
    }
    hipError_t e = hipSetDevice(device);
    ctx->static_scratch = nullptr;
    if (e == hipSuccess) e = static_scratch_address(device, &ctx->static_scratch);
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->dev, sizeof(DevState));
    if (e == hipSuccess) e = hipHostMalloc((void**)&ctx->host_stage, sizeof(DevState), hipHostMallocDefault);
    if (e == hipSuccess)
        e = hipMalloc((void**)&ctx->partials, sizeof(Fr) * ZK_MAX_PART_BLOCKS * ZK_MAX_EVALS * 2);
    if (e == hipSuccess) e = hipMemsetAsync(ctx->dev, 0, sizeof(DevState), ctx->stream);
    if (e == hipSuccess) {
        // constants of the Lagrange formulas
        Fr two = fr_add(fr_one(), fr_one());
        Fr six = fr_add(fr_add(two, two), two);
        Fr c[2] = {host_inverse(two), host_inverse(six)};
        if (!fr_eq(fr_mul(c[0], two), fr_one()) || !fr_eq(fr_mul(c[1], six), fr_one())) {
            e = hipErrorUnknown;
        } else {
            memcpy(ctx->host_stage, c, sizeof(c));
            e = hipMemcpyAsync(&ctx->dev->inv2, ctx->host_stage, sizeof(c), hipMemcpyHostToDevice,
                               ctx->stream);
            if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        }
    }
    if (e != hipSuccess) {
        int code = (int)e;
        (void)hipGetLastError();
        if (ctx->dev) (void)hipFree(ctx->dev);
        if (ctx->host_stage) (void)hipHostFree(ctx->host_stage);
        if (ctx->partials) (void)hipFree(ctx->partials);
        delete ctx;
        (void)code;
        return ZKDL_EHIP;
    }
    *out = ctx;
    return ZKDL_OK;
}

extern "C" int zkdl_ctx_destroy(zkdl_ctx* ctx) {
    if (!ctx) return ZKDL_EINVAL;
    (void)hipStreamSynchronize(ctx->stream);
    for (auto& sp : ctx->prof_spans) {
        (void)hipEventDestroy(sp.e0);
        (void)hipEventDestroy(sp.e1);
    }
    for (auto& kv : ctx->free_blocks) (void)hipFree(kv.second);
    for (auto& kv : ctx->live_blocks) (void)hipFree(kv.first);
    (void)hipFree(ctx->dev);
    (void)hipHostFree(ctx->host_stage);
    (void)hipFree(ctx->partials);
    delete ctx;
    return ZKDL_OK;
}

extern "C" int zkdl_last_hip_error(const zkdl_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

extern "C" int zkdl_ctx_set_fill_threads(zkdl_ctx* ctx, uint64_t threads) {
    if (!ctx || threads < 1 || threads > ((uint64_t)1 << 24)) return ZKDL_EINVAL;
    ctx->zk_fill_threads = threads;
    return ZKDL_OK;
}

extern "C" int zkdl_ctx_set_commit_window_bits(zkdl_ctx* ctx, int bits) {
    if (!ctx || (bits != 0 && bits != 8 && bits != 12)) return ZKDL_EINVAL;
    ctx->commit_wbits = bits;
    return ZKDL_OK;
}

// ---------------------------------------------------------------------------
// per-kernel timing
// ---------------------------------------------------------------------------
void zk_prof_begin(zkdl_ctx* ctx, int cls, double bytes) {
    if (!ctx->prof_on) return;
    if (ctx->prof_used == ctx->prof_spans.size()) {
        zkdl_ctx::ProfSpan sp;
        if (hipEventCreate(&sp.e0) != hipSuccess || hipEventCreate(&sp.e1) != hipSuccess) {
            ctx->prof_on = false;
            return;
        }
        sp.cls = 0;
        ctx->prof_spans.push_back(sp);
    }
    zkdl_ctx::ProfSpan& sp = ctx->prof_spans[ctx->prof_used];
    sp.cls = cls;
    ctx->prof_bytes[cls] += bytes;
    ctx->prof_launches[cls] += 1;
    (void)hipEventRecord(sp.e0, ctx->stream);
}

void zk_prof_end(zkdl_ctx* ctx) {
    if (!ctx->prof_on) return;
    (void)hipEventRecord(ctx->prof_spans[ctx->prof_used].e1, ctx->stream);
    ctx->prof_used += 1;
}

// folds the pending spans into the per-class totals; the stream must be idle
static void prof_collect(zkdl_ctx* ctx) {
    for (size_t i = 0; i < ctx->prof_used; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ctx->prof_spans[i].e0, ctx->prof_spans[i].e1) == hipSuccess)
            ctx->prof_ms[ctx->prof_spans[i].cls] += ms;
    }
    ctx->prof_used = 0;
}

extern "C" int zkdl_ctx_profile_enable(zkdl_ctx* ctx, int on) {
    if (!ctx) return ZKDL_EINVAL;
    ZK_HIP(ctx, hipStreamSynchronize(ctx->stream));
    prof_collect(ctx);
    ctx->prof_on = on != 0;
    return ZKDL_OK;
}

extern "C" int zkdl_ctx_profile_reset(zkdl_ctx* ctx) {
    if (!ctx) return ZKDL_EINVAL;
    ZK_HIP(ctx, hipStreamSynchronize(ctx->stream));
    ctx->prof_used = 0;
    for (int i = 0; i < ZKDL_PROF_CLASSES; ++i) {
        ctx->prof_ms[i] = ctx->prof_bytes[i] = 0.0;
        ctx->prof_launches[i] = 0;
    }
    return ZKDL_OK;
}

extern "C" int zkdl_ctx_profile_read(zkdl_ctx* ctx, int cls, uint64_t* launches, double* total_ms,
                                     double* total_bytes) {
    if (!ctx || cls < 0 || cls >= ZKDL_PROF_CLASSES) return ZKDL_EINVAL;
    ZK_HIP(ctx, hipStreamSynchronize(ctx->stream));
    prof_collect(ctx);
    if (launches) *launches = ctx->prof_launches[cls];
    if (total_ms) *total_ms = ctx->prof_ms[cls];
    if (total_bytes) *total_bytes = ctx->prof_bytes[cls];
    return ZKDL_OK;
}

// ---------------------------------------------------------------------------
// transcript (host)
// ---------------------------------------------------------------------------
extern "C" int zkdl_transcript_create(zkdl_transcript** out, uint64_t seed) {
    if (!out) return ZKDL_EINVAL;
    zkdl_transcript* t = new (std::nothrow) zkdl_transcript();
    if (!t) return ZKDL_ENOMEM;
    ts::init(t->s, seed);
    *out = t;
    return ZKDL_OK;
}

extern "C" int zkdl_transcript_destroy(zkdl_transcript* t) {
    if (!t) return ZKDL_EINVAL;
    delete t;
    return ZKDL_OK;
}

extern "C" int zkdl_transcript_absorb(zkdl_transcript* t, const char* label, const void* bytes, size_t n) {
    if (!t || !label || (!bytes && n)) return ZKDL_EINVAL;
    size_t ll = strlen(label);
    if (ll > ts::MAX_LABEL) return ZKDL_EINVAL;
    ts::absorb(t->s, label, (uint32_t)ll, (const uint8_t*)bytes, (uint64_t)n);
    return ZKDL_OK;
}

extern "C" int zkdl_transcript_challenge(zkdl_transcript* t, zkdl_fr* host_out) {
    if (!t || !host_out) return ZKDL_EINVAL;
    ts::challenge(t->s, host_out->le);
    return ZKDL_OK;
}

extern "C" int zkdl_transcript_digest(const zkdl_transcript* t, uint8_t host_out[32]) {
    if (!t || !host_out) return ZKDL_EINVAL;
    ts::digest(t->s, host_out);
    return ZKDL_OK;
}

// ---------------------------------------------------------------------------
// tensors
// ---------------------------------------------------------------------------
// 32 little-endian bytes below the modulus
static bool fr_bytes_canonical(const uint8_t* le) {
    for (int l = 7; l >= 0; --l) {
        const uint32_t w = (uint32_t)le[4 * l] | ((uint32_t)le[4 * l + 1] << 8) | ((uint32_t)le[4 * l + 2] << 16) |
                           ((uint32_t)le[4 * l + 3] << 24);
        if (w != frc::MOD[l]) return w < frc::MOD[l];
    }
    return false;
}

static bool is_pow2(uint64_t x) { return x && !(x & (x - 1)); }
static int ilog2_u64(uint64_t x) {
    int l = 0;
    while (((uint64_t)1 << l) < x) ++l;
    return l;
}

static int check_shape(const uint64_t* shape, int ndim, uint64_t* numel) {
    if (ndim < 0 || ndim > ZKDL_MAX_DIMS || (ndim > 0 && !shape)) return ZKDL_EINVAL;
    uint64_t n = 1;
    for (int i = 0; i < ndim; ++i) {
        if (!is_pow2(shape[i])) return ZKDL_EINVAL;
        if (n > ((uint64_t)1 << 40) / shape[i]) return ZKDL_EINVAL;
        n *= shape[i];
    }
    *numel = n;
    return ZKDL_OK;
}

static zkdl_tensor* new_tensor(int kind, const uint64_t* shape, int ndim, uint64_t numel) {
    zkdl_tensor* t = new (std::nothrow) zkdl_tensor();
    if (!t) return nullptr;
    t->kind = kind;
    t->ndim = ndim;
    for (int i = 0; i < ZKDL_MAX_DIMS; ++i) t->shape[i] = i < ndim ? shape[i] : 1;
    t->numel = numel;
    t->data = nullptr;
    t->owned = false;
    return t;
}

static size_t dtype_size(int dtype) { return dtype == ZKDL_I32 ? 4 : dtype == ZKDL_I64 ? 8 : 32; }

extern "C" int fr_tensor_upload(zkdl_ctx* ctx, const void* src, int dtype, int src_on_device,
                                const uint64_t* shape, int ndim, zkdl_tensor** out) {
    if (!ctx || !src || !out) return ZKDL_EINVAL;
    if (dtype != ZKDL_I32 && dtype != ZKDL_I64 && dtype != ZKDL_FR_LE) return ZKDL_EINVAL;
    uint64_t n;
    int rc = check_shape(shape, ndim, &n);
    if (rc != ZKDL_OK) return rc;
    zkdl_tensor* t = new_tensor(TK_FR, shape, ndim, n);
    if (!t) return ZKDL_ENOMEM;
    t->data = zk_alloc(ctx, n * 32);
    if (!t->data) {
        delete t;
        return ZKDL_ENOMEM;
    }
    t->owned = true;
    const void* dsrc = src;
    void* staged = nullptr;
    if (!src_on_device) {
        staged = zk_alloc(ctx, n * dtype_size(dtype));
        if (!staged) {
            zk_free(ctx, t->data);
            delete t;
            return ZKDL_ENOMEM;
        }
        hipError_t e = hipMemcpyAsync(staged, src, n * dtype_size(dtype), hipMemcpyHostToDevice, ctx->stream);
        if (e != hipSuccess) {
            ctx->last_hip = (int)e;
            zk_free(ctx, staged);
            zk_free(ctx, t->data);
            delete t;
            return ZKDL_EHIP;
        }
        dsrc = staged;
    }
    int kind = dtype == ZKDL_I32 ? TK_I32 : dtype == ZKDL_I64 ? TK_I64 : 3;
    zk_launch_convert(ctx, dsrc, kind, n, make_tab(t->data, n));
    hipError_t e = hipSuccess;
    if (staged) {
        // the host buffer is pageable: make sure the copy has consumed it before returning
        e = hipStreamSynchronize(ctx->stream);
        zk_free(ctx, staged);
    }
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) {
        ctx->last_hip = (int)e;
        zk_free(ctx, t->data);
        delete t;
        return ZKDL_EHIP;
    }
    *out = t;
    return ZKDL_OK;
}

extern "C" int zkdl_tensor_wrap_int(zkdl_ctx* ctx, const void* device_src, int dtype,
                                    const uint64_t* shape, int ndim, zkdl_tensor** out) {
    if (!ctx || !device_src || !out) return ZKDL_EINVAL;
    if (dtype != ZKDL_I32 && dtype != ZKDL_I64) return ZKDL_EINVAL;
    uint64_t n;
    int rc = check_shape(shape, ndim, &n);
    if (rc != ZKDL_OK) return rc;
    zkdl_tensor* t = new_tensor(dtype == ZKDL_I32 ? TK_I32 : TK_I64, shape, ndim, n);
    if (!t) return ZKDL_ENOMEM;
    t->data = const_cast<void*>(device_src);
    *out = t;
    return ZKDL_OK;
}

extern "C" int zkdl_tensor_ndim(const zkdl_tensor* t) { return t ? t->ndim : -1; }
extern "C" uint64_t zkdl_tensor_dim(const zkdl_tensor* t, int axis) {
    return (t && axis >= 0 && axis < t->ndim) ? t->shape[axis] : 0;
}
extern "C" uint64_t zkdl_tensor_numel(const zkdl_tensor* t) { return t ? t->numel : 0; }

extern "C" int zkdl_tensor_free(zkdl_ctx* ctx, zkdl_tensor* t) {
    if (!ctx || !t) return ZKDL_EINVAL;
    if (t->owned) zk_free(ctx, t->data);
    delete t;
    return ZKDL_OK;
}

// an Fr view of any tensor: Fr tensors as they are, integer tensors converted into scratch
struct FrView {
    FrTab tab;
    void* scratch;
};

static int as_fr(zkdl_ctx* ctx, const zkdl_tensor* t, FrView* v) {
    v->scratch = nullptr;
    if (t->kind == TK_FR) {
        v->tab = make_tab(t->data, t->numel);
        return ZKDL_OK;
    }
    v->scratch = zk_alloc(ctx, t->numel * 32);
    if (!v->scratch) return ZKDL_ENOMEM;
    v->tab = make_tab(v->scratch, t->numel);
    zk_launch_convert(ctx, t->data, t->kind, t->numel, v->tab);
    return ZKDL_OK;
}

extern "C" int zkdl_tensor_download(zkdl_ctx* ctx, const zkdl_tensor* t, zkdl_fr* host_out) {
    if (!ctx || !t || !host_out) return ZKDL_EINVAL;
    FrView v;
    int rc = as_fr(ctx, t, &v);
    if (rc != ZKDL_OK) return rc;
    void* le = zk_alloc(ctx, t->numel * 32);
    if (!le) {
        zk_free(ctx, v.scratch);
        return ZKDL_ENOMEM;
    }
    zk_launch_download(ctx, v.tab, t->numel, (uint8_t*)le);
    hipError_t e = hipMemcpyAsync(host_out, le, t->numel * 32, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    zk_free(ctx, le);
    zk_free(ctx, v.scratch);
    ZK_HIP(ctx, e);
    return ZKDL_OK;
}

// ---------------------------------------------------------------------------
// call framing: transcript state to the device, proof and challenges back
// ---------------------------------------------------------------------------
// Header words of the proof are known on the host: they are kept in the context and written over the
// device's proof bytes when the call ends.  A call that would need more than ZK_MAX_PATCHES of them
// fails in call_end (patch_overflow).
void zk_write_proof_words(zkdl_ctx* ctx, const uint32_t* words, int n) {
    if (ctx->n_patches < ZK_MAX_PATCHES) {
        HeaderPatch& p = ctx->patches[ctx->n_patches++];
        p.off = ctx->proof_len;
        p.n = n;
        for (int i = 0; i < n; ++i) p.words[i] = words[i];
    } else {
        ctx->patch_overflow = true;
    }
    ctx->proof_len += 4 * (size_t)n;
}

static int call_begin(zkdl_ctx* ctx, zkdl_transcript* tr) {
    ZK_HIP(ctx, hipSetDevice(ctx->device));
    ctx->n_chal = 0;
    ctx->proof_len = 0;
    ctx->pend_len = 0;
    ctx->n_patches = 0;
    ctx->patch_overflow = false;
    // transcript state; error word and owed claim cleared
    memset(ctx->host_stage, 0, ZK_STATE_HEAD);
    {
        DevState* h = (DevState*)ctx->host_stage;
        for (int i = 0; i < 8; ++i) h->ts_state[i] = tr->s.h[i];
        h->ts_nblk[0] = (uint32_t)tr->s.nblk;
        h->ts_nblk[1] = (uint32_t)(tr->s.nblk >> 32);
        h->ts_fill = tr->s.fill;
        for (uint32_t i = 0; i < tr->s.fill; ++i) h->ts_buf[i >> 2] |= (uint32_t)tr->s.buf[i] << (24 - 8 * (i & 3));
    }
    ZK_HIP(ctx, hipMemcpyAsync(ctx->dev, ctx->host_stage, ZK_STATE_HEAD, hipMemcpyHostToDevice, ctx->stream));
    return ZKDL_OK;
}

// the proof bytes of the call that has just ended, in the staging buffer (header words not patched in)
static const uint8_t* staged_proof(const zkdl_ctx* ctx) { return ((const DevState*)ctx->host_stage)->proof; }

// rc_in: result of the enqueue phase; on failure the stream is drained and the caller's
// transcript and buffers stay as they were
static int call_end(zkdl_ctx* ctx, zkdl_transcript* tr, int rc_in, uint8_t* proof, size_t* proof_len,
                    zkdl_fr* points_out, size_t* npoints, const int* scal_ids, int n_scal,
                    zkdl_fr* scal_out) {
    if (rc_in == ZKDL_OK && ctx->patch_overflow) rc_in = ZKDL_EINVAL;
    if (rc_in != ZKDL_OK) {
        ctx->pend_len = 0;
        ZK_HIP(ctx, hipStreamSynchronize(ctx->stream));
        return rc_in;
    }
    zk_flush_frames(ctx);
    ZK_HIP(ctx, hipGetLastError());
    uint8_t* hs = ctx->host_stage;
    // layout of the staging buffer mirrors DevState
    ZK_HIP(ctx, hipMemcpyAsync(hs, ctx->dev, offsetof(DevState, chal), hipMemcpyDeviceToHost, ctx->stream));
    if (ctx->n_chal > 0)
        ZK_HIP(ctx, hipMemcpyAsync(hs + offsetof(DevState, chal_le), ctx->dev->chal_le,
                                   32 * (size_t)ctx->n_chal, hipMemcpyDeviceToHost, ctx->stream));
    if (ctx->proof_len > 0)
        ZK_HIP(ctx, hipMemcpyAsync(hs + offsetof(DevState, proof), ctx->dev->proof, ctx->proof_len,
                                   hipMemcpyDeviceToHost, ctx->stream));
    ZK_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->prof_on) prof_collect(ctx);
    const DevState* h = (const DevState*)hs;
    if (h->err & 1u) return ZKDL_ERANGE;
    // A buffer that is too small (or a proof pointer of NULL, the query for the sizes) fails the call
    // before anything of the caller's is touched: the sizes needed are reported, the transcript stays
    // where it was, and the same call with larger buffers gives the proof the verifier replays.
    const bool proof_small = proof_len && (!proof || *proof_len < ctx->proof_len);
    const bool points_small = points_out && npoints && *npoints < (size_t)ctx->n_chal;
    if (proof_len) *proof_len = ctx->proof_len;
    if (npoints) *npoints = (size_t)ctx->n_chal;
    if (proof_small || points_small) return ZKDL_ESMALL;
    for (int i = 0; i < 8; ++i) tr->s.h[i] = h->ts_state[i];
    tr->s.nblk = ((uint64_t)h->ts_nblk[1] << 32) | h->ts_nblk[0];
    tr->s.fill = h->ts_fill;
    for (uint32_t i = 0; i < 64; ++i)
        tr->s.buf[i] = i < h->ts_fill ? (uint8_t)(h->ts_buf[i >> 2] >> (24 - 8 * (i & 3))) : 0;
    if (proof_len) {
        memcpy(proof, h->proof, ctx->proof_len);
        for (int k = 0; k < ctx->n_patches; ++k) {
            const HeaderPatch& p = ctx->patches[k];
            for (int i = 0; i < p.n; ++i)
                for (int b = 0; b < 4; ++b) proof[p.off + 4 * i + b] = (uint8_t)(p.words[i] >> (8 * b));
        }
    }
    if (points_out && npoints) memcpy(points_out, h->chal_le, 32 * (size_t)ctx->n_chal);
    for (int i = 0; i < n_scal && scal_out; ++i) {
        Fr plain = fr_from_mont(h->scal[scal_ids[i]]);
        memcpy(scal_out[i].le, plain.v, 32);
    }
    return ZKDL_OK;
}

// ---------------------------------------------------------------------------
// mle_partial_eval
// ---------------------------------------------------------------------------
extern "C" int mle_partial_eval(zkdl_ctx* ctx, const zkdl_tensor* t, int axis_lo, int axis_hi,
                                const zkdl_fr* point, size_t npoint, zkdl_tensor** out) {
    if (!ctx || !t || !out || axis_lo < 0 || axis_hi < axis_lo || axis_hi > t->ndim) return ZKDL_EINVAL;
    if (npoint && !point) return ZKDL_EINVAL;
    uint64_t O = 1, A = 1, I = 1;
    for (int i = 0; i < axis_lo; ++i) O *= t->shape[i];
    for (int i = axis_lo; i < axis_hi; ++i) A *= t->shape[i];
    for (int i = axis_hi; i < t->ndim; ++i) I *= t->shape[i];
    int m = ilog2_u64(A);
    if ((size_t)m != npoint || m > 40) return ZKDL_EINVAL;
    ZK_HIP(ctx, hipSetDevice(ctx->device));
    uint64_t oshape[ZKDL_MAX_DIMS];
    int ond = 0;
    for (int i = 0; i < axis_lo; ++i) oshape[ond++] = t->shape[i];
    for (int i = axis_hi; i < t->ndim; ++i) oshape[ond++] = t->shape[i];
    zkdl_tensor* o = new_tensor(TK_FR, oshape, ond, O * I);
    if (!o) return ZKDL_ENOMEM;
    o->data = zk_alloc(ctx, O * I * 32);
    o->owned = true;
    size_t pbytes = (size_t)(m > 0 ? m : 1) * 32;
    uint8_t* ple = (uint8_t*)zk_alloc(ctx, pbytes);
    Fr* pm = (Fr*)zk_alloc(ctx, pbytes);
    void* beta = zk_alloc(ctx, A * 32);
    int rc = (o->data && ple && pm && beta) ? ZKDL_OK : ZKDL_ENOMEM;
    if (rc == ZKDL_OK && m > 0) {
        hipError_t e = hipMemcpyAsync(ple, point, (size_t)m * 32, hipMemcpyHostToDevice, ctx->stream);
        if (e != hipSuccess) {
            ctx->last_hip = (int)e;
            rc = ZKDL_EHIP;
        }
    }
    if (rc == ZKDL_OK) {
        zk_launch_points_to_mont(ctx, ple, m, pm);
        FrTab bt = make_tab(beta, A);
        rc = zk_build_beta(ctx, pm, m, bt);
        if (rc == ZKDL_OK) {
            FrTab src_tab = make_tab(t->data, t->numel);
            const void* src = t->kind == TK_FR ? (const void*)&src_tab : t->data;
            rc = zk_partial_eval(ctx, t->kind, src, O, A, I, bt, make_tab(o->data, O * I));
        }
    }
    hipError_t e = hipStreamSynchronize(ctx->stream);   // `point` is pageable host memory
    zk_free(ctx, ple);
    zk_free(ctx, pm);
    zk_free(ctx, beta);
    if (rc == ZKDL_OK && e != hipSuccess) {
        ctx->last_hip = (int)e;
        rc = ZKDL_EHIP;
    }
    if (rc == ZKDL_OK && (e = hipGetLastError()) != hipSuccess) {
        ctx->last_hip = (int)e;
        rc = ZKDL_EHIP;
    }
    if (rc != ZKDL_OK) {
        zkdl_tensor_free(ctx, o);
        return rc;
    }
    *out = o;
    return ZKDL_OK;
}

// ---------------------------------------------------------------------------
// hyrax_open: the prover's side of the proof of evaluation for a tensor committed row by row
// (Sec. 2.3; Protocol zkdl, the proof-of-evaluation line): three partial evaluations
// ---------------------------------------------------------------------------
extern "C" int hyrax_open(zkdl_ctx* ctx, const zkdl_tensor* X, const zkdl_fr* blind, const zkdl_fr* point,
                          size_t npoint, zkdl_fr* T_out, zkdl_fr* rho_out, zkdl_fr* y_out) {
    if (!ctx || !X || !T_out || !y_out || (npoint && !point)) return ZKDL_EINVAL;
    const int m = ilog2_u64(X->numel);
    if (!is_pow2(X->numel) || (size_t)m != npoint) return ZKDL_EINVAL;
    for (size_t i = 0; i < npoint; ++i)
        if (!fr_bytes_canonical(point[i].le)) return ZKDL_EINVAL;
    const uint64_t cols = (uint64_t)1 << (m / 2), rows = (uint64_t)1 << (m - m / 2);
    const int lr = m - m / 2;
    zkdl_tensor view = *X;   // the same memory as an R x C matrix
    view.ndim = 2;
    view.shape[0] = rows;
    view.shape[1] = cols;
    view.owned = false;
    zkdl_tensor *t = nullptr, *y = nullptr, *b = nullptr, *r = nullptr;
    int rc = mle_partial_eval(ctx, &view, 0, 1, point, (size_t)lr, &t);          // T = sum_j beta~(v_row, j) X[j, :]
    if (rc == ZKDL_OK) rc = mle_partial_eval(ctx, t, 0, 1, point + lr, npoint - (size_t)lr, &y);   // <T, beta~(v_col, .)>
    if (rc == ZKDL_OK) rc = zkdl_tensor_download(ctx, t, T_out);
    if (rc == ZKDL_OK) rc = zkdl_tensor_download(ctx, y, y_out);
    if (rc == ZKDL_OK && blind && rho_out) {                                       // rho* = sum_j beta~(v_row, j) rho_j
        const uint64_t shape[1] = {rows};
        rc = fr_tensor_upload(ctx, blind, ZKDL_FR_LE, 0, shape, 1, &b);
        if (rc == ZKDL_OK) rc = mle_partial_eval(ctx, b, 0, 1, point, (size_t)lr, &r);
        if (rc == ZKDL_OK) rc = zkdl_tensor_download(ctx, r, rho_out);
    } else if (rc == ZKDL_OK && rho_out) {
        memset(rho_out->le, 0, 32);
    }
    if (t) zkdl_tensor_free(ctx, t);
    if (y) zkdl_tensor_free(ctx, y);
    if (b) zkdl_tensor_free(ctx, b);
    if (r) zkdl_tensor_free(ctx, r);
    return rc;
}

// ---------------------------------------------------------------------------
// sumcheck_product
// ---------------------------------------------------------------------------
extern "C" int sumcheck_product(zkdl_ctx* ctx, const zkdl_tensor* const* tables, int K,
                                zkdl_transcript* tr, uint8_t* proof, size_t* proof_len,
                                zkdl_fr* finals, zkdl_fr* points_out, size_t* npoints) {
    if (!ctx || !tables || !tr || K < 1 || K > 3) return ZKDL_EINVAL;
    for (int k = 0; k < K; ++k)
        if (!tables[k] || tables[k]->numel != tables[0]->numel) return ZKDL_EINVAL;
    const uint64_t n = tables[0]->numel;
    const int d = ilog2_u64(n);
    int rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    uint32_t hdr[2] = {(uint32_t)K, (uint32_t)d};
    zk_absorb_words(ctx, "sumcheck_product", hdr, 2);
    FrView views[3];
    FrTab src[3];
    void* wmem = nullptr;
    for (int k = 0; k < K; ++k) views[k].scratch = nullptr;
    for (int k = 0; k < K && rc == ZKDL_OK; ++k) {
        rc = as_fr(ctx, tables[k], &views[k]);
        src[k] = views[k].tab;
    }
    if (rc == ZKDL_OK) {
        wmem = zk_alloc(ctx, zk_sumcheck_work_bytes(K, d));
        if (!wmem) rc = ZKDL_ENOMEM;
    }
    if (rc == ZKDL_OK) rc = zk_sumcheck_product(ctx, K, src, wmem, d, 0);
    int ids[3] = {0, 1, 2};
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, ids, K, finals);
    zk_free(ctx, wmem);
    for (int k = 0; k < K; ++k) zk_free(ctx, views[k].scratch);
    return rc != ZKDL_OK ? rc : rc2;
}

// sumcheck_product with its work tables in the library's static device array: no allocation of any
// kind between entry and return (the context's state block, partial-sum slots and pinned staging
// buffer were allocated when the context was created).
extern "C" int sumcheck_product_noalloc(zkdl_ctx* ctx, const zkdl_tensor* const* tables, int K,
                                        zkdl_transcript* tr, uint8_t* proof, size_t* proof_len,
                                        zkdl_fr* finals, zkdl_fr* points_out, size_t* npoints) {
    if (!ctx || !tables || !tr || K < 1 || K > 3) return ZKDL_EINVAL;
    for (int k = 0; k < K; ++k) {
        if (!tables[k] || tables[k]->numel != tables[0]->numel) return ZKDL_EINVAL;
        if (tables[k]->kind != TK_FR) return ZKDL_EINVAL;   // an integer view would need a converted copy
    }
    if (ctx->prof_on) return ZKDL_EINVAL;                   // per-kernel timing creates events
    const uint64_t n = tables[0]->numel;
    const int d = ilog2_u64(n);
    if (d > ZKDL_NOALLOC_MAX_LOG2) return ZKDL_ETOOBIG;
    if (zk_sumcheck_work_bytes(K, d) > ZK_NOALLOC_SCRATCH_BYTES || !ctx->static_scratch) return ZKDL_ETOOBIG;
    int rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    uint32_t hdr[2] = {(uint32_t)K, (uint32_t)d};
    zk_absorb_words(ctx, "sumcheck_product", hdr, 2);
    FrTab src[3];
    for (int k = 0; k < K; ++k) src[k] = make_tab(tables[k]->data, tables[k]->numel);
    // every work-table entry a round reads was written by the round before it in this call (the first
    // round reads the inputs only), so what an earlier call left in the array is never seen
    rc = zk_sumcheck_product(ctx, K, src, ctx->static_scratch, d, 0);
    int ids[3] = {0, 1, 2};
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, ids, K, finals);
    return rc != ZKDL_OK ? rc : rc2;
}

// ---------------------------------------------------------------------------
// matmul / Hadamard (Eqs. exm-matmul-batched, exm-hadamard-batched)
// ---------------------------------------------------------------------------
struct MatmulShape {
    uint64_t N, D1, D2, D3;
};

// Enqueues one matmul sumcheck.  X0 stored [N, r0, c0], X1 stored [N, r1, c1].
// shift != 0: stack slot n uses slot n+1 of both operands, zero in the last slot of
// every `shift`-slot period (the gradA family).  Final claims are left in
// scal[scal_base .. +3): beta~(w,v_n), X0~, X1~.
static int enqueue_matmul(zkdl_ctx* ctx, const zkdl_tensor* X0, const zkdl_tensor* X1, int tr0, int tr1,
                          uint32_t shift, int scal_base, MatmulShape* shp_out) {
    if (X0->ndim != 3 || X1->ndim != 3 || X0->shape[0] != X1->shape[0]) return ZKDL_EINVAL;
    const uint64_t N = X0->shape[0];
    const uint64_t D1 = tr0 ? X0->shape[2] : X0->shape[1];
    const uint64_t D2 = tr0 ? X0->shape[1] : X0->shape[2];
    const uint64_t D2b = tr1 ? X1->shape[2] : X1->shape[1];
    const uint64_t D3 = tr1 ? X1->shape[1] : X1->shape[2];
    if (D2 != D2b) return ZKDL_EINVAL;
    if (shp_out) *shp_out = MatmulShape{N, D1, D2, D3};
    const int ln = ilog2_u64(N), l1 = ilog2_u64(D1), l2 = ilog2_u64(D2), l3 = ilog2_u64(D3);
    if (ctx->n_chal + ln + l1 + l3 + ln + l2 > ZK_MAX_CHAL) return ZKDL_EINVAL;
    uint32_t hdr[4] = {(uint32_t)N, (uint32_t)D1, (uint32_t)D2, (uint32_t)D3};
    zk_absorb_words(ctx, "sumcheck_matmul", hdr, 4);
    const int cw = ctx->n_chal, cu0 = cw + ln, cu1 = cu0 + l1;
    zk_launch_draw(ctx, cw, ln + l1 + l3);
    ctx->n_chal += ln + l1 + l3;
    const Fr* chal = ctx->dev->chal;

    const uint64_t len = N * D2;
    // scratch: beta tables (N, D1, D3), three source tables, one shift temp, the work tables
    void* mem = zk_alloc(ctx, (N + D1 + D3 + 4 * len) * 32 + zk_sumcheck_work_bytes(3, ln + l2));
    if (!mem) return ZKDL_ENOMEM;
    uint32_t* base = (uint32_t*)mem;
    FrTab bw = make_tab(base, N);
    base += 8 * N;
    FrTab bu0 = make_tab(base, D1);
    base += 8 * D1;
    FrTab bu1 = make_tab(base, D3);
    base += 8 * D3;
    FrTab src[3];
    for (int k = 0; k < 3; ++k) {
        src[k] = make_tab(base, len);
        base += 8 * len;
    }
    FrTab tmp = make_tab(base, len);
    base += 8 * len;
    void* work = base;
    const BetaJob bjobs[3] = {{chal + cw, ln, bw}, {chal + cu0, l1, bu0}, {chal + cu1, l3, bu1}};
    int rc = zk_build_beta_many(ctx, bjobs, 3);
    if (rc == ZKDL_OK) zk_launch_broadcast_rows(ctx, bw, N, D2, src[0]);
    // T0[n, i] = X0~(n, u0, i): bind the D1 axis of op(X0)
    if (rc == ZKDL_OK) {
        FrTab s0 = make_tab(X0->data, X0->numel);
        const void* sp = X0->kind == TK_FR ? (const void*)&s0 : X0->data;
        FrTab dst = shift ? tmp : src[1];
        if (!tr0) rc = zk_partial_eval(ctx, X0->kind, sp, N, D1, D2, bu0, dst);      // stored [N, D1, D2]
        else rc = zk_partial_eval(ctx, X0->kind, sp, N * D2, D1, 1, bu0, dst);       // stored [N, D2, D1]
        if (rc == ZKDL_OK && shift) zk_launch_shift_rows(ctx, tmp, N, D2, shift, src[1]);
    }
    // T1[n, i] = X1~(n, i, u1): bind the D3 axis of op(X1)
    if (rc == ZKDL_OK) {
        FrTab s1 = make_tab(X1->data, X1->numel);
        const void* sp = X1->kind == TK_FR ? (const void*)&s1 : X1->data;
        FrTab dst = shift ? tmp : src[2];
        if (!tr1) rc = zk_partial_eval(ctx, X1->kind, sp, N * D2, D3, 1, bu1, dst);  // stored [N, D2, D3]
        else rc = zk_partial_eval(ctx, X1->kind, sp, N, D3, D2, bu1, dst);           // stored [N, D3, D2]
        if (rc == ZKDL_OK && shift) zk_launch_shift_rows(ctx, tmp, N, D2, shift, src[2]);
    }
    if (rc == ZKDL_OK) rc = zk_sumcheck_product(ctx, 3, src, work, ln + l2, scal_base);
    zk_free(ctx, mem);
    return rc;
}

extern "C" int sumcheck_matmul(zkdl_ctx* ctx, const zkdl_tensor* X0, const zkdl_tensor* X1,
                               int transpose_x0, int transpose_x1, zkdl_transcript* tr, uint8_t* proof,
                               size_t* proof_len, zkdl_fr* claims, zkdl_fr* points_out, size_t* npoints) {
    if (!ctx || !X0 || !X1 || !tr) return ZKDL_EINVAL;
    if (X0->ndim != 3 || X1->ndim != 3) return ZKDL_EINVAL;
    int rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    rc = enqueue_matmul(ctx, X0, X1, transpose_x0 != 0, transpose_x1 != 0, 0, 0, nullptr);
    zkdl_fr tmp[3];
    int ids[3] = {0, 1, 2};
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, ids, 3, tmp);
    if (rc == ZKDL_OK && rc2 == ZKDL_OK && claims) {
        memcpy(claims[0].le, staged_proof(ctx) + 16, 32);   // claim_0 = Y~(w, u0, u1)
        claims[1] = tmp[1];
        claims[2] = tmp[2];
    }
    return rc != ZKDL_OK ? rc : rc2;
}

// Enqueues the optimized aggregated protocol for Y[n] = op(X0[n]) op(X1[n]) (App. B).  Final
// claims are left in scal[scal_base .. +2): X0~, X1~.
static int enqueue_matmul_ft(zkdl_ctx* ctx, const zkdl_tensor* X0, const zkdl_tensor* X1, int tr0, int tr1,
                             uint32_t shift, int scal_base) {
    if (X0->ndim != 3 || X1->ndim != 3 || X0->shape[0] != X1->shape[0]) return ZKDL_EINVAL;
    const uint64_t N = X0->shape[0];
    const uint64_t D1 = tr0 ? X0->shape[2] : X0->shape[1];
    const uint64_t D2 = tr0 ? X0->shape[1] : X0->shape[2];
    const uint64_t D2b = tr1 ? X1->shape[2] : X1->shape[1];
    const uint64_t D3 = tr1 ? X1->shape[1] : X1->shape[2];
    if (D2 != D2b) return ZKDL_EINVAL;
    const int ln = ilog2_u64(N), l1 = ilog2_u64(D1), l2 = ilog2_u64(D2), l3 = ilog2_u64(D3);
    if (ln > 13 || ctx->n_chal + ln + l1 + l3 + ln + l2 > ZK_MAX_CHAL) return ZKDL_EINVAL;
    uint32_t hdr[4] = {(uint32_t)N, (uint32_t)D1, (uint32_t)D2, (uint32_t)D3};
    zk_absorb_words(ctx, "sumcheck_matmul_ft", hdr, 4);
    const int cw = ctx->n_chal, cu0 = cw + ln, cu1 = cu0 + l1;
    zk_launch_draw(ctx, cw, ln + l1 + l3);
    ctx->n_chal += ln + l1 + l3;
    const Fr* chal = ctx->dev->chal;

    const uint64_t len = N * D2;
    // scratch: suffix tables of w (sizes N/2, N/4, .., 1), beta tables (D1, D3), two source tables,
    // the work tables
    void* mem = zk_alloc(ctx, (N + D1 + D3 + 3 * len) * 32 + zk_sumcheck_work_bytes(2, ln + l2));
    if (!mem) return ZKDL_ENOMEM;
    uint32_t* base = (uint32_t*)mem;
    FrTab wsuf[16];
    BetaJob jobs[16];
    int nj = 0;
    for (int t = 0; t < ln; ++t) {
        const uint64_t rows = (uint64_t)1 << (ln - t - 1);
        wsuf[t] = make_tab(base, rows);
        base += 8 * rows;
        jobs[nj++] = BetaJob{chal + cw + t + 1, ln - t - 1, wsuf[t]};
    }
    base = (uint32_t*)mem + 8 * N;
    FrTab bu0 = make_tab(base, D1);
    base += 8 * D1;
    FrTab bu1 = make_tab(base, D3);
    base += 8 * D3;
    jobs[nj++] = BetaJob{chal + cu0, l1, bu0};
    jobs[nj++] = BetaJob{chal + cu1, l3, bu1};
    FrTab src[2];
    for (int k = 0; k < 2; ++k) {
        src[k] = make_tab(base, len);
        base += 8 * len;
    }
    FrTab tmp = make_tab(base, len);   // shift != 0: slot n of both tables takes slot n+1 (zero in each period's last)
    base += 8 * len;
    void* work = base;
    int rc = zk_build_beta_many(ctx, jobs, nj);
    if (rc == ZKDL_OK) {
        FrTab s0 = make_tab(X0->data, X0->numel);
        const void* sp = X0->kind == TK_FR ? (const void*)&s0 : X0->data;
        FrTab dst = shift ? tmp : src[0];
        if (!tr0) rc = zk_partial_eval(ctx, X0->kind, sp, N, D1, D2, bu0, dst);
        else rc = zk_partial_eval(ctx, X0->kind, sp, N * D2, D1, 1, bu0, dst);
        if (rc == ZKDL_OK && shift) zk_launch_shift_rows(ctx, tmp, N, D2, shift, src[0]);
    }
    if (rc == ZKDL_OK) {
        FrTab s1 = make_tab(X1->data, X1->numel);
        const void* sp = X1->kind == TK_FR ? (const void*)&s1 : X1->data;
        FrTab dst = shift ? tmp : src[1];
        if (!tr1) rc = zk_partial_eval(ctx, X1->kind, sp, N * D2, D3, 1, bu1, dst);
        else rc = zk_partial_eval(ctx, X1->kind, sp, N, D3, D2, bu1, dst);
        if (rc == ZKDL_OK && shift) zk_launch_shift_rows(ctx, tmp, N, D2, shift, src[1]);
    }
    if (rc == ZKDL_OK) rc = zk_matmul_ft(ctx, src, work, ln, l2, wsuf, cw, scal_base);
    zk_free(ctx, mem);
    return rc;
}

extern "C" int sumcheck_matmul_ft(zkdl_ctx* ctx, const zkdl_tensor* X0, const zkdl_tensor* X1,
                                  int transpose_x0, int transpose_x1, zkdl_transcript* tr, uint8_t* proof,
                                  size_t* proof_len, zkdl_fr* claims, zkdl_fr* points_out, size_t* npoints) {
    if (!ctx || !X0 || !X1 || !tr) return ZKDL_EINVAL;
    if (X0->ndim != 3 || X1->ndim != 3) return ZKDL_EINVAL;
    int rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    rc = enqueue_matmul_ft(ctx, X0, X1, transpose_x0 != 0, transpose_x1 != 0, 0, 0);
    zkdl_fr tmp[2];
    int ids[2] = {0, 1};
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, ids, 2, tmp);
    if (rc == ZKDL_OK && rc2 == ZKDL_OK && claims) {
        memcpy(claims[0].le, staged_proof(ctx) + 16, 32);   // claim_0 = Y~(w, u0, u1)
        claims[1] = tmp[0];
        claims[2] = tmp[1];
    }
    return rc != ZKDL_OK ? rc : rc2;
}

extern "C" int sumcheck_matmul_general(zkdl_ctx* ctx, const zkdl_tensor* X0, const zkdl_tensor* X1,
                                       const zkdl_tensor* Y, zkdl_transcript* tr, uint8_t* proof, size_t* proof_len,
                                       zkdl_fr* claims, zkdl_fr* points_out, size_t* npoints) {
    if (!ctx || !X0 || !X1 || !Y || !tr) return ZKDL_EINVAL;
    if (X0->ndim != 3 || X1->ndim != 3 || Y->ndim != 3) return ZKDL_EINVAL;
    const uint64_t N = X0->shape[0], D1 = X0->shape[1], D2 = X0->shape[2], D3 = X1->shape[2];
    if (X1->shape[0] != N || X1->shape[1] != D2 || Y->shape[0] != N || Y->shape[1] != D1 || Y->shape[2] != D3)
        return ZKDL_EINVAL;
    // the rounds over i0, i1 and j run in one block each
    if (D1 > ((uint64_t)1 << 16) || D2 > ((uint64_t)1 << 16) || D3 > ((uint64_t)1 << 16)) return ZKDL_ETOOBIG;
    int rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    rc = zk_matmul_general(ctx, X0, X1, Y, ilog2_u64(N), ilog2_u64(D1), ilog2_u64(D2), ilog2_u64(D3), 0);
    zkdl_fr tmp[3];
    int ids[3] = {0, 1, 2};
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, ids, 3, tmp);
    if (rc == ZKDL_OK && rc2 == ZKDL_OK && claims) memcpy(claims, tmp, sizeof(tmp));
    return rc != ZKDL_OK ? rc : rc2;
}

extern "C" int sumcheck_hadamard(zkdl_ctx* ctx, const zkdl_tensor* X0, const zkdl_tensor* X1,
                                 zkdl_transcript* tr, uint8_t* proof, size_t* proof_len,
                                 zkdl_fr* claims, zkdl_fr* points_out, size_t* npoints) {
    if (!ctx || !X0 || !X1 || !tr || X0->numel != X1->numel) return ZKDL_EINVAL;
    const uint64_t n = X0->numel;
    const int d = ilog2_u64(n);
    if (2 * d > ZK_MAX_CHAL) return ZKDL_EINVAL;
    int rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    uint32_t hdr[1] = {(uint32_t)d};
    zk_absorb_words(ctx, "sumcheck_hadamard", hdr, 1);
    zk_launch_draw(ctx, 0, d);
    ctx->n_chal = d;
    FrView v0, v1;
    v0.scratch = v1.scratch = nullptr;
    if (d >= ZK_HD_MIN_LOG) {
        // large: beta~(p, .) is never a folded table; the rounds take beta~(p_[t+1:], .) as weights
        const int t_tail = d - 10;
        // two int32 stacks are read as they are by the first two rounds: no conversion pass, and the
        // first round takes its weights from two small tables instead of beta~(p_[1:], .)
        const bool ints = X0->kind == TK_I32 && X1->kind == TK_I32;
        const int t_first = ints ? 1 : 0;
        const int split_lb = d - 1 < 14 ? d - 1 : 14;
        const uint64_t split_h = (uint64_t)1 << (d - 1 - split_lb), split_l = (uint64_t)1 << split_lb;
        uint64_t suf_elems = ints ? split_h + split_l : 0;
        for (int t = t_first; t < t_tail; ++t) suf_elems += (uint64_t)1 << (d - t - 1);
        void* mem = zk_alloc(ctx, suf_elems * 32 + 2048 * 36 + zk_sumcheck_work_bytes(2, d));
        if (!mem) rc = ZKDL_ENOMEM;
        if (rc == ZKDL_OK && !ints) rc = as_fr(ctx, X0, &v0);
        if (rc == ZKDL_OK && !ints) rc = as_fr(ctx, X1, &v1);
        if (rc == ZKDL_OK) {
            std::vector<FrTab> wsuf(t_tail);
            uint32_t* w = (uint32_t*)mem;
            for (int t = 0; t < t_tail; ++t) {
                const uint64_t cnt = (uint64_t)1 << (d - t - 1);
                wsuf[t] = make_tab(t >= t_first ? w : nullptr, cnt);
                if (t >= t_first) w += 8 * cnt;
            }
            FrTab split[2] = {make_tab(nullptr, 0), make_tab(nullptr, 0)};
            if (ints) {
                split[0] = make_tab(w, split_h);
                w += 8 * split_h;
                split[1] = make_tab(w, split_l);
                w += 8 * split_l;
            }
            F9Tab eq_tail;
            eq_tail.p = w;
            eq_tail.ps = 2048;
            w += 9 * 2048;
            // the smallest table (10 variables) by doubling, every larger one from the one before
            rc = zk_build_beta(ctx, ctx->dev->chal + t_tail, d - t_tail, wsuf[t_tail - 1]);
            if (rc == ZKDL_OK) zk_hadamard_suffix_tables(ctx, wsuf.data(), t_tail - 1, t_first, d, 0);
            if (rc == ZKDL_OK && ints) {
                const BetaJob sj[2] = {{ctx->dev->chal + 1, d - 1 - split_lb, split[0]},
                                       {ctx->dev->chal + d - split_lb, split_lb, split[1]}};
                rc = zk_build_beta_many(ctx, sj, 2);
            }
            FrTab xs[2] = {v0.tab, v1.tab};
            const int32_t* xi[2] = {(const int32_t*)X0->data, (const int32_t*)X1->data};
            if (rc == ZKDL_OK)
                rc = zk_hadamard_eq(ctx, xs, ints ? xi : nullptr, wsuf.data(), split, split_lb, w, eq_tail, d, 0, 0);
        }
        zkdl_fr tmp[3];
        int ids[3] = {0, 1, 2};
        int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, ids, 3, tmp);
        if (rc == ZKDL_OK && rc2 == ZKDL_OK && claims) {
            memcpy(claims[0].le, staged_proof(ctx) + 16, 32);
            claims[1] = tmp[1];
            claims[2] = tmp[2];
        }
        zk_free(ctx, mem);
        zk_free(ctx, v0.scratch);
        zk_free(ctx, v1.scratch);
        return rc != ZKDL_OK ? rc : rc2;
    }
    void* mem = zk_alloc(ctx, n * 32 + zk_sumcheck_work_bytes(3, d));
    if (!mem) rc = ZKDL_ENOMEM;
    if (rc == ZKDL_OK) rc = as_fr(ctx, X0, &v0);
    if (rc == ZKDL_OK) rc = as_fr(ctx, X1, &v1);
    if (rc == ZKDL_OK) {
        FrTab beta = make_tab(mem, n);
        rc = zk_build_beta(ctx, ctx->dev->chal, d, beta);
        FrTab src[3] = {beta, v0.tab, v1.tab};
        if (rc == ZKDL_OK) rc = zk_sumcheck_product(ctx, 3, src, (uint32_t*)mem + 8 * n, d, 0);
    }
    zkdl_fr tmp[3];
    int ids[3] = {0, 1, 2};
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, ids, 3, tmp);
    if (rc == ZKDL_OK && rc2 == ZKDL_OK && claims) {
        memcpy(claims[0].le, staged_proof(ctx) + 16, 32);
        claims[1] = tmp[1];
        claims[2] = tmp[2];
    }
    zk_free(ctx, mem);
    zk_free(ctx, v0.scratch);
    zk_free(ctx, v1.scratch);
    return rc != ZKDL_OK ? rc : rc2;
}

// ---------------------------------------------------------------------------
// re-indexing sumcheck (Eq. sc-reindex)
// ---------------------------------------------------------------------------
static const uint32_t ZKRI_MAGIC = 0x49524B5Au;

// plain SHA-256 of a byte stream fed in pieces (the transcript's block function, standard padding)
struct HostSha {
    ts::State s;
    HostSha() {
        const uint32_t iv[8] = {0x6a09e667, 0xbb67ae85, 0x3c6ef372, 0xa54ff53a,
                                0x510e527f, 0x9b05688c, 0x1f83d9ab, 0x5be0cd19};
        for (int i = 0; i < 8; ++i) s.h[i] = iv[i];
        s.nblk = 0;
        s.fill = 0;
    }
    void bytes(const void* p, size_t n) {
        for (size_t i = 0; i < n; ++i) ts::push_byte(s, ((const uint8_t*)p)[i]);
    }
    void u32(uint32_t v) {
        for (int b = 0; b < 4; ++b) ts::push_byte(s, (uint8_t)(v >> (8 * b)));
    }
    // the digest as eight little-endian words (the form zk_absorb_words takes)
    void digest_words(uint32_t out[8]) const {
        uint8_t dg[32];
        ts::digest(s, dg);
        for (int i = 0; i < 8; ++i)
            out[i] = (uint32_t)dg[4 * i] | ((uint32_t)dg[4 * i + 1] << 8) | ((uint32_t)dg[4 * i + 2] << 16) |
                     ((uint32_t)dg[4 * i + 3] << 24);
    }
};

static int upload_bytes(zkdl_ctx* ctx, const void* host, size_t n, void** dev_out) {
    *dev_out = zk_alloc(ctx, n ? n : 4);
    if (!*dev_out) return ZKDL_ENOMEM;
    if (!n) return ZKDL_OK;
    hipError_t e = hipMemcpyAsync(*dev_out, host, n, hipMemcpyHostToDevice, ctx->stream);
    if (e != hipSuccess) {
        ctx->last_hip = (int)e;
        return ZKDL_EHIP;
    }
    return ZKDL_OK;
}

// inverse maps by stack index: counting sort of the (k, j) entries (k in the top 3 bits of an
// entry, j in the other 29); maps_flat = the maps one after the other
static void build_inverse_maps(int K, const int32_t* const* maps, const uint64_t* map_len, uint64_t N,
                               std::vector<uint32_t>& row_off, std::vector<uint32_t>& ent,
                               std::vector<uint32_t>& maps_flat) {
    uint64_t total = 0;
    for (int k = 0; k < K; ++k) total += map_len[k];
    row_off.assign(N + 1, 0);
    ent.assign(total ? total : 1, 0);
    maps_flat.assign(total ? total : 1, 0);
    for (int k = 0; k < K; ++k)
        for (uint64_t j = 0; j < map_len[k]; ++j)
            if (maps[k][j] >= 0) ++row_off[(size_t)maps[k][j] + 1];
    for (uint64_t i = 0; i < N; ++i) row_off[i + 1] += row_off[i];
    std::vector<uint32_t> cur(row_off.begin(), row_off.end() - 1);
    uint64_t f = 0;
    for (int k = 0; k < K; ++k)
        for (uint64_t j = 0; j < map_len[k]; ++j) {
            maps_flat[f++] = (uint32_t)maps[k][j];
            if (maps[k][j] >= 0) ent[cur[(size_t)maps[k][j]]++] = ((uint32_t)k << 29) | (uint32_t)j;
        }
}

extern "C" int reindex_prove(zkdl_ctx* ctx, const zkdl_tensor* X, int K, const int32_t* const* maps,
                             const uint64_t* map_len, const zkdl_fr* const* points, const zkdl_fr* u,
                             zkdl_transcript* tr, uint8_t* proof, size_t* proof_len, zkdl_fr* claims,
                             zkdl_fr* points_out, size_t* npoints) {
    if (!ctx || !X || !tr || !maps || !map_len || K < 1 || K > ZKDL_REINDEX_MAX_K || X->ndim < 1) return ZKDL_EINVAL;
    const uint64_t N = X->shape[0], D = X->numel / N;
    if (!is_pow2(N) || !is_pow2(D) || N > ((uint64_t)1 << 29) || D > ((uint64_t)1 << 31)) return ZKDL_EINVAL;
    const int ln = ilog2_u64(N), ld = ilog2_u64(D);
    if (ld > 0 && !u) return ZKDL_EINVAL;
    uint64_t total = 0;
    int lk[ZKDL_REINDEX_MAX_K], npts = ld;
    for (int k = 0; k < K; ++k) {
        if (!maps[k] || !is_pow2(map_len[k]) || map_len[k] > ((uint64_t)1 << 29)) return ZKDL_EINVAL;
        lk[k] = ilog2_u64(map_len[k]);
        if (lk[k] > 0 && (!points || !points[k])) return ZKDL_EINVAL;
        for (uint64_t j = 0; j < map_len[k]; ++j)
            if (maps[k][j] < -1 || (int64_t)maps[k][j] >= (int64_t)N) return ZKDL_EINVAL;
        total += map_len[k];
        npts += lk[k];
    }
    if (total >= ((uint64_t)1 << 32) || K + ln > ZK_MAX_CHAL) return ZKDL_EINVAL;

    // the statement's public part, hashed; all points in one buffer (u first)
    HostSha hs;
    hs.u32((uint32_t)N);
    hs.u32((uint32_t)D);
    hs.u32((uint32_t)K);
    for (int k = 0; k < K; ++k) {
        hs.u32((uint32_t)map_len[k]);
        for (uint64_t j = 0; j < map_len[k]; ++j) hs.u32((uint32_t)maps[k][j]);
    }
    std::vector<uint8_t> pts((size_t)(npts > 0 ? npts : 1) * 32);
    size_t at = (size_t)ld * 32;
    if (ld > 0) memcpy(pts.data(), u, (size_t)ld * 32);
    for (int k = 0; k < K; ++k) {
        if (lk[k] > 0) memcpy(pts.data() + at, points[k], (size_t)lk[k] * 32);
        hs.bytes(pts.data() + at, (size_t)lk[k] * 32);
        at += (size_t)lk[k] * 32;
    }
    hs.bytes(pts.data(), (size_t)ld * 32);
    uint32_t dgw[8];
    hs.digest_words(dgw);

    std::vector<uint32_t> row_off, ent, maps_flat;
    build_inverse_maps(K, maps, map_len, N, row_off, ent, maps_flat);

    int rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    zk_absorb_words(ctx, "reindex", dgw, 8);
    uint32_t hdr[4] = {ZKRI_MAGIC, (uint32_t)N, (uint32_t)D, (uint32_t)K};
    zk_write_proof_words(ctx, hdr, 4);

    void *d_pts = nullptr, *d_row = nullptr, *d_ent = nullptr, *d_maps = nullptr;
    rc = upload_bytes(ctx, pts.data(), (size_t)npts * 32, &d_pts);
    if (rc == ZKDL_OK) rc = upload_bytes(ctx, row_off.data(), (N + 1) * 4, &d_row);
    if (rc == ZKDL_OK) rc = upload_bytes(ctx, ent.data(), total * 4, &d_ent);
    if (rc == ZKDL_OK) rc = upload_bytes(ctx, maps_flat.data(), total * 4, &d_maps);
    // X~(i, u) is taken in two steps over the row-major inner index x = (x_hi, x_lo): the low half of
    // u's coordinates first (N * hi dot products of length lo), then the high half
    const int lhi = ld / 2;
    const uint64_t hi = (uint64_t)1 << lhi, lo = D >> lhi;
    // device memory: Montgomery points | beta_hi | beta_lo | by_hi [N hi] | beta_k [len k] | T [N] | P [N] | work
    const size_t fr_elems = (size_t)(npts > 0 ? npts : 1) + hi + lo + N * hi + total + 2 * N;
    void* mem = rc == ZKDL_OK ? zk_alloc(ctx, fr_elems * 32 + zk_sumcheck_work_bytes(2, ln)) : nullptr;
    if (rc == ZKDL_OK && !mem) rc = ZKDL_ENOMEM;
    if (rc == ZKDL_OK) {
        Fr* pm = (Fr*)mem;
        uint32_t* w = (uint32_t*)mem + 8 * (size_t)(npts > 0 ? npts : 1);
        if (npts > 0) zk_launch_points_to_mont(ctx, (const uint8_t*)d_pts, npts, pm);
        BetaJob jobs[ZKDL_REINDEX_MAX_K + 2];
        ReindexJob job;
        job.K = K;
        jobs[0].point = pm;
        jobs[0].m = lhi;
        jobs[0].out = make_tab(w, hi);
        w += 8 * hi;
        jobs[1].point = pm + lhi;
        jobs[1].m = ld - lhi;
        jobs[1].out = make_tab(w, lo);
        w += 8 * lo;
        const FrTab by_hi = make_tab(w, N * hi);
        w += 8 * N * hi;
        const Fr* pk = pm + ld;
        const int32_t* mk = (const int32_t*)d_maps;
        for (int k = 0; k < K; ++k) {
            jobs[2 + k].point = pk;
            jobs[2 + k].m = lk[k];
            jobs[2 + k].out = make_tab(w, map_len[k]);
            job.map[k] = mk;
            job.len[k] = map_len[k];
            job.beta[k] = jobs[2 + k].out;
            w += 8 * map_len[k];
            pk += lk[k];
            mk += map_len[k];
        }
        job.row_off = (const uint32_t*)d_row;
        job.ent = (const uint32_t*)d_ent;
        const FrTab T = make_tab(w, N);
        w += 8 * N;
        const FrTab P = make_tab(w, N);
        w += 8 * N;
        rc = zk_build_beta_many(ctx, jobs, K + 2);
        if (rc == ZKDL_OK) {
            FrTab xs = make_tab(X->data, X->numel);
            const void* sp = X->kind == TK_FR ? (const void*)&xs : X->data;
            rc = zk_partial_eval(ctx, X->kind, sp, N * hi, lo, 1, jobs[1].out, by_hi);
            if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_FR, &by_hi, N, hi, 1, jobs[0].out, T);
        }
        if (rc == ZKDL_OK) rc = zk_reindex(ctx, job, T, P, ln, w);
    }
    int ids[ZKDL_REINDEX_MAX_K + 2];
    for (int k = 0; k < K; ++k) ids[k] = 8 + k;
    ids[K] = 0;
    ids[K + 1] = 1;
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, ids, K + 2, claims);
    zk_free(ctx, mem);
    zk_free(ctx, d_pts);
    zk_free(ctx, d_row);
    zk_free(ctx, d_ent);
    zk_free(ctx, d_maps);
    return rc != ZKDL_OK ? rc : rc2;
}

// ---------------------------------------------------------------------------
// several claims on one tensor -> one
// ---------------------------------------------------------------------------
static const uint32_t ZKMG_MAGIC = 0x474D4B5Au;

// Device part shared by the entry point and the linked aggregate: K points of d coordinates each,
// point k = the challenges from `points[k]` on (device, Montgomery form); x = the tensor as field
// elements.  `keep` receives the work memory (to be freed once the stream has drained).
static int enqueue_merge(zkdl_ctx* ctx, int K, const Fr* const* points, FrTab x, int d, std::vector<void*>& keep) {
    if (ctx->n_chal + K + d > ZK_MAX_CHAL) return ZKDL_EINVAL;
    const uint64_t n = (uint64_t)1 << d;
    uint32_t hdr[4] = {ZKMG_MAGIC, (uint32_t)d, (uint32_t)K, 0};
    zk_write_proof_words(ctx, hdr, 4);
    void* mem = zk_alloc(ctx, (size_t)(K + 1) * n * 32 + zk_sumcheck_work_bytes(2, d));
    if (!mem) return ZKDL_ENOMEM;
    keep.push_back(mem);
    uint32_t* w = (uint32_t*)mem;
    BetaJob jobs[ZKDL_REINDEX_MAX_K];
    FrTab beta[ZKDL_REINDEX_MAX_K];
    for (int k = 0; k < K; ++k) {
        jobs[k].point = points[k];
        jobs[k].m = d;
        jobs[k].out = beta[k] = make_tab(w, n);
        w += 8 * n;
    }
    const FrTab P = make_tab(w, n);
    w += 8 * n;
    int rc = zk_build_beta_many(ctx, jobs, K);
    if (rc == ZKDL_OK) rc = zk_merge(ctx, K, beta, x, P, d, w);
    return rc;
}

extern "C" int claims_merge_prove(zkdl_ctx* ctx, const zkdl_tensor* X, int K, const zkdl_fr* const* points,
                                  zkdl_transcript* tr, uint8_t* proof, size_t* proof_len, zkdl_fr* claims,
                                  zkdl_fr* points_out, size_t* npoints) {
    if (!ctx || !X || !tr || K < 1 || K > ZKDL_REINDEX_MAX_K || !is_pow2(X->numel)) return ZKDL_EINVAL;
    const int d = ilog2_u64(X->numel);
    if (d > 0 && !points) return ZKDL_EINVAL;
    if (d > 30) return ZKDL_EINVAL;
    std::vector<uint8_t> pts((size_t)(K * d > 0 ? K * d : 1) * 32);
    for (int k = 0; k < K && d > 0; ++k) {
        if (!points[k]) return ZKDL_EINVAL;
        for (int i = 0; i < d; ++i)
            if (!fr_bytes_canonical(points[k][i].le)) return ZKDL_EINVAL;
        memcpy(pts.data() + (size_t)k * d * 32, points[k], (size_t)d * 32);
    }
    HostSha hs;
    hs.u32((uint32_t)d);
    hs.u32((uint32_t)K);
    hs.bytes(pts.data(), (size_t)K * d * 32);
    uint32_t dgw[8];
    hs.digest_words(dgw);
    int rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    zk_absorb_words(ctx, "merge", dgw, 8);
    void* d_pts = nullptr;
    Fr* pm = (Fr*)zk_alloc(ctx, pts.size());
    FrView view;
    view.scratch = nullptr;
    std::vector<void*> keep;
    rc = pm ? upload_bytes(ctx, pts.data(), (size_t)K * d * 32, &d_pts) : ZKDL_ENOMEM;
    if (rc == ZKDL_OK) rc = as_fr(ctx, X, &view);
    if (rc == ZKDL_OK) {
        zk_launch_points_to_mont(ctx, (const uint8_t*)d_pts, K * d, pm);
        const Fr* pk[ZKDL_REINDEX_MAX_K];
        for (int k = 0; k < K; ++k) pk[k] = pm + (size_t)k * d;
        rc = enqueue_merge(ctx, K, pk, view.tab, d, keep);
    }
    int ids[ZKDL_REINDEX_MAX_K + 2];
    for (int k = 0; k < K; ++k) ids[k] = 8 + k;
    ids[K] = 0;
    ids[K + 1] = 1;
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, ids, K + 2, claims);
    for (void* p : keep) zk_free(ctx, p);
    zk_free(ctx, view.scratch);
    zk_free(ctx, pm);
    zk_free(ctx, d_pts);
    return rc != ZKDL_OK ? rc : rc2;
}

static const uint32_t ZKMS_MAGIC = 0x534D4B5Au;

extern "C" int claims_merge_stack_prove(zkdl_ctx* ctx, const zkdl_tensor* X, int K, const zkdl_fr* const* points,
                                        zkdl_transcript* tr, uint8_t* proof, size_t* proof_len, zkdl_fr* claims,
                                        zkdl_fr* points_out, size_t* npoints) {
    if (!ctx || !X || !tr || K < 1 || K > ZKDL_REINDEX_MAX_K || X->ndim < 1 || !is_pow2(X->numel)) return ZKDL_EINVAL;
    const uint64_t N = X->shape[0], D = X->numel / N;
    // the row-major inner index as (rows, cols) with about equally many bits each: X~(i, v) is taken
    // over the columns first
    const uint64_t rows = (uint64_t)1 << (ilog2_u64(D) / 2), cols = D / rows;
    const int d = ilog2_u64(X->numel);
    if (d > 0 && !points) return ZKDL_EINVAL;
    if (N > ((uint64_t)1 << 29) || D > ((uint64_t)1 << 29)) return ZKDL_EINVAL;
    std::vector<uint8_t> pts((size_t)(K * d > 0 ? K * d : 1) * 32);
    for (int k = 0; k < K && d > 0; ++k) {
        if (!points[k]) return ZKDL_EINVAL;
        for (int i = 0; i < d; ++i)
            if (!fr_bytes_canonical(points[k][i].le)) return ZKDL_EINVAL;
        memcpy(pts.data() + (size_t)k * d * 32, points[k], (size_t)d * 32);
    }
    HostSha hs;
    hs.u32((uint32_t)N);
    hs.u32((uint32_t)D);
    hs.u32((uint32_t)K);
    hs.bytes(pts.data(), (size_t)K * d * 32);
    uint32_t dgw[8];
    hs.digest_words(dgw);
    int rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    zk_absorb_words(ctx, "merge_stack", dgw, 8);
    uint32_t hdr[4] = {ZKMS_MAGIC, (uint32_t)N, (uint32_t)D, (uint32_t)K};
    zk_write_proof_words(ctx, hdr, 4);
    void* d_pts = nullptr;
    Fr* pm = (Fr*)zk_alloc(ctx, pts.size());
    std::vector<void*> keep;
    rc = pm ? upload_bytes(ctx, pts.data(), (size_t)K * d * 32, &d_pts) : ZKDL_ENOMEM;
    FrTab xs = make_tab(X->data, X->numel);
    if (rc == ZKDL_OK) {
        zk_launch_points_to_mont(ctx, (const uint8_t*)d_pts, K * d, pm);
        StackMergeJob job = {};
        job.K = K;
        for (int k = 0; k < K; ++k) job.point[k] = pm + (size_t)k * d;
        job.kind = X->kind;
        job.X = X->kind == TK_FR ? (const void*)&xs : X->data;
        job.N = N;
        job.rows = rows;
        job.cols = cols;
        rc = zk_stack_merge(ctx, job, keep);
    }
    int ids[ZKDL_REINDEX_MAX_K + 2];
    for (int k = 0; k < K; ++k) ids[k] = 8 + k;
    ids[K] = 0;
    ids[K + 1] = 1;
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, ids, K + 2, claims);
    for (void* p : keep) zk_free(ctx, p);
    zk_free(ctx, pm);
    zk_free(ctx, d_pts);
    return rc != ZKDL_OK ? rc : rc2;
}

// ---------------------------------------------------------------------------
// zkReLU and the aggregated proof
// ---------------------------------------------------------------------------
static int stage_ints(zkdl_ctx* ctx, const int64_t* host, uint64_t n, void** dev_out) {
    *dev_out = zk_alloc(ctx, n * 8);
    if (!*dev_out) return ZKDL_ENOMEM;
    hipError_t e = hipMemcpyAsync(*dev_out, host, n * 8, hipMemcpyHostToDevice, ctx->stream);
    if (e != hipSuccess) {
        ctx->last_hip = (int)e;
        return ZKDL_EHIP;
    }
    return ZKDL_OK;
}

static const uint32_t ZKRL_MAGIC = 0x4C524B5Au;
static const uint32_t ZKAG_MAGIC = 0x47414B5Au;

// mode 0: all five points drawn.  mode 1 / 2: the four points of the input claims stand in
// chal[n_chal ..) already; 1 binds them through `digest` (8 words), 2 does not (they are
// functions of this transcript).
static int enqueue_zkrelu(zkdl_ctx* ctx, const int64_t* z_dev, const int64_t* ga_dev, uint64_t D, int Q,
                          int R, int mode, const uint32_t* digest) {
    if (!is_pow2(D) || Q < 1 || R < 1 || Q + R > 64 || Q + R < 2) return ZKDL_EINVAL;
    uint32_t hw[5] = {(uint32_t)ilog2_u64(D), (uint32_t)Q, (uint32_t)R, ga_dev ? 1u : 0u, (uint32_t)mode};
    if (mode == 0) {
        zk_absorb_words(ctx, "zkrelu", hw, 4);
    } else {
        zk_absorb_words(ctx, "zkrelu_at", hw, 5);
        if (mode == 1) zk_absorb_words(ctx, "u", digest, 8);
    }
    uint32_t hdr[8] = {ZKRL_MAGIC, hw[0], hw[1], hw[2], hw[3], hw[4], 0, 0};
    zk_write_proof_words(ctx, hdr, 8);
    return zk_zkrelu(ctx, z_dev, ga_dev, D, Q, R, mode != 0);
}

static int zkrelu_call(zkdl_ctx* ctx, const int64_t* Z, const int64_t* GA, uint64_t D, int Q, int R,
                       int src_on_device, const zkdl_fr* points, zkdl_transcript* tr, uint8_t* proof,
                       size_t* proof_len, zkdl_fr* claims, zkdl_fr* points_out, size_t* npoints) {
    if (!ctx || !Z || !tr) return ZKDL_EINVAL;
    if (!is_pow2(D) || D > ((uint64_t)1 << 30)) return ZKDL_EINVAL;
    const int li = ilog2_u64(D);
    int rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    void *zs = nullptr, *gs = nullptr, *d_pts = nullptr;
    uint32_t dgw[8] = {};
    if (points) {
        // the four points, in the order u_Z, u_A, u_GA, u_GZ: hashed, and placed where the
        // drawn ones would stand
        HostSha hs;
        hs.bytes(points, (size_t)4 * li * 32);
        hs.digest_words(dgw);
        if (li > 0) {
            rc = upload_bytes(ctx, points, (size_t)4 * li * 32, &d_pts);
            if (rc == ZKDL_OK) zk_launch_chal_set(ctx, ctx->n_chal, 4 * li, (const uint8_t*)d_pts, nullptr);
        }
    }
    const int64_t* zd = Z;
    const int64_t* gd = GA;
    if (rc == ZKDL_OK && !src_on_device) {
        rc = stage_ints(ctx, Z, D, &zs);
        zd = (const int64_t*)zs;
        if (rc == ZKDL_OK && GA) {
            rc = stage_ints(ctx, GA, D, &gs);
            gd = (const int64_t*)gs;
        }
    }
    if (rc == ZKDL_OK) rc = enqueue_zkrelu(ctx, zd, gd, D, Q, R, points ? 1 : 0, dgw);
    int ids[4] = {0, 1, 2, 3};
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, ids, 4, claims);
    zk_free(ctx, zs);
    zk_free(ctx, gs);
    zk_free(ctx, d_pts);
    return rc != ZKDL_OK ? rc : rc2;
}

extern "C" int zkrelu_prove(zkdl_ctx* ctx, const int64_t* Z, const int64_t* GA, uint64_t D, int Q, int R,
                            int src_on_device, zkdl_transcript* tr, uint8_t* proof, size_t* proof_len,
                            zkdl_fr* claims, zkdl_fr* points_out, size_t* npoints) {
    return zkrelu_call(ctx, Z, GA, D, Q, R, src_on_device, nullptr, tr, proof, proof_len, claims, points_out,
                       npoints);
}

extern "C" int zkrelu_prove_at(zkdl_ctx* ctx, const int64_t* Z, const int64_t* GA, uint64_t D, int Q, int R,
                               int src_on_device, const zkdl_fr* points, zkdl_transcript* tr, uint8_t* proof,
                               size_t* proof_len, zkdl_fr* claims, zkdl_fr* points_out, size_t* npoints) {
    if (!is_pow2(D) || (D > 1 && !points)) return ZKDL_EINVAL;
    static const zkdl_fr none = {};
    for (int i = 0; i < 4 * ilog2_u64(D); ++i)
        if (!fr_bytes_canonical(points[i].le)) return ZKDL_EINVAL;
    if (!points) points = &none;   // D = 1: no coordinates, the header still says "given"
    return zkrelu_call(ctx, Z, GA, D, Q, R, src_on_device, points, tr, proof, proof_len, claims, points_out,
                       npoints);
}

// ---- proof of the parameter update ------------------------------------------------------------
static const uint32_t ZKUP_MAGIC = 0x50554B5Au;

// zu = [g; -g], au = ReLU(rescale(zu)) with zkReLU's rescaling (round half up): au = [U+; U-]
__global__ __launch_bounds__(ZK_BLOCK) void k_update_witness(const int64_t* g, uint64_t D, int r_bits, int64_t* zu,
                                                             int64_t* au) {
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < D; i += (uint64_t)gridDim.x * blockDim.x) {
        const int64_t x = g[i];
        const int64_t nx = (int64_t)((uint64_t)0 - (uint64_t)x);
        zu[i] = x;
        zu[D + i] = nx;
        const int64_t up = (x >> r_bits) + ((x >> (r_bits - 1)) & 1);
        const int64_t un = (nx >> r_bits) + ((nx >> (r_bits - 1)) & 1);
        au[i] = up > 0 ? up : 0;
        au[D + i] = un > 0 ? un : 0;
    }
}

// ---- the list of claims a window leaves (host side, after the call has ended) ----
struct ClaimList {
    zkdl_claim* out;
    size_t n;
    const uint8_t* proof;   // the staged proof bytes of the call
    void add(uint32_t tensor, std::initializer_list<std::pair<int, int>> segs, const uint8_t* value_le) {
        zkdl_claim& c = out[n++];
        memset(&c, 0, sizeof c);
        c.tensor = tensor;
        for (const auto& sg : segs) {
            if (sg.second <= 0) continue;   // an axis of size one has no coordinates
            c.seg_off[c.nseg] = (uint32_t)sg.first;
            c.seg_len[c.nseg] = (uint32_t)sg.second;
            c.nseg += 1;
        }
        memcpy(c.value.le, value_le, 32);
    }
    void add_at(uint32_t tensor, std::initializer_list<std::pair<int, int>> segs, size_t proof_off) {
        add(tensor, segs, proof + proof_off);
    }
};

// capacity of the caller's list, checked before anything runs
static int claims_capacity(zkdl_claim* claims_out, size_t* nclaims, const zkdl_fr* points_out, size_t need) {
    if (!claims_out) return ZKDL_OK;
    if (!nclaims || !points_out) return ZKDL_EINVAL;
    if (*nclaims < need) {
        *nclaims = need;
        return ZKDL_ESMALL;
    }
    return ZKDL_OK;
}

// byte offsets inside a product-sumcheck block that starts at `at`
static size_t sc_claim0(size_t at) { return at + 16; }
static size_t sc_final(size_t at, int rounds, int degree, int k) {
    return at + 16 + 32 + (size_t)rounds * (degree + 1) * 32 + 32 * (size_t)k;
}

static Fr fr_from_le32(const uint8_t* p) {
    Fr x;
    memcpy(x.v, p, 32);
    return fr_to_mont(x);
}

extern "C" int update_prove(zkdl_ctx* ctx, const int64_t* GW, uint64_t D, int Q, int R, int src_on_device,
                            zkdl_transcript* tr, uint8_t* proof, size_t* proof_len, zkdl_fr* points_out, size_t* npoints,
                            zkdl_claim* claims_out, size_t* nclaims) {
    if (!ctx || !GW || !tr) return ZKDL_EINVAL;
    if (!is_pow2(D) || D > ((uint64_t)1 << 29) || Q < 1 || R < 1 || Q + R > 63) return ZKDL_EINVAL;
    int rc = claims_capacity(claims_out, nclaims, points_out, ZKDL_UPDATE_NCLAIMS);
    if (rc != ZKDL_OK) return rc;
    const int ld = ilog2_u64(D), li = ld + 1;
    int lj = 0;
    while ((1 << lj) < Q + R) ++lj;
    rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    void* gs = nullptr;
    const int64_t* gd = GW;
    if (!src_on_device) {
        rc = stage_ints(ctx, GW, D, &gs);
        gd = (const int64_t*)gs;
    }
    int64_t* zu = (int64_t*)zk_alloc(ctx, 2 * D * 8);
    int64_t* au = (int64_t*)zk_alloc(ctx, 2 * D * 8);
    void* bmem = zk_alloc(ctx, (D + 2) * 32);
    if (rc == ZKDL_OK && (!zu || !au || !bmem)) rc = ZKDL_ENOMEM;
    if (rc == ZKDL_OK && ctx->n_chal + ld + 1 + 4 * li > ZK_MAX_CHAL) rc = ZKDL_EINVAL;
    int cp = 0, c_rho = 0, cz = 0;
    size_t p_claims = 0, pz = 0, pz_end = 0;
    if (rc == ZKDL_OK) {
        const uint64_t blocks = (D + ZK_BLOCK - 1) / ZK_BLOCK;
        hipLaunchKernelGGL(k_update_witness, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(ZK_BLOCK), 0, ctx->stream,
                           gd, D, R, zu, au);
        uint32_t hw[3] = {(uint32_t)ld, (uint32_t)Q, (uint32_t)R};
        zk_absorb_words(ctx, "update", hw, 3);
        uint32_t hdr[8] = {ZKUP_MAGIC, hw[0], hw[1], hw[2], 0, 0, 0, 0};
        zk_write_proof_words(ctx, hdr, 8);
        cp = ctx->n_chal;
        zk_launch_draw(ctx, cp, ld);
        ctx->n_chal += ld;
        // the two claims Au~(0, p), Au~(1, p): the rows of Au [2, D] against beta~(p, .)
        const FrTab bp = make_tab(bmem, D), two = make_tab((uint32_t*)bmem + 8 * D, 2);
        rc = zk_build_beta(ctx, ctx->dev->chal + cp, ld, bp);
        if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_I64, au, 2, D, 1, bp, two);
        if (rc == ZKDL_OK) {
            const int claims_scal = 8;
            zk_launch_soa_to_aos(ctx, two, 2, ctx->dev->scal + claims_scal);
            // absorbed, then rho and u_Z in one draw: u_Z stands where zkReLU's first given point does
            p_claims = ctx->proof_len;
            c_rho = ctx->n_chal;
            zk_launch_absorb_claims(ctx, claims_scal, 2, (uint32_t)p_claims, c_rho, 1 + li);
            ctx->proof_len += 64;
            ctx->n_chal += 1;
            cz = ctx->n_chal;
            // u_A = (rho, p): the two claims lie on a line in the stack coordinate; the backward points
            // (unused: there is no gradient side) are copies of u_Z
            ChalIdx idx = {};
            int at = 0;
            idx.v[at++] = (int16_t)c_rho;
            for (int i = 0; i < ld; ++i) idx.v[at++] = (int16_t)(cp + i);
            for (int rep = 0; rep < 2; ++rep)
                for (int i = 0; i < li; ++i) idx.v[at++] = (int16_t)(cz + i);
            zk_launch_chal_set(ctx, cz + li, 3 * li, nullptr, &idx);
            pz = ctx->proof_len;
            rc = enqueue_zkrelu(ctx, zu, nullptr, 2 * D, Q, R, 2, nullptr);
            pz_end = ctx->proof_len;
        }
    }
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, nullptr, 0, nullptr);
    if (rc == ZKDL_OK && rc2 == ZKDL_OK && claims_out) {
        const uint8_t* sp = staged_proof(ctx);
        const uint8_t* chal_le = ((const DevState*)ctx->host_stage)->chal_le;
        ClaimList cl = {claims_out, 0, sp};
        // U~(p) = Au~(0, p) - Au~(1, p)
        const Fr u = fr_from_mont(fr_sub(fr_from_le32(sp + p_claims), fr_from_le32(sp + p_claims + 32)));
        cl.add(ZKDL_T_U, {{cp, ld}}, (const uint8_t*)u.v);
        // Zu~(u_Z) = (1 - 2 u_Z[0]) G_W~(u_Z[1:])
        const Fr u0 = fr_from_le32(chal_le + 32 * (size_t)cz);
        const Fr den = fr_sub(fr_one(), fr_add(u0, u0));
        const Fr zero = fr_zero();
        const Fr g = fr_eq(den, zero) ? zero : fr_mul(fr_from_le32(sp + pz + 32), host_inverse(den));
        const Fr gp = fr_from_mont(g);
        cl.add(ZKDL_T_GW, {{cz + 1, ld}}, (const uint8_t*)gp.v);
        const int c_v = cz + 5 * li + lj + 2, c_vm = c_v + li + lj + 3;
        cl.add_at(ZKDL_T_AUX, {{c_vm, 1}, {c_v, li}, {c_vm + 1, lj}}, pz_end - 64);
        *nclaims = cl.n;
    }
    zk_free(ctx, zu);
    zk_free(ctx, au);
    zk_free(ctx, bmem);
    zk_free(ctx, gs);
    return rc != ZKDL_OK ? rc : rc2;
}

extern "C" int aggregate_prove(zkdl_ctx* ctx, const zkdl_fcnn_witness* w, zkdl_transcript* tr,
                               uint8_t* proof, size_t* proof_len, zkdl_fr* points_out, size_t* npoints,
                               zkdl_claim* claims_out, size_t* nclaims) {
    if (!ctx || !w || !tr || !w->A || !w->W || !w->GZ || !w->Zr || !w->GA) return ZKDL_EINVAL;
    if (!is_pow2(w->L) || !is_pow2(w->B) || !is_pow2(w->width) || !is_pow2(w->T)) return ZKDL_EINVAL;
    const uint64_t N = (uint64_t)w->L * w->T;
    int rc = claims_capacity(claims_out, nclaims, points_out, ZKDL_AGGREGATE_NCLAIMS);
    if (rc != ZKDL_OK) return rc;
    rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    uint32_t hw[6] = {w->L, w->B, w->width, w->T, w->Q, w->R};
    zk_absorb_words(ctx, "aggregate", hw, 6);
    uint32_t hdr[8] = {ZKAG_MAGIC, w->L, w->B, w->width, w->T, w->Q, w->R, 0};
    zk_write_proof_words(ctx, hdr, 8);
    uint64_t sa[3] = {N, w->B, w->width}, sw[3] = {N, w->width, w->width};
    zkdl_tensor tA = {TK_I32, 3, {sa[0], sa[1], sa[2], 1}, N * w->B * w->width, (void*)w->A, false};
    zkdl_tensor tG = {TK_I32, 3, {sa[0], sa[1], sa[2], 1}, N * w->B * w->width, (void*)w->GZ, false};
    zkdl_tensor tW = {TK_I32, 3, {sw[0], sw[1], sw[2], 1}, N * w->width * w->width, (void*)w->W, false};
    // forward: Z = A W
    const int cf = ctx->n_chal;
    const size_t pf = ctx->proof_len;
    rc = enqueue_matmul(ctx, &tA, &tW, 0, 0, 0, 8, nullptr);
    // gradA: G_A^(l) = G_Z^(l+1) W^(l+1)T, slot of the last layer zero
    const int ca = ctx->n_chal;
    const size_t pa = ctx->proof_len;
    if (rc == ZKDL_OK) rc = enqueue_matmul(ctx, &tG, &tW, 0, 1, w->L, 12, nullptr);
    // gradW: G_W^(l) = A^(l-1)T G_Z^(l)
    const int cw = ctx->n_chal;
    const size_t pw = ctx->proof_len;
    if (rc == ZKDL_OK) rc = enqueue_matmul(ctx, &tA, &tG, 1, 0, 0, 16, nullptr);
    const int cz = ctx->n_chal;
    const size_t pz = ctx->proof_len;
    if (rc == ZKDL_OK) rc = enqueue_zkrelu(ctx, w->Zr, w->GA, N * w->B * w->width, (int)w->Q, (int)w->R, 0, nullptr);
    const size_t pend = ctx->proof_len;
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, nullptr, 0, nullptr);
    if (rc == ZKDL_OK && rc2 == ZKDL_OK && claims_out)
        *nclaims = zk_claims_unlinked(claims_out, staged_proof(ctx), w->L, w->B, w->width, w->T, w->Q, w->R, cf, pf, ca, pa,
                                      cw, pw, cz, pz, pend);
    return rc != ZKDL_OK ? rc : rc2;
}

// The 14 claims of an unlinked window from its proof bytes: c* = first challenge index and p* = proof offset of
// forward, gradA, gradW and zkReLU, pend = end of the proof.
size_t zk_claims_unlinked(zkdl_claim* claims_out, const uint8_t* proof, uint32_t L, uint32_t B, uint32_t width, uint32_t T,
                          uint32_t Q, uint32_t R, int cf, size_t pf, int ca, size_t pa, int cw, size_t pw, int cz, size_t pz,
                          size_t pend) {
    {
        const uint64_t N = (uint64_t)L * T;
        const int ln = ilog2_u64(N), lb = ilog2_u64(B), lw = ilog2_u64(width);
        const int li = ln + lb + lw;
        int lj = 0;
        while ((1u << lj) < Q + R) ++lj;
        ClaimList cl = {claims_out, 0, proof};
        // a family's challenges: w (ln), u0 (l1), u1 (l3), then the rounds v_n (ln), v_i (l2)
        {   // forward: l1 = lb, l2 = lw, l3 = lw
            const int u0 = cf + ln, u1 = u0 + lb, vn = u1 + lw, vi = vn + ln, rounds = ln + lw;
            cl.add_at(ZKDL_T_Z, {{cf, li}}, sc_claim0(pf));
            cl.add_at(ZKDL_T_A, {{vn, ln}, {u0, lb}, {vi, lw}}, sc_final(pf, rounds, 3, 1));
            cl.add_at(ZKDL_T_W, {{vn, ln}, {vi, lw}, {u1, lw}}, sc_final(pf, rounds, 3, 2));
        }
        {   // gradA: the same shape; its second operand is the transposed next layer's W
            const int u0 = ca + ln, u1 = u0 + lb, vn = u1 + lw, vi = vn + ln, rounds = ln + lw;
            cl.add_at(ZKDL_T_GA, {{ca, li}}, sc_claim0(pa));
            cl.add_at(ZKDL_T_GZ_NEXT, {{vn, ln}, {u0, lb}, {vi, lw}}, sc_final(pa, rounds, 3, 1));
            cl.add_at(ZKDL_T_W_NEXT, {{vn, ln}, {u1, lw}, {vi, lw}}, sc_final(pa, rounds, 3, 2));
        }
        {   // gradW: l1 = lw, l2 = lb, l3 = lw; its first operand is A transposed
            const int u0 = cw + ln, u1 = u0 + lw, vn = u1 + lw, vi = vn + ln, rounds = ln + lb;
            cl.add_at(ZKDL_T_GW, {{cw, ln + lw + lw}}, sc_claim0(pw));
            cl.add_at(ZKDL_T_A, {{vn, ln}, {vi, lb}, {u0, lw}}, sc_final(pw, rounds, 3, 1));
            cl.add_at(ZKDL_T_GZ, {{vn, ln}, {vi, lb}, {u1, lw}}, sc_final(pw, rounds, 3, 2));
        }
        // zkReLU: u_Z, u_A, u_GA, u_GZ (li each), u_bin (li + lj), r, r', rounds (li + lj), rho (3), merge (1 + lj)
        const int c_v = cz + 5 * li + lj + 2, c_vm = c_v + li + lj + 3;
        cl.add_at(ZKDL_T_ZR, {{cz, li}}, pz + 32);
        cl.add_at(ZKDL_T_A_RELU, {{cz + li, li}}, pz + 64);
        cl.add_at(ZKDL_T_GA, {{cz + 2 * li, li}}, pz + 96);
        cl.add_at(ZKDL_T_GZ_RELU, {{cz + 3 * li, li}}, pz + 128);
        cl.add_at(ZKDL_T_AUX, {{c_vm, 1}, {c_v, li}, {c_vm + 1, lj}}, pend - 64);
        return cl.n;
    }
}

// The same window with its three matrix-product families in the optimized aggregated form (App. B,
// Protocol tensor-op-aggr-optimized): the stack rounds carry f_t and fold two tables, not three.
static const uint32_t ZKAF_MAGIC = 0x46414B5Au;

extern "C" int aggregate_prove_ft(zkdl_ctx* ctx, const zkdl_fcnn_witness* w, zkdl_transcript* tr, uint8_t* proof,
                                  size_t* proof_len, zkdl_fr* points_out, size_t* npoints) {
    if (!ctx || !w || !tr || !w->A || !w->W || !w->GZ || !w->Zr || !w->GA) return ZKDL_EINVAL;
    if (!is_pow2(w->L) || !is_pow2(w->B) || !is_pow2(w->width) || !is_pow2(w->T)) return ZKDL_EINVAL;
    const uint64_t N = (uint64_t)w->L * w->T;
    int rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    uint32_t hw[6] = {w->L, w->B, w->width, w->T, w->Q, w->R};
    zk_absorb_words(ctx, "aggregate_ft", hw, 6);
    uint32_t hdr[8] = {ZKAF_MAGIC, w->L, w->B, w->width, w->T, w->Q, w->R, 0};
    zk_write_proof_words(ctx, hdr, 8);
    uint64_t sa[3] = {N, w->B, w->width}, sw[3] = {N, w->width, w->width};
    zkdl_tensor tA = {TK_I32, 3, {sa[0], sa[1], sa[2], 1}, N * w->B * w->width, (void*)w->A, false};
    zkdl_tensor tG = {TK_I32, 3, {sa[0], sa[1], sa[2], 1}, N * w->B * w->width, (void*)w->GZ, false};
    zkdl_tensor tW = {TK_I32, 3, {sw[0], sw[1], sw[2], 1}, N * w->width * w->width, (void*)w->W, false};
    rc = enqueue_matmul_ft(ctx, &tA, &tW, 0, 0, 0, 8);
    if (rc == ZKDL_OK) rc = enqueue_matmul_ft(ctx, &tG, &tW, 0, 1, w->L, 12);
    if (rc == ZKDL_OK) rc = enqueue_matmul_ft(ctx, &tA, &tG, 1, 0, 0, 16);
    if (rc == ZKDL_OK) rc = enqueue_zkrelu(ctx, w->Zr, w->GA, N * w->B * w->width, (int)w->Q, (int)w->R, 0, nullptr);
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, nullptr, 0, nullptr);
    return rc != ZKDL_OK ? rc : rc2;
}

// ---------------------------------------------------------------------------
// the same window with the claims linked (Sec. 3.2; Sec. 4, Eq. sc-reindex; Protocol zkdl)
// ---------------------------------------------------------------------------
static const uint32_t ZKAL_MAGIC = 0x4C414B5Au;

// The index maps of the re-indexings of a chained window on the device: K = 2 (the stack itself and the
// stack shifted by one layer) or K = 1 (the shifted stack alone).
struct RiPrepared {
    int K = 0;
    void *d_row = nullptr, *d_ent = nullptr, *d_maps = nullptr;
};

static int prepare_layer_maps(zkdl_ctx* ctx, uint64_t N, uint32_t L, int with_ident, RiPrepared& out) {
    out.K = with_ident ? 2 : 1;
    const uint64_t total = (uint64_t)out.K * N;
    out.d_row = zk_alloc(ctx, (N + 1) * 4);
    out.d_ent = zk_alloc(ctx, total * 4);
    out.d_maps = zk_alloc(ctx, total * 4);
    if (!out.d_row || !out.d_ent || !out.d_maps) return ZKDL_ENOMEM;
    zk_launch_layer_maps(ctx, (uint32_t)N, L, with_ident, (int32_t*)out.d_maps, (uint32_t*)out.d_row,
                         (uint32_t*)out.d_ent);
    return ZKDL_OK;
}

static void free_reindex_linked(zkdl_ctx* ctx, RiPrepared& p) {
    zk_free(ctx, p.d_row);
    zk_free(ctx, p.d_ent);
    zk_free(ctx, p.d_maps);
}

// One re-indexing sumcheck inside a larger proof: the stack X [N, D] of int32, the sub-stacks of
// `maps`, every stack point = the ln challenges from chal[point_chal[k]] on, the common point u =
// the ld challenges listed in u_idx.  The header frame carries N, D, K only (maps and points are
// fixed by the transcript so far).  The work memory is handed back in `keep` and must live until
// the stream has drained.
static int enqueue_reindex_linked(zkdl_ctx* ctx, const int32_t* X, uint64_t N, uint64_t rows, uint64_t cols,
                                  const RiPrepared& maps, const int* point_chal, const ChalIdx& u_idx,
                                  std::vector<void*>& keep) {
    const uint64_t D = rows * cols;
    const int ln = ilog2_u64(N), lr = ilog2_u64(rows), ld = ilog2_u64(D), K = maps.K;
    if (ld > ZK_CHAL_SET_MAX || ctx->n_chal + K + ln > ZK_MAX_CHAL - ZK_CHAL_SET_MAX) return ZKDL_EINVAL;
    const uint64_t total = (uint64_t)K * N;
    uint32_t hw[3] = {(uint32_t)N, (uint32_t)D, (uint32_t)K};
    zk_absorb_words(ctx, "reindex", hw, 3);
    uint32_t hdr[4] = {ZKRI_MAGIC, (uint32_t)N, (uint32_t)D, (uint32_t)K};
    zk_write_proof_words(ctx, hdr, 4);
    // the coordinates of u, gathered behind the challenges this call can draw
    const int u_at = ZK_MAX_CHAL - ZK_CHAL_SET_MAX;
    zk_launch_chal_set(ctx, u_at, ld, nullptr, &u_idx);
    const Fr* chal = ctx->dev->chal;
    // X~(n, u) in two steps, columns then rows: N * rows dot products of length cols keep the
    // machine busy where N products of length rows * cols would not
    void* mem = zk_alloc(ctx, (rows + cols + N * rows + total + 2 * N) * 32 + zk_sumcheck_work_bytes(2, ln));
    if (!mem) return ZKDL_ENOMEM;
    keep.push_back(mem);
    uint32_t* w = (uint32_t*)mem;
    BetaJob jobs[ZKDL_REINDEX_MAX_K + 2];
    ReindexJob job;
    job.K = K;
    jobs[0].point = chal + u_at;
    jobs[0].m = lr;
    jobs[0].out = make_tab(w, rows);
    w += 8 * rows;
    jobs[1].point = chal + u_at + lr;
    jobs[1].m = ld - lr;
    jobs[1].out = make_tab(w, cols);
    w += 8 * cols;
    const FrTab by_row = make_tab(w, N * rows);
    w += 8 * N * rows;
    for (int k = 0; k < K; ++k) {
        jobs[2 + k].point = chal + point_chal[k];
        jobs[2 + k].m = ln;
        jobs[2 + k].out = make_tab(w, N);
        job.map[k] = (const int32_t*)maps.d_maps + (uint64_t)k * N;
        job.len[k] = N;
        job.beta[k] = jobs[2 + k].out;
        w += 8 * N;
    }
    job.row_off = (const uint32_t*)maps.d_row;
    job.ent = (const uint32_t*)maps.d_ent;
    const FrTab T = make_tab(w, N);
    w += 8 * N;
    const FrTab P = make_tab(w, N);
    w += 8 * N;
    int rc = zk_build_beta_many(ctx, jobs, K + 2);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_I32, X, N * rows, cols, 1, jobs[1].out, by_row);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_FR, &by_row, N, rows, 1, jobs[0].out, T);
    if (rc == ZKDL_OK) rc = zk_reindex(ctx, job, T, P, ln, w);
    return rc;
}

extern "C" int aggregate_prove_linked(zkdl_ctx* ctx, const zkdl_fcnn_witness* w, zkdl_transcript* tr,
                                      uint8_t* proof, size_t* proof_len, zkdl_fr* points_out, size_t* npoints,
                                      zkdl_claim* claims_out, size_t* nclaims) {
    if (!ctx || !w || !tr || !w->A || !w->W || !w->GZ || !w->Zr || !w->GA) return ZKDL_EINVAL;
    if (!is_pow2(w->L) || !is_pow2(w->B) || !is_pow2(w->width) || !is_pow2(w->T)) return ZKDL_EINVAL;
    const uint64_t N = (uint64_t)w->L * w->T;
    const int ln = ilog2_u64(N), lb = ilog2_u64(w->B), lw = ilog2_u64(w->width);
    const int li = ln + lb + lw;
    if (4 * li > ZK_CHAL_SET_MAX || N > ((uint64_t)1 << 28)) return ZKDL_EINVAL;
    int rc = claims_capacity(claims_out, nclaims, points_out, ZKDL_AGGREGATE_LINKED_NCLAIMS);
    if (rc != ZKDL_OK) return rc;
    rc = call_begin(ctx, tr);
    if (rc != ZKDL_OK) return rc;
    // the index maps of the three re-indexings: the stack itself, and the stack whose slot (t, l)
    // is slot (t, l+1), zero for the last layer
    RiPrepared maps_a, maps_down;
    rc = prepare_layer_maps(ctx, N, w->L, 1, maps_a);
    if (rc == ZKDL_OK) rc = prepare_layer_maps(ctx, N, w->L, 0, maps_down);
    uint32_t hw[6] = {w->L, w->B, w->width, w->T, w->Q, w->R};
    zk_absorb_words(ctx, "aggregate_linked", hw, 6);
    uint32_t hdr[8] = {ZKAL_MAGIC, w->L, w->B, w->width, w->T, w->Q, w->R, 0};
    zk_write_proof_words(ctx, hdr, 8);
    uint64_t sa[3] = {N, w->B, w->width}, sw[3] = {N, w->width, w->width};
    zkdl_tensor tA = {TK_I32, 3, {sa[0], sa[1], sa[2], 1}, N * w->B * w->width, (void*)w->A, false};
    zkdl_tensor tG = {TK_I32, 3, {sa[0], sa[1], sa[2], 1}, N * w->B * w->width, (void*)w->GZ, false};
    zkdl_tensor tW = {TK_I32, 3, {sw[0], sw[1], sw[2], 1}, N * w->width * w->width, (void*)w->W, false};
    // challenges of a family: w (ln), u0 (l1), u1 (l3), then the rounds v_n (ln), v_i (l2)
    const int cf = ctx->n_chal;                       // forward: l1 = lb, l2 = lw, l3 = lw
    const size_t pf = ctx->proof_len;
    if (rc == ZKDL_OK) rc = enqueue_matmul(ctx, &tA, &tW, 0, 0, 0, 8, nullptr);
    const int ca = ctx->n_chal;                       // gradA: the same shape
    if (rc == ZKDL_OK) rc = enqueue_matmul(ctx, &tG, &tW, 0, 1, w->L, 12, nullptr);
    const int cw = ctx->n_chal;                       // gradW: l1 = lw, l2 = lb, l3 = lw
    const size_t pw = ctx->proof_len;
    if (rc == ZKDL_OK) rc = enqueue_matmul(ctx, &tA, &tG, 1, 0, 0, 16, nullptr);
    int cz = 0, ri_g_v = 0, c_ma_end = 0, c_mw_end = 0;   // challenge indices the list of claims refers to
    size_t pz = 0, pz_end = 0, p_rg_end = 0, p_ma_end = 0, p_mw_end = 0;
    const int f_u0 = cf + ln, f_vn = cf + ln + lb + lw, f_vi = f_vn + ln;
    const int a_u0 = ca + ln, a_u1 = a_u0 + lb, a_vn = ca + ln + lb + lw, a_vi = a_vn + ln;
    const int w_u0 = cw + ln, w_u1 = cw + ln + lw, w_vn = cw + ln + lw + lw, w_vi = w_vn + ln;
    const int f_u1 = f_u0 + lb;
    int ri_a_v = 0, ri_w_v = 0;   // first round challenge of the re-indexing sumchecks on A and W
    std::vector<void*> keep;
    if (rc == ZKDL_OK) {
        // zkReLU at the points the three families have left: u_Z = point of forward's claim_0,
        // u_A = point of its final on A, u_GA = point of gradA's claim_0, u_GZ = point of gradW's
        // final on G_Z
        ChalIdx idx = {};
        int at = 0;
        auto put = [&](int from, int count) {
            for (int i = 0; i < count; ++i) idx.v[at++] = (int16_t)(from + i);
        };
        put(cf, li);
        put(f_vn, ln), put(f_u0, lb), put(f_vi, lw);
        put(ca, li);
        put(w_vn, ln), put(w_vi, lb), put(w_u1, lw);
        if (ctx->n_chal + 4 * li > ZK_MAX_CHAL) rc = ZKDL_EINVAL;
        if (rc == ZKDL_OK) {
            zk_launch_chal_set(ctx, ctx->n_chal, 4 * li, nullptr, &idx);
            cz = ctx->n_chal;
            pz = ctx->proof_len;
            rc = enqueue_zkrelu(ctx, w->Zr, w->GA, N * w->B * w->width, (int)w->Q, (int)w->R, 2, nullptr);
            pz_end = ctx->proof_len;
        }
    }
    if (rc == ZKDL_OK) {
        // A: itself and its shifted stack (the ReLU outputs) at forward's stack point, u = (u0, v_i)
        {
            const int pts[2] = {f_vn, f_vn};
            ChalIdx u = {};
            for (int i = 0; i < lb; ++i) u.v[i] = (int16_t)(f_u0 + i);
            for (int i = 0; i < lw; ++i) u.v[lb + i] = (int16_t)(f_vi + i);
            ri_a_v = ctx->n_chal + 2;   // its two coefficients come first, then the ln rounds
            rc = enqueue_reindex_linked(ctx, w->A, N, w->B, w->width, maps_a, pts, u, keep);
        }
        // G_Z: gradA's first final is an evaluation of the shifted stack, u = (u0, v_i)
        if (rc == ZKDL_OK) {
            const int pts[1] = {a_vn};
            ChalIdx u = {};
            for (int i = 0; i < lb; ++i) u.v[i] = (int16_t)(a_u0 + i);
            for (int i = 0; i < lw; ++i) u.v[lb + i] = (int16_t)(a_vi + i);
            ri_g_v = ctx->n_chal + 1;   // one coefficient, then the ln rounds
            rc = enqueue_reindex_linked(ctx, w->GZ, N, w->B, w->width, maps_down, pts, u, keep);
            p_rg_end = ctx->proof_len;
        }
        // W: gradA's second final is an evaluation of the shifted, transposed stack: rows take u1
        if (rc == ZKDL_OK) {
            const int pts[1] = {a_vn};
            ChalIdx u = {};
            for (int i = 0; i < lw; ++i) u.v[i] = (int16_t)(a_u1 + i);
            for (int i = 0; i < lw; ++i) u.v[lw + i] = (int16_t)(a_vi + i);
            ri_w_v = ctx->n_chal + 1;
            rc = enqueue_reindex_linked(ctx, w->W, N, w->width, w->width, maps_down, pts, u, keep);
        }
    }
    // the two claims on A (re-indexing's, gradW's final on A^T) and on W (forward's final,
    // re-indexing's) become one each
    auto merge2 = [&](const int32_t* X, uint64_t rows, uint64_t cols, const ChalIdx& p0, const ChalIdx& p1) -> int {
        const int d = ln + ilog2_u64(rows) + ilog2_u64(cols);
        if (d > ZK_CHAL_SET_MAX / 2) return ZKDL_EINVAL;
        const int at0 = ZK_MAX_CHAL - ZK_CHAL_SET_MAX, at1 = at0 + ZK_CHAL_SET_MAX / 2;
        if (ctx->n_chal + 2 + 1 + d > at0) return ZKDL_EINVAL;
        uint32_t hw3[3] = {(uint32_t)N, (uint32_t)(rows * cols), 2};
        zk_absorb_words(ctx, "merge_stack", hw3, 3);
        uint32_t mh[4] = {ZKMS_MAGIC, hw3[0], hw3[1], 2};
        zk_write_proof_words(ctx, mh, 4);
        zk_launch_chal_set(ctx, at0, d, nullptr, &p0);
        zk_launch_chal_set(ctx, at1, d, nullptr, &p1);
        StackMergeJob job = {};
        job.K = 2;
        job.point[0] = ctx->dev->chal + at0;
        job.point[1] = ctx->dev->chal + at1;
        job.kind = TK_I32;
        job.X = X;
        job.N = N;
        job.rows = rows;
        job.cols = cols;
        return zk_stack_merge(ctx, job, keep);
    };
    // the re-indexing sumchecks' own challenges: K coefficients, then ln rounds
    if (rc == ZKDL_OK) {
        ChalIdx p0 = {}, p1 = {};
        int at = 0;
        auto put = [&](ChalIdx& p, int from, int count) {
            for (int i = 0; i < count; ++i) p.v[at++] = (int16_t)(from + i);
        };
        put(p0, ri_a_v, ln), put(p0, f_u0, lb), put(p0, f_vi, lw);
        at = 0;
        put(p1, w_vn, ln), put(p1, w_vi, lb), put(p1, w_u0, lw);
        rc = merge2(w->A, w->B, w->width, p0, p1);
        c_ma_end = ctx->n_chal;
        p_ma_end = ctx->proof_len;
        if (rc == ZKDL_OK) {
            ChalIdx q0 = {}, q1 = {};
            at = 0;
            put(q0, f_vn, ln), put(q0, f_vi, lw), put(q0, f_u1, lw);
            at = 0;
            put(q1, ri_w_v, ln), put(q1, a_u1, lw), put(q1, a_vi, lw);
            rc = merge2(w->W, w->width, w->width, q0, q1);
            c_mw_end = ctx->n_chal;
            p_mw_end = ctx->proof_len;
        }
    }
    int rc2 = call_end(ctx, tr, rc, proof, proof_len, points_out, npoints, nullptr, 0, nullptr);
    if (rc == ZKDL_OK && rc2 == ZKDL_OK && claims_out) {
        const uint8_t* sp = staged_proof(ctx);
        const uint8_t* chal_le = ((const DevState*)ctx->host_stage)->chal_le;
        ClaimList cl = {claims_out, 0, sp};
        int lj = 0;
        while ((1u << lj) < w->Q + w->R) ++lj;
        const int lt = ilog2_u64(w->T), ll = ln - lt;
        // a merge on a stack draws 2 coefficients, runs 1 + ld inner rounds (rho, v) and ln outer rounds (v_n);
        // its last final is the claim left on the stack at (v_n, v)
        const int ld_a = lb + lw, ld_w = lw + lw;
        cl.add_at(ZKDL_T_A, {{c_ma_end - ln, ln}, {c_ma_end - ln - ld_a, ld_a}}, p_ma_end - 32);
        cl.add_at(ZKDL_T_W, {{c_mw_end - ln, ln}, {c_mw_end - ln - ld_w, ld_w}}, p_mw_end - 32);
        // G_Z: the re-indexing's final at (its rounds, gradA's u0, gradA's v_i)
        cl.add_at(ZKDL_T_GZ, {{ri_g_v, ln}, {a_u0, lb}, {a_vi, lw}}, p_rg_end - 32);
        // the last layer's share of forward's claim_0 and of gradW's final on G_Z, divided by beta~ of the
        // layer coordinates (the low ll ones of the stack point) at L - 1, whose bits are all ones
        auto last_layer = [&](size_t total_off, size_t part_off, int stack_chal) {
            Fr fac = fr_one();
            for (int c = lt; c < ln; ++c) fac = fr_mul(fac, fr_from_le32(chal_le + 32 * (size_t)(stack_chal + c)));
            Fr diff = fr_sub(fr_from_le32(sp + total_off), fr_from_le32(sp + part_off));
            Fr zero = fr_zero();
            Fr val = fr_eq(fac, zero) ? zero : fr_mul(diff, host_inverse(fac));
            return fr_from_mont(val);
        };
        (void)ll;
        const int rounds_w = ln + lb;
        Fr zl = last_layer(sc_claim0(pf), pz + 32, cf);
        Fr gl = last_layer(sc_final(pw, rounds_w, 3, 2), pz + 128, w_vn);
        cl.add(ZKDL_T_Z_LAST, {{cf, lt}, {f_u0, lb + lw}}, (const uint8_t*)zl.v);
        cl.add(ZKDL_T_GZ_LAST, {{w_vn, lt}, {w_vi, lb}, {w_u1, lw}}, (const uint8_t*)gl.v);
        cl.add_at(ZKDL_T_GW, {{cw, ln + lw + lw}}, sc_claim0(pw));
        // zkReLU with given points: the 4 li given coordinates, u_bin (li + lj), r, r', rounds, rho, merge rounds
        const int c_v = cz + 5 * li + lj + 2, c_vm = c_v + li + lj + 3;
        cl.add_at(ZKDL_T_AUX, {{c_vm, 1}, {c_v, li}, {c_vm + 1, lj}}, pz_end - 64);
        *nclaims = cl.n;
    }
    for (void* p : keep) zk_free(ctx, p);
    free_reindex_linked(ctx, maps_a);
    free_reindex_linked(ctx, maps_down);
    return rc != ZKDL_OK ? rc : rc2;
}
