// Verifier of an aggregated proof (Sec. 2.2: the round check g_t(0) + g_t(1) = claim and the final check;
// App. A: the final claim of the combined zkReLU sumcheck; App. B: the verifier's side of both protocols),
// as one sequential program that runs on the GPU next to the prover (Sec. 6: verification is
// "predominantly sequential") and, compiled for the host, in the library's CPU self-checks.
// It replays the Fiat-Shamir transcript, so it re-derives every challenge itself.
//
// Returns 0 if the proof is accepted, else a code that names the first failed check
// (100 * stage + detail; stages: 1 header, 2 forward, 3 gradA, 4 gradW, 5 zkReLU, 6 merge of the aux claims).
#pragma once
#include "fr.cuh"
#include "sha256.cuh"
#if defined(__HIPCC__)
#include "dev_common.cuh"
#endif

#define VF_HD __host__ __device__ inline
// the building blocks are kept out of line on the device: the program runs once, from a cold instruction
// cache, so its size is its cost
#define VF_NI __host__ __device__ __noinline__ inline

namespace vf {

VF_HD Fr mulx(const Fr& a, const Fr& b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return fr_mul_ni(a, b);
#else
    return fr_mul(a, b);
#endif
}

constexpr uint32_t SC_MAGIC = 0x43534B5Au, ZKAG_MAGIC = 0x47414B5Au, ZKAF_MAGIC = 0x46414B5Au, ZKRL_MAGIC = 0x4C524B5Au,
                   FT_MAGIC = 0x46534B5Au, ZKAL_MAGIC = 0x4C414B5Au, ZKRI_MAGIC = 0x49524B5Au, ZKMS_MAGIC = 0x534D4B5Au,
                   ZKUP_MAGIC = 0x50554B5Au, ZKGA_MAGIC = 0x41474B5Au;
constexpr int MAX_CHAL = 1024;
constexpr int MAX_PT = 48;    // coordinates of a point that the program assembles from pieces
constexpr int MAX_RD = 4;   // elements one read may take

// the proof: 4-byte aligned on the device, every field at a multiple of four bytes
struct Reader {
    const uint8_t* p;
    size_t len, at;
    bool bad;
};

VF_HD uint32_t rd_u32(Reader& r) {
    if (r.at + 4 > r.len) {
        r.bad = true;
        return 0;
    }
    const uint8_t* q = r.p + r.at;
    r.at += 4;
#if defined(__HIP_DEVICE_COMPILE__)
    return *(const uint32_t*)q;
#else
    return (uint32_t)q[0] | ((uint32_t)q[1] << 8) | ((uint32_t)q[2] << 16) | ((uint32_t)q[3] << 24);
#endif
}

VF_HD bool below_modulus(const Fr& x) {
    bool below = false, above = false;
    for (int l = 7; l >= 0; --l) {
        if (below || above) break;
        if (x.v[l] > frc::MOD[l]) above = true;
        else if (x.v[l] < frc::MOD[l]) below = true;
    }
    return below;
}

// value at v of the polynomial through (k, g[k]), k < npts, npts = 3 or 4
VF_NI Fr lagrange_serial(const Fr& inv2, const Fr& inv6, const Fr* g, int npts, const Fr& v) {
    const Fr one = fr_one();
    const Fr v1 = fr_sub(v, one), v2 = fr_sub(v1, one), v3 = fr_sub(v2, one);
    if (npts == 4) {   // g(v) = (v-2)(v-3) [c0 (v-1) + c1 v] + v (v-1) [c2 (v-3) + c3 (v-2)], c = (-g0/6, g1/2, -g2/2, g3/6)
        const Fr c0 = fr_neg(mulx(g[0], inv6)), c1 = mulx(g[1], inv2), c2 = fr_neg(mulx(g[2], inv2)),
                 c3 = mulx(g[3], inv6);
        const Fr a = mulx(mulx(v2, v3), fr_add(mulx(c0, v1), mulx(c1, v)));
        const Fr b = mulx(mulx(v, v1), fr_add(mulx(c2, v3), mulx(c3, v2)));
        return fr_add(a, b);
    }
    // g(v) = (v-2) [c0 (v-1) + c1 v] + c2 v (v-1), c = (g0/2, -g1, g2/2)
    const Fr c0 = mulx(g[0], inv2), c1 = fr_neg(g[1]), c2 = mulx(g[2], inv2);
    return fr_add(mulx(v2, fr_add(mulx(c0, v1), mulx(c1, v))), mulx(c2, mulx(v, v1)));
}

// beta~(u, v) = prod_k (u_k v_k + (1 - u_k)(1 - v_k))
VF_NI Fr beta_point_serial(const Fr* u, const Fr* v, int m) {
    Fr acc = fr_one();
    const Fr one = fr_one();
    for (int k = 0; k < m; ++k)
        acc = mulx(acc, fr_add(mulx(u[k], v[k]), mulx(fr_sub(one, u[k]), fr_sub(one, v[k]))));
    return acc;
}

// multilinear extension of a table of J = 2^lj signed integers at wbar: sum_j tab[j] beta~(wbar, j)
VF_NI Fr mle_small_serial(const Fr* tab, int lj, const Fr* wbar) {
    Fr beta[64];
    beta[0] = fr_one();
    int len = 1;
    const Fr one = fr_one();
    for (int k = lj - 1; k >= 0; --k) {   // coordinate 0 pairs with the most significant bit
        for (int b = 0; b < len; ++b) {
            const Fr e = beta[b];
            beta[len + b] = mulx(e, wbar[k]);
            beta[b] = mulx(e, fr_sub(one, wbar[k]));
        }
        len *= 2;
    }
    Fr acc = fr_zero();
    for (int j = 0; j < len; ++j) acc = fr_add(acc, mulx(tab[j], beta[j]));
    return acc;
}

// beta~(u, j) for an index j of m bits (coordinate 0 pairs with the most significant bit)
VF_NI Fr beta_index(const Fr* u, int m, uint64_t j) {
    Fr acc = fr_one();
    const Fr one = fr_one();
    for (int k = 0; k < m; ++k) acc = mulx(acc, ((j >> (m - 1 - k)) & 1) ? u[k] : fr_sub(one, u[k]));
    return acc;
}

// sum over the slots j of a stack of 2^ln tensors, L per step, that are not a step's last layer, of
// beta~(u, j) beta~(v, j + 1): the weight P~(v) of the sub-stack "slot (t, l) <- slot (t, l + 1)" (Eq. sc-reindex)
VF_NI Fr shift_weight_serial(const Fr* u, const Fr* v, int ln, uint64_t L) {
    Fr acc = fr_zero();
    const uint64_t n = (uint64_t)1 << ln;
    for (uint64_t j = 0; j + 1 < n; ++j)
        if (j % L != L - 1) acc = fr_add(acc, mulx(beta_index(u, ln, j), beta_index(v, ln, j + 1)));
    return acc;
}

// What the program needs from its surroundings: the transcript, the challenges drawn so far, reading field
// elements of the proof.  Two implementations with the same members:
//   HostCtx  one thread, the byte-wise transcript of the host side;
//   DevCtx   one block of 256 threads that all run the program (same branches: the proof decides them) and
//            share the transcript steps out as the prover's kernels do.
//   rd_elems(r, n, out, src)        n <= MAX_RD consecutive elements: canonical (else r.bad), Montgomery form out
//   absorb_words(label, len, w, n)  a header frame of n <= 8 words
//   absorb_elems(label, src, n)     n elements as they stand in the proof, one-character label
//   absorb_draw1(label, src, n, skip1, v)  the same (skip1: without element 1), then a draw of one challenge
//   draw(n)                         a draw of n challenges; both return the index of the first
//   lagrange(g, npts, v), beta_point(u, v, m), mle_small(tab, lj, wbar), shift_weight(u, v, ln, L)
//                                   the verifier's own arithmetic: serial on
//                                   the host, one term per lane on the device
struct CtxBase {
    Fr* chal;       // room for MAX_CHAL challenges (Montgomery form)
    int n_chal;
    Fr inv2, inv6;
    bool overflow;
};

struct HostCtx : CtxBase {
    ts::State* s;

    __host__ void rd_elems(Reader& r, int n, Fr* out, const uint8_t** src) {
        for (int e = 0; e < n; ++e) out[e] = fr_zero();
        if (r.at + 32 * (size_t)n > r.len) {
            r.bad = true;
            return;
        }
        const uint8_t* q = r.p + r.at;
        if (src) *src = q;
        r.at += 32 * (size_t)n;
        for (int e = 0; e < n; ++e) {
            Fr x;
            for (int l = 0; l < 8; ++l) {
                const uint8_t* b = q + 32 * e + 4 * l;
                x.v[l] = (uint32_t)b[0] | ((uint32_t)b[1] << 8) | ((uint32_t)b[2] << 16) | ((uint32_t)b[3] << 24);
            }
            if (!below_modulus(x)) r.bad = true;
            out[e] = fr_to_mont(x);
        }
    }
    __host__ void absorb_words(const char* label, uint32_t label_len, const uint32_t* w, int n) {
        uint8_t b[32];
        for (int i = 0; i < n; ++i)
            for (int k = 0; k < 4; ++k) b[4 * i + k] = (uint8_t)(w[i] >> (8 * k));
        ts::absorb(*s, label, label_len, b, 4 * (uint64_t)n);
    }
    __host__ void absorb_elems(char label, const uint8_t* src, int n) { ts::absorb(*s, &label, 1, src, 32 * (uint64_t)n); }
    __host__ int draw(int n) {
        const int base = n_chal;
        if (base + n > MAX_CHAL) {
            overflow = true;
            return 0;
        }
        for (int i = 0; i < n; ++i) chal[base + i] = ts::challenge_elem(*s, (uint32_t)i);
        if (n > 0) ts::ratchet(*s);
        n_chal += n;
        return base;
    }
    __host__ Fr lagrange(const Fr* g, int npts, const Fr& v) const { return lagrange_serial(inv2, inv6, g, npts, v); }
    __host__ Fr beta_point(const Fr* u, const Fr* v, int m) const { return beta_point_serial(u, v, m); }
    __host__ Fr mle_small(const Fr* tab, int lj, const Fr* wbar) const { return mle_small_serial(tab, lj, wbar); }
    __host__ Fr shift_weight(const Fr* u, const Fr* v, int ln, uint64_t L) const { return shift_weight_serial(u, v, ln, L); }
    __host__ int absorb_draw1(char label, const uint8_t* src, int n, bool skip1, Fr* v) {
        uint8_t msg[32 * MAX_RD];
        int nm = 0;
        for (int e = 0; e < n; ++e) {
            if (skip1 && e == 1) continue;
            for (int b = 0; b < 32; ++b) msg[32 * nm + b] = src[32 * e + b];
            ++nm;
        }
        ts::absorb(*s, &label, 1, msg, 32 * (uint64_t)nm);
        const int ci = draw(1);
        *v = overflow ? fr_zero() : chal[ci];
        return ci;
    }
};

#if defined(__HIPCC__)
// LDS of the device side next to the transcript's
struct DevShared {
    Fr mont[MAX_RD];
    uint32_t bad[MAX_RD];
    uint32_t words[8];
};

// The block-wide transcript steps, kept out of line (one copy each) and given only pointers and scalars, so
// that a caller's own state can stay in registers across them.
__device__ __noinline__ inline void dev_absorb1(TsShared* S, char label, int n) { block_absorb1(*S, label, n, false); }
__device__ __noinline__ inline Fr dev_absorb_draw1(TsShared* S, DevState* st, char label, int count, int ci) {
    return block_absorb_draw1(*S, st, label, count, ci);
}
__device__ __noinline__ inline void dev_challenges(TsShared* S, DevState* st, int base, int n) {
    block_challenges(*S, st, base, n);
}
__device__ __noinline__ inline Fr dev_wave_lagrange(const Fr* coef, int npts, Fr v) { return wave_lagrange(coef, npts, v); }

struct DevCtx : CtxBase {
    TsShared* S;
    DevShared* D;
    DevState* st;   // chal = st->chal; the canonical forms go to st->chal_le as they are drawn

    __device__ __forceinline__ static Fr lane0(const Fr& x) {   // lane 0's value to every lane of the wave
        Fr y;
        for (int l = 0; l < 8; ++l) y.v[l] = __shfl(x.v[l], 0, 64);
        return y;
    }
    // g(v) with one coefficient per lane and the two-level evaluation of the prover's kernels; every wave does
    // the same, so nothing goes through memory afterwards
    __device__ __forceinline__ Fr lagrange(const Fr* g, int npts, const Fr& v) {
        const int tid = threadIdx.x;
        __syncthreads();
        if (tid < npts) {
            Fr ck = tid == 0 ? g[0] : tid == 1 ? g[1] : tid == 2 ? g[2] : g[3];
            if (npts == 3) {
                ck = (tid == 1) ? fr_neg(ck) : mulx(ck, inv2);
            } else {
                ck = mulx(ck, (tid == 0 || tid == 3) ? inv6 : inv2);
                if (tid == 0 || tid == 2) ck = fr_neg(ck);
            }
            S->tmp[tid] = ck;
        }
        __syncthreads();
        return lane0(dev_wave_lagrange(S->tmp, npts, v));
    }
    // product of the lanes' values over a wave (lane 0 holds it)
    __device__ static Fr wave_product(Fr x) {
        for (int off = 32; off >= 1; off >>= 1) {
            Fr y;
            for (int l = 0; l < 8; ++l) y.v[l] = __shfl_down(x.v[l], off, 64);
            x = mulx(x, y);
        }
        return x;
    }
    // u, v: the same values in every thread (challenges, or arrays every thread has built alike)
    __device__ Fr beta_point(const Fr* u, const Fr* v, int m) {
        const int lane = threadIdx.x & 63;
        const Fr one = fr_one();
        Fr acc = one;
        for (int k0 = 0; k0 < m; k0 += 64) {
            Fr t = one;
            if (k0 + lane < m) {
                const Fr a = u[k0 + lane], b = v[k0 + lane];
                t = fr_add(mulx(a, b), mulx(fr_sub(one, a), fr_sub(one, b)));
            }
            acc = mulx(acc, lane0(wave_product(t)));
        }
        return acc;
    }
    __device__ Fr shift_weight(const Fr* u, const Fr* v, int ln, uint64_t L) {   // one slot per lane at a time
        const int lane = threadIdx.x & 63;
        const uint64_t n = (uint64_t)1 << ln;
        Fr t = fr_zero();
        for (uint64_t j0 = 0; j0 < n; j0 += 64) {
            const uint64_t j = j0 + (uint64_t)lane;
            if (j + 1 < n && j % L != L - 1) t = fr_add(t, mulx(beta_index(u, ln, j), beta_index(v, ln, j + 1)));
        }
        for (int off = 32; off >= 1; off >>= 1) {
            Fr y;
            for (int l = 0; l < 8; ++l) y.v[l] = __shfl_down(t.v[l], off, 64);
            t = fr_add(t, y);
        }
        return lane0(t);
    }
    __device__ Fr mle_small(const Fr* tab, int lj, const Fr* wbar) {   // lj <= 6
        const int lane = threadIdx.x & 63;
        const Fr one = fr_one();
        Fr t = fr_zero();
        if (lane < (1 << lj)) {
            t = tab[lane];
            for (int k = 0; k < lj; ++k)   // coordinate 0 pairs with the most significant bit
                t = mulx(t, ((lane >> (lj - 1 - k)) & 1) ? wbar[k] : fr_sub(one, wbar[k]));
        }
        for (int off = 32; off >= 1; off >>= 1) {
            Fr y;
            for (int l = 0; l < 8; ++l) y.v[l] = __shfl_down(t.v[l], off, 64);
            t = fr_add(t, y);
        }
        return lane0(t);
    }

    __device__ __forceinline__ void rd_elems(Reader& r, int n, Fr* out, const uint8_t** src) {
        const int tid = threadIdx.x;
#pragma unroll
        for (int e = 0; e < MAX_RD; ++e)
            if (e < n) out[e] = fr_zero();
        if (r.at + 32 * (size_t)n > r.len) {
            r.bad = true;
            return;
        }
        const uint32_t* q = (const uint32_t*)(r.p + r.at);   // LDS when the kernel has staged the proof there
        if (src) *src = (const uint8_t*)q;
        r.at += 32 * (size_t)n;
        __syncthreads();   // the arrays may still be read from the call before
        if (tid < n) {     // one lane per element
            Fr x;
            for (int l = 0; l < 8; ++l) x.v[l] = q[8 * tid + l];
            D->bad[tid] = below_modulus(x) ? 0u : 1u;
            D->mont[tid] = mulx(fr_const(frc::R2), x);
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < MAX_RD; ++e) {
            if (e < n) {
                out[e] = D->mont[e];
                if (D->bad[e]) r.bad = true;
            }
        }
    }
    __device__ void absorb_words(const char* label, uint32_t label_len, const uint32_t* w, int n) {
        __syncthreads();
        if (threadIdx.x < (unsigned)n) D->words[threadIdx.x] = w[threadIdx.x];
        const uint32_t data_len = 4u * (uint32_t)n;
        const DevShared* d = D;
        auto frame = [=](uint32_t q) -> uint32_t {
            if (q == 0) return label_len;
            if (q <= label_len) return (uint32_t)(uint8_t)label[q - 1];
            const uint32_t k = q - 1 - label_len;
            if (k < 8) return k < 4 ? (data_len >> (8 * k)) & 0xffu : 0u;
            const uint32_t b = k - 8;
            return (d->words[b >> 2] >> (8 * (b & 3))) & 0xffu;
        };
        block_append(*S, 1u + label_len + 8u + data_len, frame, false);
    }
    __device__ __forceinline__ void fill_canon(const uint8_t* src, int n, bool skip1) {
        __syncthreads();
        const int tid = threadIdx.x;
        if (tid < 8 * n) {
            const int e = tid >> 3;
            if (!(skip1 && e == 1)) S->canon[(skip1 && e > 1) ? e - 1 : e][tid & 7] = ((const uint32_t*)src)[tid];
        }
    }
    __device__ __forceinline__ void absorb_elems(char label, const uint8_t* src, int n) {
        fill_canon(src, n, false);
        dev_absorb1(S, label, n);
    }
    __device__ __forceinline__ int draw(int n) {
        const int base = n_chal;
        if (base + n > MAX_CHAL) {
            overflow = true;
            return 0;
        }
        dev_challenges(S, st, base, n);
        __threadfence_block();   // every thread reads every challenge afterwards
        __syncthreads();
        n_chal += n;
        return base;
    }
    __device__ __forceinline__ int absorb_draw1(char label, const uint8_t* src, int n, bool skip1, Fr* v) {
        const int ci = n_chal;
        if (ci + 1 > MAX_CHAL) {
            overflow = true;
            *v = fr_zero();
            return 0;
        }
        fill_canon(src, n, skip1);
        *v = dev_absorb_draw1(S, st, label, skip1 ? n - 1 : n, ci);
        __threadfence_block();
        __syncthreads();
        n_chal += 1;
        return ci;
    }
};
#endif

VF_HD int ilog2(uint64_t x) {   // -1 if x is no power of two
    int l = 0;
    if (x == 0) return -1;
    while (((uint64_t)1 << l) < x) ++l;
    return (((uint64_t)1 << l) == x) ? l : -1;
}

// The rounds of one SC block: every g_t(0) + g_t(1) against the running claim, the challenges re-derived
// (appended to c.chal).  `claim` holds claim_0 on entry (already checked / absorbed by the caller as the
// protocol says) and the final claim on return.  The rounds absorb g(0), g(2), .., g(degree) under "g".
// Returns 0 or a detail code.
template <class C>
VF_NI int rounds(C& c_io, Reader& r_io, int nrounds, int degree, Fr& claim_io, int* first_chal) {
    // work on copies: the caller's objects live in memory, these in registers
    C c = c_io;
    Reader r = r_io;
    Fr claim = claim_io;
    *first_chal = c.n_chal;
    int rc = 0;
    for (int t = 0; t < nrounds && rc == 0; ++t) {
        Fr g[MAX_RD];
        const uint8_t* src = nullptr;
        c.rd_elems(r, degree + 1, g, &src);
        if (r.bad) {
            rc = 1;
        } else if (!fr_eq(fr_add(g[0], g[1]), claim)) {   // Sec. 2.2
            rc = 2;
        } else {
            Fr v;
            c.absorb_draw1('g', src, degree + 1, true, &v);
            if (c.overflow) rc = 3;
            else claim = c.lagrange(g, degree + 1, v);
        }
    }
    c_io = c;
    r_io = r;
    claim_io = claim;
    return rc;
}

struct ScHeader {
    uint32_t n_finals, degree, rounds;
};

VF_HD bool rd_sc_header(Reader& r, ScHeader& h) {
    const uint32_t magic = rd_u32(r);
    h.n_finals = rd_u32(r);
    h.degree = rd_u32(r);
    h.rounds = rd_u32(r);
    return !r.bad && magic == SC_MAGIC;
}

// Eq. exm-matmul-batched, the prover's g_t form: header, draw (w, u0, u1), claim_0, rounds over (n, i), the
// finals (beta~(w, v_n), X0~, X1~) with beta~(w, v_n) recomputed and their product against the last claim.
struct MatmulOut {
    int cw, cv;        // first challenge of (w, u0, u1) and of the rounds (v_n, v_i)
    Fr claim0, f1, f2; // Y~(w, u0, u1), X0~(v_n, u0, v_i), X1~(v_n, v_i, u1)
};

template <class C>
VF_NI int matmul(C& c, Reader& r, uint64_t n, uint64_t d1, uint64_t d2, uint64_t d3, MatmulOut* out = nullptr) {
    const int ln = ilog2(n), l1 = ilog2(d1), l2 = ilog2(d2), l3 = ilog2(d3);
    ScHeader h;
    if (!rd_sc_header(r, h) || h.n_finals != 3 || h.degree != 3 || (int)h.rounds != ln + l2) return 10;
    const uint32_t words[4] = {(uint32_t)n, (uint32_t)d1, (uint32_t)d2, (uint32_t)d3};
    c.absorb_words("sumcheck_matmul", 15, words, 4);
    const int cw = c.draw(ln + l1 + l3);
    const uint8_t* src = nullptr;
    Fr claim;
    c.rd_elems(r, 1, &claim, &src);
    if (r.bad || c.overflow) return 11;
    c.absorb_elems('c', src, 1);
    const Fr claim0 = claim;
    int cv;
    const int rc = rounds(c, r, ln + l2, 3, claim, &cv);
    if (rc) return 20 + rc;
    const uint8_t* fsrc = nullptr;
    Fr f[3];
    c.rd_elems(r, 3, f, &fsrc);
    if (r.bad) return 12;
    c.absorb_elems('f', fsrc, 3);
    if (!fr_eq(f[0], c.beta_point(c.chal + cw, c.chal + cv, ln))) return 13;
    if (!fr_eq(mulx(mulx(f[0], f[1]), f[2]), claim)) return 14;
    if (out) {
        out->cw = cw;
        out->cv = cv;
        out->claim0 = claim0;
        out->f1 = f[1];
        out->f2 = f[2];
    }
    return 0;
}

// The optimized aggregated protocol (App. B): stack rounds with f_t, (1 - w_t) f_t(0) + w_t f_t(1) = claim,
// then the single product's sumcheck (K = 2), whose claim_0 must be f_{n-1}(v_{n-1}).
template <class C>
VF_NI int matmul_ft(C& c, Reader& r, uint64_t n, uint64_t d1, uint64_t d2, uint64_t d3) {
    const int ln = ilog2(n), l1 = ilog2(d1), l2 = ilog2(d2), l3 = ilog2(d3);
    const uint32_t magic = rd_u32(r), pln = rd_u32(r), pl2 = rd_u32(r), zero = rd_u32(r);
    if (r.bad || magic != FT_MAGIC || (int)pln != ln || (int)pl2 != l2 || zero != 0) return 10;
    const uint32_t words[4] = {(uint32_t)n, (uint32_t)d1, (uint32_t)d2, (uint32_t)d3};
    c.absorb_words("sumcheck_matmul_ft", 18, words, 4);
    const int cw = c.draw(ln + l1 + l3);
    const uint8_t* src = nullptr;
    Fr claim;
    c.rd_elems(r, 1, &claim, &src);
    if (r.bad || c.overflow) return 11;
    c.absorb_elems('c', src, 1);
    const Fr one = fr_one();
    for (int t = 0; t < ln; ++t) {
        Fr f[3];
        const uint8_t* fs = nullptr;
        c.rd_elems(r, 3, f, &fs);
        if (r.bad) return 15;
        const Fr wt = c.chal[cw + t];
        if (!fr_eq(fr_add(mulx(fr_sub(one, wt), f[0]), mulx(wt, f[1])), claim)) return 16;
        Fr v;
        c.absorb_draw1('f', fs, 3, false, &v);
        if (c.overflow) return 17;
        claim = c.lagrange(f, 3, v);
    }
    ScHeader h;
    if (!rd_sc_header(r, h) || h.n_finals != 2 || h.degree != 2 || (int)h.rounds != l2) return 18;
    Fr inner0;
    c.rd_elems(r, 1, &inner0, nullptr);
    if (r.bad || !fr_eq(inner0, claim)) return 19;
    int cv;
    const int rc = rounds(c, r, l2, 2, claim, &cv);
    if (rc) return 20 + rc;
    const uint8_t* fsrc = nullptr;
    Fr f[2];
    c.rd_elems(r, 2, f, &fsrc);
    if (r.bad) return 12;
    c.absorb_elems('f', fsrc, 2);
    if (!fr_eq(mulx(f[0], f[1]), claim)) return 14;
    return 0;
}

// zkReLU (App. A and the merge of the three claims on aux).  given == nullptr: all five points drawn (mode 0).
// Otherwise the four points u_Z, u_A, u_GA, u_GZ (li coordinates each, one after the other) are the caller's,
// functions of this transcript already (mode 2), and only u_bin is drawn.
struct ZkOut {
    Fr c_in[4];
    int has_ga;
};

template <class C>
VF_NI int zkrelu(C& c, Reader& r, int li_expect, uint32_t q_expect, uint32_t r_expect, const Fr* given = nullptr,
                 ZkOut* out = nullptr) {
    const uint32_t magic = rd_u32(r), pli = rd_u32(r), q = rd_u32(r), rb = rd_u32(r), has_ga = rd_u32(r), mode = rd_u32(r);
    const uint32_t pad0 = rd_u32(r), pad1 = rd_u32(r);
    if (r.bad || pad0 != 0 || pad1 != 0 || magic != ZKRL_MAGIC || (int)pli != li_expect || q != q_expect || rb != r_expect ||
        mode != (given ? 2u : 0u) || has_ga > 1)
        return 1;
    const int li = (int)pli, b = (int)(q + rb);
    if (b < 2 || b > 64 || rb < 1) return 1;
    int lj = 0;
    while ((1 << lj) < b) ++lj;
    const int J = 1 << lj;
    const uint8_t* csrc = nullptr;
    Fr c_in[4];
    c.rd_elems(r, 4, c_in, &csrc);
    ScHeader h, hm;
    if (!rd_sc_header(r, h) || h.n_finals != 3 || h.degree != 3 || (int)h.rounds != li + lj) return 2;
    const Fr *u_z, *u_a, *u_ga, *u_gz;
    int c_bin;
    if (given) {
        const uint32_t words[5] = {pli, q, rb, has_ga, mode};
        c.absorb_words("zkrelu_at", 9, words, 5);
        c_bin = c.draw(li + lj);
        u_z = given;
        u_a = given + li;
        u_ga = given + 2 * li;
        u_gz = given + 3 * li;
    } else {
        const uint32_t words[4] = {pli, q, rb, has_ga};
        c.absorb_words("zkrelu", 6, words, 4);
        const int cu = c.draw(5 * li + lj);   // u_Z, u_A, u_GA, u_GZ (li each), u_bin (li + lj)
        u_z = c.chal + cu;
        u_a = u_z + li;
        u_ga = u_a + li;
        u_gz = u_ga + li;
        c_bin = cu + 4 * li;
    }
    if (r.bad || c.overflow) return 3;
    c.absorb_elems('c', csrc, 4);
    const int cr = c.draw(2);
    if (c.overflow) return 3;
    if (out) {
        for (int k = 0; k < 4; ++k) out->c_in[k] = c_in[k];
        out->has_ga = (int)has_ga;
    }
    const Fr rr = c.chal[cr], rp = c.chal[cr + 1], r2 = mulx(rr, rr);
    const Fr w_z = r2, w_a = rr, w_ga = mulx(rp, r2), w_gz = mulx(rp, rr);
    Fr claim;
    c.rd_elems(r, 1, &claim, nullptr);
    const Fr expect0 = fr_add(fr_add(mulx(w_z, c_in[0]), mulx(w_a, c_in[1])), fr_add(mulx(w_ga, c_in[2]), mulx(w_gz, c_in[3])));
    if (r.bad || !fr_eq(claim, expect0)) return 4;   // the combined claim is the weighted sum of the input claims
    int cv;
    int rc = rounds(c, r, li + lj, 3, claim, &cv);
    if (rc) return 10 + rc;
    const uint8_t* fsrc = nullptr;
    Fr fin[3];
    c.rd_elems(r, 3, fin, &fsrc);
    if (r.bad) return 5;
    const Fr a0 = fin[0], a1 = fin[1], sg = fin[2];
    c.absorb_elems('f', fsrc, 3);
    // s_{Q+R} = (1, 2, .., 2^(B-2), -2^(B-1)) and s' = (0^(R-1), 1, 1, 2, .., 2^(Q-2), -2^(Q-1)), zero-padded
    Fr s_tab[64], sp_tab[64];
    for (int j = 0; j < J; ++j) s_tab[j] = sp_tab[j] = fr_zero();
    Fr pw = fr_one();
    for (int j = 0; j < b - 1; ++j) {
        s_tab[j] = pw;
        pw = fr_add(pw, pw);
    }
    s_tab[b - 1] = fr_neg(pw);                     // pw = 2^(B-1)
    sp_tab[rb - 1] = fr_one();
    pw = fr_one();
    for (int j = (int)rb; j < b - 1; ++j) {
        sp_tab[j] = pw;
        pw = fr_add(pw, pw);
    }
    sp_tab[b - 1] = fr_neg(pw);                    // pw = 2^(Q-1)
    const Fr* v_i = c.chal + cv;
    const Fr* wbar = c.chal + cv + li;
    const Fr s_w = c.mle_small(s_tab, lj, wbar), sp_w = c.mle_small(sp_tab, lj, wbar);
    const Fr b_bin = c.beta_point(c.chal + c_bin, c.chal + cv, li + lj);
    const Fr one = fr_one();
    const Fr ns = fr_sub(one, sg);
    auto side = [&](const Fr& a, const Fr& w_in, const Fr& w_out, const Fr* u_in, const Fr* u_out) {
        Fr t = mulx(mulx(mulx(w_in, c.beta_point(u_in, v_i, li)), a), s_w);
        t = fr_add(t, mulx(mulx(mulx(mulx(w_out, c.beta_point(u_out, v_i, li)), ns), a), sp_w));
        return fr_add(t, mulx(b_bin, fr_sub(mulx(a, a), a)));
    };
    const Fr fwd = side(a0, w_z, w_a, u_z, u_a);
    Fr bwd = mulx(mulx(mulx(w_ga, c.beta_point(u_ga, v_i, li)), a1), s_w);
    bwd = fr_add(bwd, mulx(mulx(mulx(mulx(w_gz, c.beta_point(u_gz, v_i, li)), ns), a1), sp_w));
    bwd = fr_add(bwd, mulx(mulx(rp, b_bin), fr_sub(mulx(a1, a1), a1)));
    if (!fr_eq(fr_add(fwd, bwd), claim)) return 6;   // App. A: the six equations at the challenge point
    // merge of the three claims on aux (degree 2 over 1 + lj variables)
    if (!rd_sc_header(r, hm) || hm.n_finals != 2 || hm.degree != 2 || (int)hm.rounds != 1 + lj) return 7;
    const int crho = c.draw(3);
    if (c.overflow) return 3;
    Fr mclaim;
    c.rd_elems(r, 1, &mclaim, nullptr);
    const Fr em = fr_add(fr_add(mulx(c.chal[crho], a0), mulx(c.chal[crho + 1], a1)), mulx(c.chal[crho + 2], sg));
    if (r.bad || !fr_eq(mclaim, em)) return 8;
    int cm;
    rc = rounds(c, r, 1 + lj, 2, mclaim, &cm);
    if (rc) return 100 + rc;
    const uint8_t* msrc = nullptr;
    Fr mf[2];
    c.rd_elems(r, 2, mf, &msrc);
    if (r.bad) return 5;
    const Fr m_f = mf[0], e_f = mf[1];
    c.absorb_elems('f', msrc, 2);
    // E~ at the merge's point: rho0 beta~((0, wbar), vm) + rho1 beta~((1, wbar), vm) + rho2 beta~((0, e_{B-1}), vm)
    Fr p0[8], p1[8], p2[8];
    p0[0] = fr_zero();
    p1[0] = fr_one();
    p2[0] = fr_zero();
    for (int k = 0; k < lj; ++k) {
        p0[1 + k] = wbar[k];
        p1[1 + k] = wbar[k];
        p2[1 + k] = (((b - 1) >> (lj - 1 - k)) & 1) ? fr_one() : fr_zero();
    }
    const Fr* vm = c.chal + cm;
    const Fr e_pub = fr_add(fr_add(mulx(c.chal[crho], c.beta_point(p0, vm, 1 + lj)), mulx(c.chal[crho + 1], c.beta_point(p1, vm, 1 + lj))),
                            mulx(c.chal[crho + 2], c.beta_point(p2, vm, 1 + lj)));
    if (!fr_eq(e_f, e_pub)) return 101;
    if (!fr_eq(mulx(m_f, e_f), mclaim)) return 102;
    return 0;
}

// One product sumcheck on two tables inside a re-indexing or a merge: header (2 finals, degree 2), claim_0
// against `expect` and absorbed, the rounds, the two finals absorbed, their product against the last claim.
template <class C>
VF_NI int product2(C& c, Reader& r, int nrounds, const Fr& expect, int* cv, Fr* f0, Fr* f1) {
    ScHeader h;
    if (!rd_sc_header(r, h) || h.n_finals != 2 || h.degree != 2 || (int)h.rounds != nrounds) return 1;
    const uint8_t* src = nullptr;
    Fr claim;
    c.rd_elems(r, 1, &claim, &src);
    if (r.bad || !fr_eq(claim, expect)) return 2;
    c.absorb_elems('c', src, 1);
    const int rc = rounds(c, r, nrounds, 2, claim, cv);
    if (rc) return 10 + rc;
    const uint8_t* fsrc = nullptr;
    Fr f[2];
    c.rd_elems(r, 2, f, &fsrc);
    if (r.bad) return 3;
    c.absorb_elems('f', fsrc, 2);
    if (!fr_eq(mulx(f[0], f[1]), claim)) return 4;
    *f0 = f[0];
    *f1 = f[1];
    return 0;
}

// K <= 2 claims on a stack [n, d] merged into one (Eq. sc-reindex; the "ZKMS" block inside a larger proof):
// pts[k] = the ln + ld coordinates of claim k, stack coordinates first.  On return claims[k] are the claims the
// block states, *cvn / *cv the first challenges of the point (v_n, v) of the one claim *left.
template <class C>
VF_NI int stack_merge(C& c, Reader& r, uint64_t n, uint64_t d, int K, const Fr* const* pts, Fr* claims, int* cvn, int* cv,
                      Fr* left) {
    const int ln = ilog2(n), ld = ilog2(d);
    int lk = 0;
    while ((1 << lk) < K) ++lk;
    const uint32_t magic = rd_u32(r), pn = rd_u32(r), pd = rd_u32(r), pk = rd_u32(r);
    if (r.bad || magic != ZKMS_MAGIC || pn != (uint32_t)n || pd != (uint32_t)d || (int)pk != K || K < 1 || K > 2) return 1;
    const uint32_t words[3] = {(uint32_t)n, (uint32_t)d, (uint32_t)K};
    c.absorb_words("merge_stack", 11, words, 3);
    const uint8_t* src = nullptr;
    c.rd_elems(r, K, claims, &src);
    if (r.bad) return 2;
    c.absorb_elems('c', src, K);
    const int cr = c.draw(K);
    if (c.overflow) return 3;
    Fr expect = fr_zero();
    for (int k = 0; k < K; ++k) expect = fr_add(expect, mulx(c.chal[cr + k], claims[k]));
    int c1;
    Fr ef, tf;
    int rc = product2(c, r, lk + ld, expect, &c1, &ef, &tf);
    if (rc) return 20 + rc;
    const Fr* rho = c.chal + c1;
    const Fr* v = c.chal + c1 + lk;
    Fr e_pub = fr_zero();
    for (int k = 0; k < K; ++k)
        e_pub = fr_add(e_pub, mulx(mulx(beta_index(rho, lk, (uint64_t)k), c.chal[cr + k]), c.beta_point(pts[k] + ln, v, ld)));
    if (!fr_eq(ef, e_pub)) return 4;
    int c2;
    Fr pf, xf;
    rc = product2(c, r, ln, tf, &c2, &pf, &xf);
    if (rc) return 40 + rc;
    Fr p_pub = fr_zero();
    for (int k = 0; k < K; ++k) p_pub = fr_add(p_pub, mulx(beta_index(rho, lk, (uint64_t)k), c.beta_point(pts[k], c.chal + c2, ln)));
    if (!fr_eq(pf, p_pub)) return 5;
    *cvn = c2;
    *cv = c1 + lk;
    *left = xf;
    return 0;
}

// Re-indexing of a stack of n = 2^ln tensors with L per step (Eq. sc-reindex; the "ZKRI" block inside a larger
// proof): K <= 2 sub-stacks, each the stack itself (shifted[k] == false) or the stack with slot (t, l) <- slot
// (t, l + 1) and a zero tensor for a step's last layer (shifted[k] == true), with its stack point stack_pts[k].
template <class C>
VF_NI int reindex_layers(C& c, Reader& r, uint64_t n, uint64_t L, uint64_t d, int K, const bool* shifted,
                         const Fr* const* stack_pts, Fr* claims, int* cv, Fr* left) {
    const int ln = ilog2(n);
    const uint32_t magic = rd_u32(r), pn = rd_u32(r), pd = rd_u32(r), pk = rd_u32(r);
    if (r.bad || magic != ZKRI_MAGIC || pn != (uint32_t)n || pd != (uint32_t)d || (int)pk != K || K < 1 || K > 2) return 1;
    const uint32_t words[3] = {(uint32_t)n, (uint32_t)d, (uint32_t)K};
    c.absorb_words("reindex", 7, words, 3);
    const uint8_t* src = nullptr;
    c.rd_elems(r, K, claims, &src);
    if (r.bad) return 2;
    c.absorb_elems('c', src, K);
    const int cr = c.draw(K);
    if (c.overflow) return 3;
    Fr expect = fr_zero();
    for (int k = 0; k < K; ++k) expect = fr_add(expect, mulx(c.chal[cr + k], claims[k]));
    Fr pw, xw;
    const int rc = product2(c, r, ln, expect, cv, &pw, &xw);
    if (rc) return 20 + rc;
    Fr p_pub = fr_zero();
    for (int k = 0; k < K; ++k) {
        const Fr wk = shifted[k] ? c.shift_weight(stack_pts[k], c.chal + *cv, ln, L) : c.beta_point(stack_pts[k], c.chal + *cv, ln);
        p_pub = fr_add(p_pub, mulx(c.chal[cr + k], wk));
    }
    if (!fr_eq(pw, p_pub)) return 4;
    *left = xw;
    return 0;
}

VF_HD void put_coords(Fr* dst, int* at, const Fr* src, int n) {
    for (int i = 0; i < n; ++i) dst[(*at)++] = src[i];
}

// The window with its claims chained ("ZKAL"): the three matrix products, zkReLU at the points they leave, the
// re-indexing of A, G_Z and W, the merges on A and W; every link between the parts is checked here (Sec. 3.2;
// Protocol zkdl: one claim per stack is left).  Stages in the codes: 2..4 the matrix products, 5 / 6 zkReLU,
// 7 the links, 8..10 the re-indexings, 11 / 12 the merges.
template <class C>
VF_NI int aggregate_linked(C& c, Reader& r, uint32_t L, uint32_t B, uint32_t width, uint32_t T, uint32_t Q, uint32_t R) {
    const uint32_t words[6] = {L, B, width, T, Q, R};
    c.absorb_words("aggregate_linked", 16, words, 6);
    const uint64_t n = (uint64_t)L * T;
    const int ln = ilog2(n), lb = ilog2(B), lw = ilog2(width), ll = ilog2(L), lt = ln - ll;
    if (ln + lb + lw + lw > MAX_PT) return 101;
    const uint64_t dims[3][3] = {{B, width, width}, {B, width, width}, {width, B, width}};
    MatmulOut m[3];
    for (int fam = 0; fam < 3; ++fam) {
        const int rc = matmul(c, r, n, dims[fam][0], dims[fam][1], dims[fam][2], &m[fam]);
        if (rc) return 100 * (2 + fam) + rc;
    }
    const MatmulOut &f = m[0], &g = m[1], &h = m[2];
    // challenge layout of a matrix product: w (ln), u0 (l1), u1 (l3) from cw; v_n (ln), v_i (l2) from cv
    const Fr *f_w = c.chal + f.cw, *f_u0 = f_w + ln, *f_u1 = f_u0 + lb, *f_vn = c.chal + f.cv, *f_vi = f_vn + ln;
    const Fr *g_w = c.chal + g.cw, *g_u0 = g_w + ln, *g_u1 = g_u0 + lb, *g_vn = c.chal + g.cv, *g_vi = g_vn + ln;
    const Fr *h_w = c.chal + h.cw, *h_u0 = h_w + ln, *h_u1 = h_u0 + lw, *h_vn = c.chal + h.cv, *h_vi = h_vn + ln;
    (void)h_w;
    const int li = ln + lb + lw;
    Fr given[4 * MAX_PT];
    int at = 0;
    put_coords(given, &at, f_w, li);                                                              // u_Z
    put_coords(given, &at, f_vn, ln), put_coords(given, &at, f_u0, lb), put_coords(given, &at, f_vi, lw);   // u_A
    put_coords(given, &at, g_w, li);                                                              // u_GA
    put_coords(given, &at, h_vn, ln), put_coords(given, &at, h_vi, lb), put_coords(given, &at, h_u1, lw);   // u_GZ
    ZkOut zk;
    int rc = zkrelu(c, r, li, Q, R, given, &zk);
    if (rc) return (rc >= 100 ? 600 + rc - 100 : 500 + rc);
    if (!fr_eq(zk.c_in[2], g.claim0)) return 701;   // G_A is the gradA family's product
    // the last layer's share of forward's claim_0 and of gradW's final on G_Z: where its weight beta~(layer
    // coordinates, L - 1) vanishes there is no share to take
    {
        Fr fac_f = fr_one(), fac_h = fr_one();
        for (int k = lt; k < ln; ++k) {
            fac_f = mulx(fac_f, f_w[k]);
            fac_h = mulx(fac_h, h_vn[k]);
        }
        const Fr zero = fr_zero();
        if (fr_eq(fac_f, zero) && !fr_eq(f.claim0, zk.c_in[0])) return 702;
        if (fr_eq(fac_h, zero) && !fr_eq(h.f2, zk.c_in[3])) return 703;
    }
    // A: itself and its shifted stack at forward's stack point
    Fr cl[2], a_left, gz_left, w_left;
    int c_ra, c_rg, c_rw;
    {
        const bool sh[2] = {false, true};
        const Fr* sp[2] = {f_vn, f_vn};
        rc = reindex_layers(c, r, n, L, (uint64_t)B * width, 2, sh, sp, cl, &c_ra, &a_left);
        if (rc) return 800 + rc;
        if (!fr_eq(cl[0], f.f1) || !fr_eq(cl[1], zk.c_in[1])) return 704;   // the next layer's input is this ReLU's output
    }
    {
        const bool sh[1] = {true};
        const Fr* sp[1] = {g_vn};
        rc = reindex_layers(c, r, n, L, (uint64_t)B * width, 1, sh, sp, cl, &c_rg, &gz_left);
        if (rc) return 900 + rc;
        if (!fr_eq(cl[0], g.f1)) return 705;
        rc = reindex_layers(c, r, n, L, (uint64_t)width * width, 1, sh, sp, cl, &c_rw, &w_left);
        if (rc) return 1000 + rc;
        if (!fr_eq(cl[0], g.f2)) return 706;
    }
    (void)gz_left;
    (void)c_rg;
    // the two claims on A and the two on W become one each
    Fr p0[MAX_PT], p1[MAX_PT], one_left;
    int cvn, cv;
    {
        at = 0;
        put_coords(p0, &at, c.chal + c_ra, ln), put_coords(p0, &at, f_u0, lb), put_coords(p0, &at, f_vi, lw);
        at = 0;
        put_coords(p1, &at, h_vn, ln), put_coords(p1, &at, h_vi, lb), put_coords(p1, &at, h_u0, lw);
        const Fr* pts[2] = {p0, p1};
        rc = stack_merge(c, r, n, (uint64_t)B * width, 2, pts, cl, &cvn, &cv, &one_left);
        if (rc) return 1100 + rc;
        if (!fr_eq(cl[0], a_left) || !fr_eq(cl[1], h.f1)) return 707;
    }
    {
        at = 0;
        put_coords(p0, &at, f_vn, ln), put_coords(p0, &at, f_vi, lw), put_coords(p0, &at, f_u1, lw);
        at = 0;
        put_coords(p1, &at, c.chal + c_rw, ln), put_coords(p1, &at, g_u1, lw), put_coords(p1, &at, g_vi, lw);
        const Fr* pts[2] = {p0, p1};
        rc = stack_merge(c, r, n, (uint64_t)width * width, 2, pts, cl, &cvn, &cv, &one_left);
        if (rc) return 1200 + rc;
        if (!fr_eq(cl[0], f.f2) || !fr_eq(cl[1], w_left)) return 708;
    }
    return 0;
}

// The proof of the parameter update ("ZKUP"; Sec. 5, Example FCNN, last item): the two claims a0 = Au~(0, p),
// a1 = Au~(1, p), the point rho on the line through them, then zkReLU's forward half on [G_W; -G_W] at
// u_A = (rho, p) and a drawn u_Z, whose claim on Au must be (1 - rho) a0 + rho a1.
// Stages in the codes: 13 header and claims, 15 / 16 zkReLU, 17 the links.
template <class C>
VF_NI int update(C& c, Reader& r, uint32_t ld, uint32_t Q, uint32_t R) {
    if (ld > 30 || Q + R > 63) return 1301;
    const uint32_t words[3] = {ld, Q, R};
    c.absorb_words("update", 6, words, 3);
    const int cp = c.draw((int)ld);
    if (c.overflow) return 1302;
    const uint8_t* src = nullptr;
    Fr a[2];
    c.rd_elems(r, 2, a, &src);
    if (r.bad) return 1303;
    c.absorb_elems('c', src, 2);
    const int li = (int)ld + 1;
    const int c_rho = c.draw(1 + li);
    if (c.overflow) return 1302;
    const int cz = c_rho + 1;
    Fr given[4 * MAX_PT];
    int at = 0;
    put_coords(given, &at, c.chal + cz, li);
    put_coords(given, &at, c.chal + c_rho, 1), put_coords(given, &at, c.chal + cp, (int)ld);
    put_coords(given, &at, c.chal + cz, li);
    put_coords(given, &at, c.chal + cz, li);
    ZkOut zk;
    const int rc = zkrelu(c, r, li, Q, R, given, &zk);
    if (rc) return (rc >= 100 ? 1600 + rc - 100 : 1500 + rc);
    if (zk.has_ga != 0) return 1701;
    const Fr rho = c.chal[c_rho];
    const Fr line = fr_add(a[0], mulx(rho, fr_sub(a[1], a[0])));
    if (!fr_eq(zk.c_in[1], line)) return 1702;   // zkReLU starts from the claim on the line
    const Fr zero = fr_zero();
    if (!fr_eq(zk.c_in[2], zero) || !fr_eq(zk.c_in[3], zero)) return 1703;
    return 0;
}

// The batched matrix product in the general aggregated form ("ZKGA"; Eq. tensor-op-aggr, Protocol tensor-op-aggr):
// stack rounds with f_t starting from the claim 0, the sumcheck over (i0, i1, j), and the final check
// beta~(u, v_i) (D2^-1 Y~ - X0~ X1~) = last claim.  Stage 18 in the codes.
template <class C>
VF_NI int matmul_general(C& c, Reader& r, uint32_t ln, uint32_t l1, uint32_t l3, uint32_t l2) {
    if (ln > 13 || l1 > 16 || l2 > 16 || l3 > 16) return 1801;
    const uint32_t words[4] = {1u << ln, 1u << l1, 1u << l2, 1u << l3};
    c.absorb_words("tensor_op_aggr", 14, words, 4);
    const int cw = c.draw((int)(ln + l1 + l3));
    if (c.overflow) return 1802;
    const Fr one = fr_one();
    Fr claim = fr_zero();
    for (uint32_t t = 0; t < ln; ++t) {
        Fr f[3];
        const uint8_t* fs = nullptr;
        c.rd_elems(r, 3, f, &fs);
        if (r.bad) return 1803;
        const Fr wt = c.chal[cw + (int)t];
        if (!fr_eq(fr_add(mulx(fr_sub(one, wt), f[0]), mulx(wt, f[1])), claim)) return 1804;
        Fr v;
        c.absorb_draw1('f', fs, 3, false, &v);
        if (c.overflow) return 1802;
        claim = c.lagrange(f, 3, v);
    }
    ScHeader h;
    if (!rd_sc_header(r, h) || h.n_finals != 3 || h.degree != 2 || h.rounds != l1 + l3 + l2) return 1805;
    Fr inner0;
    c.rd_elems(r, 1, &inner0, nullptr);
    if (r.bad || !fr_eq(inner0, claim)) return 1806;   // written, not absorbed: the transcript fixes it
    int cv;
    const int rc = rounds(c, r, (int)(l1 + l3 + l2), 2, claim, &cv);
    if (rc) return 1810 + rc;
    const uint8_t* fsrc = nullptr;
    Fr f[3];
    c.rd_elems(r, 3, f, &fsrc);
    if (r.bad) return 1807;
    c.absorb_elems('f', fsrc, 3);
    Fr dinv = one;
    for (uint32_t k = 0; k < l2; ++k) dinv = mulx(dinv, c.inv2);
    const Fr b = c.beta_point(c.chal + cw + (int)ln, c.chal + cv, (int)(l1 + l3));
    if (!fr_eq(mulx(b, fr_sub(mulx(dinv, f[0]), mulx(f[1], f[2]))), claim)) return 1808;
    return 0;
}

// A whole proof: a window ("ZKAG": g_t form; "ZKAF": f_t form for the matrix products; "ZKAL": the claims chained)
// a parameter update ("ZKUP") or a matrix product in the general aggregated form ("ZKGA").  The context's transcript is
// the one before the proof and, on return, after it; c.chal / c.n_chal every challenge in draw order; c.inv2 and
// c.inv6 are 1/2 and 1/6 (checked here).
template <class C>
VF_HD int aggregate(C& c, const uint8_t* proof, size_t len) {
    Reader r = {proof, len, 0, false};
    c.n_chal = 0;
    c.overflow = false;
    {
        const Fr two = fr_add(fr_one(), fr_one());
        const Fr six = fr_add(fr_add(two, two), two);
        if (!fr_eq(mulx(c.inv2, two), fr_one()) || !fr_eq(mulx(c.inv6, six), fr_one())) return 199;
    }
    const uint32_t magic = rd_u32(r), L = rd_u32(r), B = rd_u32(r), width = rd_u32(r), T = rd_u32(r), Q = rd_u32(r), R = rd_u32(r);
    const uint32_t pad = rd_u32(r);
    if (r.bad) return 100;
    if (magic == ZKGA_MAGIC) {   // "ZKGA", log2 N, log2 D1, log2 D3, log2 D2, 0, 0, 0
        if (Q != 0 || R != 0 || pad != 0) return 100;
        const int rc = matmul_general(c, r, L, B, width, T);
        if (rc) return rc;
        return r.at == len ? 0 : 103;
    }
    if (magic == ZKUP_MAGIC) {   // "ZKUP", log2 D, Q, R, 0, 0, 0, 0
        if (T != 0 || Q != 0 || R != 0 || pad != 0) return 100;
        const int rc = update(c, r, L, B, width);
        if (rc) return rc;
        return r.at == len ? 0 : 103;
    }
    if (pad != 0 || (magic != ZKAG_MAGIC && magic != ZKAF_MAGIC && magic != ZKAL_MAGIC)) return 100;
    if (ilog2(L) < 0 || ilog2(B) < 0 || ilog2(width) < 0 || ilog2(T) < 0) return 101;
    if (magic == ZKAL_MAGIC) {
        const int rc = aggregate_linked(c, r, L, B, width, T, Q, R);
        if (rc) return rc;
        return r.at == len ? 0 : 103;
    }
    const bool ft = magic == ZKAF_MAGIC;
    const uint32_t words[6] = {L, B, width, T, Q, R};
    if (ft) c.absorb_words("aggregate_ft", 12, words, 6);
    else c.absorb_words("aggregate", 9, words, 6);
    const uint64_t n = (uint64_t)L * T;
    const uint64_t dims[3][3] = {{B, width, width}, {B, width, width}, {width, B, width}};
    for (int fam = 0; fam < 3; ++fam) {
        const int rc = ft ? matmul_ft(c, r, n, dims[fam][0], dims[fam][1], dims[fam][2])
                          : matmul(c, r, n, dims[fam][0], dims[fam][1], dims[fam][2]);
        if (rc) return 100 * (2 + fam) + rc;
    }
    const int rc = zkrelu(c, r, ilog2(n) + ilog2(B) + ilog2(width), Q, R);
    if (rc) return (rc >= 100 ? 600 + rc - 100 : 500 + rc);
    if (r.at != len) return 103;
    return 0;
}

// 1/2 and 1/6 by Fermat (the host side; the device takes them from the context's constants)
inline void host_inverses(Fr& inv2, Fr& inv6) {
    uint32_t e[8];
    for (int i = 0; i < 8; ++i) e[i] = frc::MOD[i];
    e[0] = 0xffffffffu;   // r - 2: r[0] = 1 borrows from the next limb, which is 0xffffffff
    e[1] -= 1u;
    const Fr two = fr_add(fr_one(), fr_one());
    const Fr six = fr_add(fr_add(two, two), two);
    inv2 = fr_pow(two, e);
    inv6 = fr_pow(six, e);
}

}  // namespace vf
