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

VF_NI void absorb_bytes(ts::State& s, const char* label, uint32_t label_len, const uint8_t* data, uint64_t n) {
    ts::absorb(s, label, label_len, data, n);
}

// lanes that run the program side by side (the device runs one wave, every lane the same program; a draw of
// several challenges is shared out among them)
VF_HD int lane_id() {
#if defined(__HIP_DEVICE_COMPILE__)
    return (int)threadIdx.x;
#else
    return 0;
#endif
}
VF_HD int lane_count() {
#if defined(__HIP_DEVICE_COMPILE__)
    return (int)blockDim.x;
#else
    return 1;
#endif
}
VF_HD void lanes_sync() {
#if defined(__HIP_DEVICE_COMPILE__)
    __threadfence_block();
    __syncthreads();
#endif
}

constexpr uint32_t SC_MAGIC = 0x43534B5Au, ZKAG_MAGIC = 0x47414B5Au, ZKAF_MAGIC = 0x46414B5Au, ZKRL_MAGIC = 0x4C524B5Au,
                   FT_MAGIC = 0x46534B5Au;
constexpr int MAX_CHAL = 1024;

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
    return (uint32_t)q[0] | ((uint32_t)q[1] << 8) | ((uint32_t)q[2] << 16) | ((uint32_t)q[3] << 24);
}

// a field element of the proof: 32 canonical little-endian bytes; Montgomery form out, the bytes' position in *src
VF_NI Fr rd_fr(Reader& r, const uint8_t** src) {
    Fr x = fr_zero();
    if (r.at + 32 > r.len) {
        r.bad = true;
        return x;
    }
    const uint8_t* q = r.p + r.at;
    if (src) *src = q;
    r.at += 32;
    for (int l = 0; l < 8; ++l)
        x.v[l] = (uint32_t)q[4 * l] | ((uint32_t)q[4 * l + 1] << 8) | ((uint32_t)q[4 * l + 2] << 16) | ((uint32_t)q[4 * l + 3] << 24);
    bool below = false, above = false;   // canonical: below r
    for (int l = 7; l >= 0; --l) {
        if (below || above) break;
        if (x.v[l] > frc::MOD[l]) above = true;
        else if (x.v[l] < frc::MOD[l]) below = true;
    }
    if (!below) r.bad = true;
    return fr_to_mont(x);
}

struct Ctx {
    ts::State& s;   // the transcript; on the device it lives in LDS (byte-wise updates of private memory are slow)
    ts::State& tmp; // work copy for the hashes of a draw, in the same kind of memory
    Fr* chal;       // room for MAX_CHAL challenges (Montgomery form)
    int n_chal;
    Fr inv2, inv6;
    bool overflow;
};

VF_HD void absorb_words(Ctx& c, const char* label, uint32_t label_len, const uint32_t* w, int n) {
    uint8_t b[32];
    for (int i = 0; i < n; ++i)
        for (int k = 0; k < 4; ++k) b[4 * i + k] = (uint8_t)(w[i] >> (8 * k));
    absorb_bytes(c.s, label, label_len, b, 4 * (uint64_t)n);
}

// element idx of a draw, hashed in the context's work copy of the transcript
VF_NI Fr challenge_elem(Ctx& c, uint32_t idx) {
    uint32_t d[2][8];
    for (uint32_t j = 0; j < 2; ++j) {
        c.tmp = c.s;
        ts::State& f = c.tmp;
        const uint64_t bits = (c.s.nblk * 64 + c.s.fill + 5) * 8;
        ts::push_byte(f, (uint8_t)(0xF0 + j));
        for (int k = 0; k < 4; ++k) ts::push_byte(f, (uint8_t)(idx >> (8 * k)));
        ts::push_byte(f, 0x80);
        while (f.fill != 56) ts::push_byte(f, 0);
        for (int i = 7; i >= 0; --i) ts::push_byte(f, (uint8_t)(bits >> (8 * i)));
        for (int i = 0; i < 8; ++i) d[j][i] = f.h[i];
    }
    Fr lo, hi;
    for (int l = 0; l < 8; ++l) {
        lo.v[l] = sha::bswap32(d[0][l]);
        hi.v[l] = sha::bswap32(d[1][l]);
    }
    return fr_add(mulx(fr_const(frc::R2), lo), mulx(fr_const(frc::W3), hi));   // lo + 2^256 hi mod r
}

// one draw of n challenges, appended to c.chal; returns the index of the first
VF_NI int draw(Ctx& c, int n) {
    const int base = c.n_chal;
    if (base + n > MAX_CHAL) {
        c.overflow = true;
        return 0;
    }
    if (lane_count() == 1) {
        for (int i = 0; i < n; ++i) c.chal[base + i] = challenge_elem(c, (uint32_t)i);
    } else if (n == 1) {
        c.chal[base] = challenge_elem(c, 0);   // every lane the same element, in the shared work copy
    } else {
        // each lane its own elements: the work copy is per lane then (private memory)
        for (int i = lane_id(); i < n; i += lane_count()) c.chal[base + i] = ts::challenge_elem(c.s, (uint32_t)i);
    }
    lanes_sync();   // every lane reads every challenge afterwards
    if (n > 0) ts::ratchet(c.s);
    c.n_chal += n;
    return base;
}

VF_HD int ilog2(uint64_t x) {   // -1 if x is no power of two
    int l = 0;
    if (x == 0) return -1;
    while (((uint64_t)1 << l) < x) ++l;
    return (((uint64_t)1 << l) == x) ? l : -1;
}

// value at v of the polynomial through (k, g[k]), k < npts, npts = 3 or 4
VF_NI Fr lagrange(const Ctx& c, const Fr* g, int npts, const Fr& v) {
    const Fr one = fr_one();
    const Fr v1 = fr_sub(v, one), v2 = fr_sub(v1, one), v3 = fr_sub(v2, one);
    if (npts == 4) {   // g(v) = (v-2)(v-3) [c0 (v-1) + c1 v] + v (v-1) [c2 (v-3) + c3 (v-2)], c = (-g0/6, g1/2, -g2/2, g3/6)
        const Fr c0 = fr_neg(mulx(g[0], c.inv6)), c1 = mulx(g[1], c.inv2), c2 = fr_neg(mulx(g[2], c.inv2)),
                 c3 = mulx(g[3], c.inv6);
        const Fr a = mulx(mulx(v2, v3), fr_add(mulx(c0, v1), mulx(c1, v)));
        const Fr b = mulx(mulx(v, v1), fr_add(mulx(c2, v3), mulx(c3, v2)));
        return fr_add(a, b);
    }
    // g(v) = (v-2) [c0 (v-1) + c1 v] + c2 v (v-1), c = (g0/2, -g1, g2/2)
    const Fr c0 = mulx(g[0], c.inv2), c1 = fr_neg(g[1]), c2 = mulx(g[2], c.inv2);
    return fr_add(mulx(v2, fr_add(mulx(c0, v1), mulx(c1, v))), mulx(c2, mulx(v, v1)));
}

// beta~(u, v) = prod_k (u_k v_k + (1 - u_k)(1 - v_k))
VF_NI Fr beta_point(const Fr* u, const Fr* v, int m) {
    Fr acc = fr_one();
    const Fr one = fr_one();
    for (int k = 0; k < m; ++k)
        acc = mulx(acc, fr_add(mulx(u[k], v[k]), mulx(fr_sub(one, u[k]), fr_sub(one, v[k]))));
    return acc;
}

// The rounds of one SC block: every g_t(0) + g_t(1) against the running claim, the challenges re-derived
// (appended to c.chal).  `claim` holds claim_0 on entry (already checked / absorbed by the caller as the
// protocol says) and the final claim on return.  first_label: 'g' rounds absorb g(0), g(2), .., g(degree).
// Returns 0 or a detail code.
VF_NI int rounds(Ctx& c, Reader& r, int nrounds, int degree, Fr& claim, int* first_chal) {
    *first_chal = c.n_chal;
    for (int t = 0; t < nrounds; ++t) {
        Fr g[4];
        const uint8_t* src[4];
        for (int x = 0; x <= degree; ++x) g[x] = rd_fr(r, &src[x]);
        if (r.bad) return 1;
        if (!fr_eq(fr_add(g[0], g[1]), claim)) return 2;   // Sec. 2.2
        uint8_t msg[96];
        int nm = 0;
        for (int x = 0; x <= degree; ++x) {
            if (x == 1) continue;
            for (int b = 0; b < 32; ++b) msg[32 * nm + b] = src[x][b];
            ++nm;
        }
        absorb_bytes(c.s, "g", 1, msg, 32 * (uint64_t)nm);
        const int ci = draw(c, 1);
        if (c.overflow) return 3;
        claim = lagrange(c, g, degree + 1, c.chal[ci]);
    }
    return 0;
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
VF_NI int matmul(Ctx& c, Reader& r, uint64_t n, uint64_t d1, uint64_t d2, uint64_t d3) {
    const int ln = ilog2(n), l1 = ilog2(d1), l2 = ilog2(d2), l3 = ilog2(d3);
    ScHeader h;
    if (!rd_sc_header(r, h) || h.n_finals != 3 || h.degree != 3 || (int)h.rounds != ln + l2) return 10;
    const uint32_t words[4] = {(uint32_t)n, (uint32_t)d1, (uint32_t)d2, (uint32_t)d3};
    absorb_words(c, "sumcheck_matmul", 15, words, 4);
    const int cw = draw(c, ln + l1 + l3);
    const uint8_t* src;
    Fr claim = rd_fr(r, &src);
    if (r.bad || c.overflow) return 11;
    absorb_bytes(c.s, "c", 1, src, 32);
    int cv;
    const int rc = rounds(c, r, ln + l2, 3, claim, &cv);
    if (rc) return 20 + rc;
    const uint8_t* fsrc;
    const Fr fb = rd_fr(r, &fsrc), f0 = rd_fr(r, nullptr), f1 = rd_fr(r, nullptr);
    if (r.bad) return 12;
    absorb_bytes(c.s, "f", 1, fsrc, 96);
    if (!fr_eq(fb, beta_point(c.chal + cw, c.chal + cv, ln))) return 13;
    if (!fr_eq(mulx(mulx(fb, f0), f1), claim)) return 14;
    return 0;
}

// The optimized aggregated protocol (App. B): stack rounds with f_t, (1 - w_t) f_t(0) + w_t f_t(1) = claim,
// then the single product's sumcheck (K = 2), whose claim_0 must be f_{n-1}(v_{n-1}).
VF_NI int matmul_ft(Ctx& c, Reader& r, uint64_t n, uint64_t d1, uint64_t d2, uint64_t d3) {
    const int ln = ilog2(n), l1 = ilog2(d1), l2 = ilog2(d2), l3 = ilog2(d3);
    const uint32_t magic = rd_u32(r), pln = rd_u32(r), pl2 = rd_u32(r), zero = rd_u32(r);
    if (r.bad || magic != FT_MAGIC || (int)pln != ln || (int)pl2 != l2 || zero != 0) return 10;
    const uint32_t words[4] = {(uint32_t)n, (uint32_t)d1, (uint32_t)d2, (uint32_t)d3};
    absorb_words(c, "sumcheck_matmul_ft", 18, words, 4);
    const int cw = draw(c, ln + l1 + l3);
    const uint8_t* src;
    Fr claim = rd_fr(r, &src);
    if (r.bad || c.overflow) return 11;
    absorb_bytes(c.s, "c", 1, src, 32);
    const Fr one = fr_one();
    for (int t = 0; t < ln; ++t) {
        Fr f[3];
        const uint8_t* fs;
        f[0] = rd_fr(r, &fs);
        f[1] = rd_fr(r, nullptr);
        f[2] = rd_fr(r, nullptr);
        if (r.bad) return 15;
        const Fr wt = c.chal[cw + t];
        if (!fr_eq(fr_add(mulx(fr_sub(one, wt), f[0]), mulx(wt, f[1])), claim)) return 16;
        absorb_bytes(c.s, "f", 1, fs, 96);
        const int ci = draw(c, 1);
        if (c.overflow) return 17;
        claim = lagrange(c, f, 3, c.chal[ci]);
    }
    ScHeader h;
    if (!rd_sc_header(r, h) || h.n_finals != 2 || h.degree != 2 || (int)h.rounds != l2) return 18;
    Fr inner0 = rd_fr(r, nullptr);
    if (r.bad || !fr_eq(inner0, claim)) return 19;
    int cv;
    const int rc = rounds(c, r, l2, 2, claim, &cv);
    if (rc) return 20 + rc;
    const uint8_t* fsrc;
    const Fr f0 = rd_fr(r, &fsrc), f1 = rd_fr(r, nullptr);
    if (r.bad) return 12;
    absorb_bytes(c.s, "f", 1, fsrc, 64);
    if (!fr_eq(mulx(f0, f1), claim)) return 14;
    return 0;
}

// multilinear extension of a table of J = 2^lj signed integers at wbar: sum_j tab[j] beta~(wbar, j)
VF_NI Fr mle_small(const Fr* tab, int lj, const Fr* wbar) {
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

// zkReLU with all five points drawn (App. A and the merge of the three claims on aux)
VF_NI int zkrelu(Ctx& c, Reader& r, int li_expect, uint32_t q_expect, uint32_t r_expect) {
    const uint32_t magic = rd_u32(r), pli = rd_u32(r), q = rd_u32(r), rb = rd_u32(r), has_ga = rd_u32(r), mode = rd_u32(r);
    const uint32_t pad0 = rd_u32(r), pad1 = rd_u32(r);
    if (r.bad || pad0 != 0 || pad1 != 0 || magic != ZKRL_MAGIC || (int)pli != li_expect || q != q_expect || rb != r_expect || mode != 0 || has_ga > 1)
        return 1;
    const int li = (int)pli, b = (int)(q + rb);
    if (b < 2 || b > 64 || rb < 1) return 1;
    int lj = 0;
    while ((1 << lj) < b) ++lj;
    const int J = 1 << lj;
    const uint8_t* csrc;
    Fr c_in[4];
    c_in[0] = rd_fr(r, &csrc);
    for (int k = 1; k < 4; ++k) c_in[k] = rd_fr(r, nullptr);
    ScHeader h, hm;
    if (!rd_sc_header(r, h) || h.n_finals != 3 || h.degree != 3 || (int)h.rounds != li + lj) return 2;
    const uint32_t words[4] = {pli, q, rb, has_ga};
    absorb_words(c, "zkrelu", 6, words, 4);
    const int cu = draw(c, 5 * li + lj);   // u_Z, u_A, u_GA, u_GZ (li each), u_bin (li + lj)
    absorb_bytes(c.s, "c", 1, csrc, 128);
    const int cr = draw(c, 2);
    if (c.overflow) return 3;
    const Fr rr = c.chal[cr], rp = c.chal[cr + 1], r2 = mulx(rr, rr);
    const Fr w_z = r2, w_a = rr, w_ga = mulx(rp, r2), w_gz = mulx(rp, rr);
    Fr claim = rd_fr(r, nullptr);
    const Fr expect0 = fr_add(fr_add(mulx(w_z, c_in[0]), mulx(w_a, c_in[1])), fr_add(mulx(w_ga, c_in[2]), mulx(w_gz, c_in[3])));
    if (r.bad || !fr_eq(claim, expect0)) return 4;   // the combined claim is the weighted sum of the input claims
    int cv;
    int rc = rounds(c, r, li + lj, 3, claim, &cv);
    if (rc) return 10 + rc;
    const uint8_t* fsrc;
    const Fr a0 = rd_fr(r, &fsrc), a1 = rd_fr(r, nullptr), sg = rd_fr(r, nullptr);
    if (r.bad) return 5;
    absorb_bytes(c.s, "f", 1, fsrc, 96);
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
    const Fr s_w = mle_small(s_tab, lj, wbar), sp_w = mle_small(sp_tab, lj, wbar);
    const Fr b_bin = beta_point(c.chal + cu + 4 * li, c.chal + cv, li + lj);
    const Fr one = fr_one();
    const Fr ns = fr_sub(one, sg);
    auto side = [&](const Fr& a, const Fr& w_in, const Fr& w_out, const Fr* u_in, const Fr* u_out) {
        Fr t = mulx(mulx(mulx(w_in, beta_point(u_in, v_i, li)), a), s_w);
        t = fr_add(t, mulx(mulx(mulx(mulx(w_out, beta_point(u_out, v_i, li)), ns), a), sp_w));
        return fr_add(t, mulx(b_bin, fr_sub(mulx(a, a), a)));
    };
    const Fr fwd = side(a0, w_z, w_a, c.chal + cu, c.chal + cu + li);
    Fr bwd = mulx(mulx(mulx(w_ga, beta_point(c.chal + cu + 2 * li, v_i, li)), a1), s_w);
    bwd = fr_add(bwd, mulx(mulx(mulx(mulx(w_gz, beta_point(c.chal + cu + 3 * li, v_i, li)), ns), a1), sp_w));
    bwd = fr_add(bwd, mulx(mulx(rp, b_bin), fr_sub(mulx(a1, a1), a1)));
    if (!fr_eq(fr_add(fwd, bwd), claim)) return 6;   // App. A: the six equations at the challenge point
    // merge of the three claims on aux (degree 2 over 1 + lj variables)
    if (!rd_sc_header(r, hm) || hm.n_finals != 2 || hm.degree != 2 || (int)hm.rounds != 1 + lj) return 7;
    const int crho = draw(c, 3);
    if (c.overflow) return 3;
    Fr mclaim = rd_fr(r, nullptr);
    const Fr em = fr_add(fr_add(mulx(c.chal[crho], a0), mulx(c.chal[crho + 1], a1)), mulx(c.chal[crho + 2], sg));
    if (r.bad || !fr_eq(mclaim, em)) return 8;
    int cm;
    rc = rounds(c, r, 1 + lj, 2, mclaim, &cm);
    if (rc) return 100 + rc;
    const uint8_t* msrc;
    const Fr m_f = rd_fr(r, &msrc), e_f = rd_fr(r, nullptr);
    if (r.bad) return 5;
    absorb_bytes(c.s, "f", 1, msrc, 64);
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
    const Fr e_pub = fr_add(fr_add(mulx(c.chal[crho], beta_point(p0, vm, 1 + lj)), mulx(c.chal[crho + 1], beta_point(p1, vm, 1 + lj))),
                            mulx(c.chal[crho + 2], beta_point(p2, vm, 1 + lj)));
    if (!fr_eq(e_f, e_pub)) return 101;
    if (!fr_eq(mulx(m_f, e_f), mclaim)) return 102;
    return 0;
}

// The whole window ("ZKAG": g_t form; "ZKAF": f_t form for the matrix products).  c.s is the transcript before
// the proof and after it on return; c.chal / c.n_chal every challenge in draw order.
VF_HD int aggregate(Ctx& c, const uint8_t* proof, size_t len) {
    Reader r = {proof, len, 0, false};
    c.n_chal = 0;
    c.overflow = false;
    {   // 1/2 and 1/6 by Fermat
        uint32_t e[8];
        for (int i = 0; i < 8; ++i) e[i] = frc::MOD[i];
        e[0] = 0xffffffffu;   // r - 2: r[0] = 1 borrows from the next limb, which is 0xffffffff
        e[1] -= 1u;
        const Fr two = fr_add(fr_one(), fr_one());
        const Fr six = fr_add(fr_add(two, two), two);
        c.inv2 = fr_pow(two, e);
        c.inv6 = fr_pow(six, e);
        if (!fr_eq(mulx(c.inv2, two), fr_one()) || !fr_eq(mulx(c.inv6, six), fr_one())) return 199;
    }
    const uint32_t magic = rd_u32(r), L = rd_u32(r), B = rd_u32(r), width = rd_u32(r), T = rd_u32(r), Q = rd_u32(r), R = rd_u32(r);
    const uint32_t pad = rd_u32(r);
    if (r.bad || pad != 0 || (magic != ZKAG_MAGIC && magic != ZKAF_MAGIC)) return 100;
    if (ilog2(L) < 0 || ilog2(B) < 0 || ilog2(width) < 0 || ilog2(T) < 0) return 101;
    const bool ft = magic == ZKAF_MAGIC;
    const uint32_t words[6] = {L, B, width, T, Q, R};
    if (ft) absorb_words(c, "aggregate_ft", 12, words, 6);
    else absorb_words(c, "aggregate", 9, words, 6);
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

}  // namespace vf
