/* zkdl_oracle.c - second tier of the CPU oracle, in plain C, for inputs too large for the
 * Python-integer tier: the product sumcheck and the multilinear-extension partial evaluation
 * (the 2^24-entry kernel micro-benchmark) and, in the second part of this file, the provers of
 * the matrix product, the Hadamard product, zkReLU, re-indexing, the merge of claims and the
 * aggregated window (the width-1024 and width-4096 networks).
 *
 * Test infrastructure: used by tests, the smoke check and the benchmark's CPU baseline only,
 * never by the product.  It shares no code with the HIP library: field elements are canonical
 * (no Montgomery form) in four 64-bit limbs, products are schoolbook 4 x 4 with unsigned
 * __int128 and reduced with Barrett's method as in the Handbook of Applied Cryptography,
 * Alg. 14.42 (b = 2^64, k = 4; q3 m is taken mod b^(k+1) as step 2 of the algorithm states, and the
 * at most two closing subtractions are selected with masks), SHA-256 is written from FIPS 180-4.
 * It is pinned byte for byte against the Python tier on small inputs (tests/test_oracle_c.py).
 *
 * What is computed, in the paper's terms:
 *  - beta~(u, b) = prod_k (u_k b_k + (1 - u_k)(1 - b_k)), coordinate 0 = most significant bit
 *    of b (Sec. 2.2: the multilinear extension of the equality indicator);
 *  - partial evaluation out[o, i] = sum_a beta~(u, a) T[o, a, i] (Eq. multilinear-extension
 *    applied to one axis);
 *  - the sumcheck prover for sum_b prod_k T_k[b] (Sec. 2.2): per round the evaluations
 *    g_t(0..K), a challenge, the fold T'[b] = T[b] + v (T[b + half] - T[b]);
 *  - the Fiat-Shamir transcript in this build's own byte format (the protocols of App. B are
 *    interactive): see transcript_* below.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef unsigned __int128 u128;

typedef struct {
    uint64_t l[4]; /* value < r, little-endian limbs */
} fe;

/* r = 0x73eda753299d7d483339d80809a1d80553bda402fffe5bfeffffffff00000001 (Sec. 6: BLS12-381 scalar field) */
static const uint64_t MOD[4] = {0xffffffff00000001ULL, 0x53bda402fffe5bfeULL, 0x3339d80809a1d805ULL,
                                0x73eda753299d7d48ULL};
static uint64_t MU[5]; /* floor(2^512 / r) */
static int mu_ready = 0;

/* ---- multi-limb helpers: n limbs, little-endian ---- */
static int mp_cmp(const uint64_t* a, const uint64_t* b, int n) {
    for (int i = n - 1; i >= 0; --i) {
        if (a[i] < b[i]) return -1;
        if (a[i] > b[i]) return 1;
    }
    return 0;
}

static uint64_t mp_sub(uint64_t* a, const uint64_t* b, int n) { /* a -= b, returns borrow */
    uint64_t borrow = 0;
    for (int i = 0; i < n; ++i) {
        u128 d = (u128)a[i] - b[i] - borrow;
        a[i] = (uint64_t)d;
        borrow = (uint64_t)(d >> 64) & 1;
    }
    return borrow;
}

/* floor(2^512 / r) by binary long division */
static void init_mu(void) {
    if (mu_ready) return;
    uint64_t rem[5] = {0, 0, 0, 0, 0}, m5[5] = {MOD[0], MOD[1], MOD[2], MOD[3], 0};
    uint64_t q[9];
    memset(q, 0, sizeof q);
    for (int bit = 512; bit >= 0; --bit) {
        /* rem = 2 rem + bit of 2^512 */
        for (int i = 4; i > 0; --i) rem[i] = (rem[i] << 1) | (rem[i - 1] >> 63);
        rem[0] = (rem[0] << 1) | (bit == 512 ? 1u : 0u);
        if (mp_cmp(rem, m5, 5) >= 0) {
            mp_sub(rem, m5, 5);
            q[bit / 64] |= (uint64_t)1 << (bit % 64);
        }
    }
    for (int i = 0; i < 5; ++i) MU[i] = q[i];
    mu_ready = 1;
}

/* Fixed-size forms of the helpers above for the three calls that carry the run time (plain loops
 * with constant bounds, so that the compiler unrolls them; same arithmetic). */
static inline uint64_t sub_n(uint64_t* a, const uint64_t* b, const int n) { /* a -= b, returns borrow */
    uint64_t borrow = 0;
    for (int i = 0; i < n; ++i) {
        u128 d = (u128)a[i] - b[i] - borrow;
        a[i] = (uint64_t)d;
        borrow = (uint64_t)(d >> 64) & 1;
    }
    return borrow;
}

/* low `keep` limbs of the product of two 5-limb numbers; keep = 10 gives the whole product */
static inline void mul5_low(const uint64_t* a, const uint64_t* b, uint64_t* out, const int keep) {
    for (int i = 0; i < keep; ++i) out[i] = 0;
    for (int i = 0; i < 5; ++i) {
        uint64_t carry = 0;
        for (int j = 0; j < 5 && i + j < keep; ++j) {
            u128 t = (u128)a[i] * b[j] + out[i + j] + carry;
            out[i + j] = (uint64_t)t;
            carry = (uint64_t)(t >> 64);
        }
        if (i + 5 < keep) out[i + 5] = carry;
    }
}

/* x (8 limbs, any value below 2^512) mod r: HAC Alg. 14.42 with b = 2^64, k = 4 */
static fe reduce512(const uint64_t x[8]) {
    uint64_t q2[10], r2[5], r1[5];
    mul5_low(x + 3, MU, q2, 10);        /* q1 = floor(x / b^(k-1)); q2 = q1 mu */
    const uint64_t* q3 = q2 + 5;        /* q3 = floor(q2 / b^(k+1)) */
    const uint64_t m5[5] = {MOD[0], MOD[1], MOD[2], MOD[3], 0};
    mul5_low(q3, m5, r2, 5);            /* r2 = q3 m mod b^(k+1) */
    for (int i = 0; i < 5; ++i) r1[i] = x[i];
    sub_n(r1, r2, 5);                   /* r = r1 - r2 mod b^(k+1): the wrap-around is the "+ b^(k+1)" step */
    for (int pass = 0; pass < 2; ++pass) { /* at most two subtractions of r remain (HAC 14.43) */
        uint64_t t[5] = {r1[0], r1[1], r1[2], r1[3], r1[4]};
        const uint64_t keep = (uint64_t)0 - sub_n(t, m5, 5); /* all ones if r1 < r */
        for (int i = 0; i < 5; ++i) r1[i] = (r1[i] & keep) | (t[i] & ~keep);
    }
    fe o = {{r1[0], r1[1], r1[2], r1[3]}};
    return o;
}

static fe fe_mul(fe a, fe b) {
    uint64_t p[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int i = 0; i < 4; ++i) { /* schoolbook 4 x 4 */
        uint64_t carry = 0;
        for (int j = 0; j < 4; ++j) {
            u128 t = (u128)a.l[i] * b.l[j] + p[i + j] + carry;
            p[i + j] = (uint64_t)t;
            carry = (uint64_t)(t >> 64);
        }
        p[i + 4] = carry;
    }
    return reduce512(p);
}

static fe fe_add(fe a, fe b) { /* a + b < 2 r < 2^256: no carry out of the fourth limb */
    uint64_t carry = 0;
    for (int i = 0; i < 4; ++i) {
        u128 s = (u128)a.l[i] + b.l[i] + carry;
        a.l[i] = (uint64_t)s;
        carry = (uint64_t)(s >> 64);
    }
    fe t = a;
    const uint64_t keep = (uint64_t)0 - sub_n(t.l, MOD, 4); /* all ones if a + b < r (selected without a branch) */
    for (int i = 0; i < 4; ++i) a.l[i] = (a.l[i] & keep) | (t.l[i] & ~keep);
    return a;
}

static fe fe_sub(fe a, fe b) {
    const uint64_t below = (uint64_t)0 - sub_n(a.l, b.l, 4); /* all ones if a < b: add r back */
    uint64_t carry = 0;
    for (int i = 0; i < 4; ++i) {
        u128 s = (u128)a.l[i] + (MOD[i] & below) + carry;
        a.l[i] = (uint64_t)s;
        carry = (uint64_t)(s >> 64);
    }
    return a;
}

static fe fe_zero(void) {
    fe z = {{0, 0, 0, 0}};
    return z;
}

static fe fe_one(void) {
    fe o = {{1, 0, 0, 0}};
    return o;
}

static fe fe_load(const uint8_t* p) { /* 32 canonical little-endian bytes */
    fe a;
    for (int i = 0; i < 4; ++i) {
        uint64_t w = 0;
        for (int b = 7; b >= 0; --b) w = (w << 8) | p[8 * i + b];
        a.l[i] = w;
    }
    return a;
}

static void fe_store(fe a, uint8_t* p) {
    for (int i = 0; i < 4; ++i)
        for (int b = 0; b < 8; ++b) p[8 * i + b] = (uint8_t)(a.l[i] >> (8 * b));
}

/* ---- SHA-256, FIPS 180-4 ---- */
typedef struct {
    uint32_t h[8];
    uint8_t buf[64];
    uint32_t fill;
    uint64_t len; /* bytes absorbed */
} sha_ctx;

static uint32_t rotr32(uint32_t x, int n) { return (x >> n) | (x << (32 - n)); }

static const uint32_t SHA_K[64] = {
    0x428a2f98, 0x71374491, 0xb5c0fbcf, 0xe9b5dba5, 0x3956c25b, 0x59f111f1, 0x923f82a4, 0xab1c5ed5, 0xd807aa98,
    0x12835b01, 0x243185be, 0x550c7dc3, 0x72be5d74, 0x80deb1fe, 0x9bdc06a7, 0xc19bf174, 0xe49b69c1, 0xefbe4786,
    0x0fc19dc6, 0x240ca1cc, 0x2de92c6f, 0x4a7484aa, 0x5cb0a9dc, 0x76f988da, 0x983e5152, 0xa831c66d, 0xb00327c8,
    0xbf597fc7, 0xc6e00bf3, 0xd5a79147, 0x06ca6351, 0x14292967, 0x27b70a85, 0x2e1b2138, 0x4d2c6dfc, 0x53380d13,
    0x650a7354, 0x766a0abb, 0x81c2c92e, 0x92722c85, 0xa2bfe8a1, 0xa81a664b, 0xc24b8b70, 0xc76c51a3, 0xd192e819,
    0xd6990624, 0xf40e3585, 0x106aa070, 0x19a4c116, 0x1e376c08, 0x2748774c, 0x34b0bcb5, 0x391c0cb3, 0x4ed8aa4a,
    0x5b9cca4f, 0x682e6ff3, 0x748f82ee, 0x78a5636f, 0x84c87814, 0x8cc70208, 0x90befffa, 0xa4506ceb, 0xbef9a3f7,
    0xc67178f2};

static void sha_block(uint32_t h[8], const uint8_t* p) {
    uint32_t w[64];
    for (int t = 0; t < 16; ++t)
        w[t] = ((uint32_t)p[4 * t] << 24) | ((uint32_t)p[4 * t + 1] << 16) | ((uint32_t)p[4 * t + 2] << 8) | p[4 * t + 3];
    for (int t = 16; t < 64; ++t) {
        uint32_t s0 = rotr32(w[t - 15], 7) ^ rotr32(w[t - 15], 18) ^ (w[t - 15] >> 3);
        uint32_t s1 = rotr32(w[t - 2], 17) ^ rotr32(w[t - 2], 19) ^ (w[t - 2] >> 10);
        w[t] = w[t - 16] + s0 + w[t - 7] + s1;
    }
    uint32_t a = h[0], b = h[1], c = h[2], d = h[3], e = h[4], f = h[5], g = h[6], hh = h[7];
    for (int t = 0; t < 64; ++t) {
        uint32_t t1 = hh + (rotr32(e, 6) ^ rotr32(e, 11) ^ rotr32(e, 25)) + ((e & f) ^ (~e & g)) + SHA_K[t] + w[t];
        uint32_t t2 = (rotr32(a, 2) ^ rotr32(a, 13) ^ rotr32(a, 22)) + ((a & b) ^ (a & c) ^ (b & c));
        hh = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + t2;
    }
    h[0] += a; h[1] += b; h[2] += c; h[3] += d; h[4] += e; h[5] += f; h[6] += g; h[7] += hh;
}

static void sha_init(sha_ctx* c) {
    static const uint32_t iv[8] = {0x6a09e667, 0xbb67ae85, 0x3c6ef372, 0xa54ff53a,
                                   0x510e527f, 0x9b05688c, 0x1f83d9ab, 0x5be0cd19};
    memcpy(c->h, iv, sizeof iv);
    c->fill = 0;
    c->len = 0;
}

static void sha_update(sha_ctx* c, const uint8_t* p, size_t n) {
    for (size_t i = 0; i < n; ++i) {
        c->buf[c->fill++] = p[i];
        if (c->fill == 64) {
            sha_block(c->h, c->buf);
            c->fill = 0;
        }
    }
    c->len += n;
}

static void sha_final(const sha_ctx* c0, uint8_t out[32]) { /* does not change c0 */
    sha_ctx c = *c0;
    uint64_t bits = c.len * 8;
    uint8_t pad = 0x80, zero = 0;
    sha_update(&c, &pad, 1);
    while (c.fill != 56) sha_update(&c, &zero, 1);
    uint8_t lenb[8];
    for (int i = 0; i < 8; ++i) lenb[i] = (uint8_t)(bits >> (8 * (7 - i)));
    sha_update(&c, lenb, 8);
    for (int i = 0; i < 8; ++i) {
        out[4 * i] = (uint8_t)(c.h[i] >> 24);
        out[4 * i + 1] = (uint8_t)(c.h[i] >> 16);
        out[4 * i + 2] = (uint8_t)(c.h[i] >> 8);
        out[4 * i + 3] = (uint8_t)c.h[i];
    }
}

/* ---- transcript: one byte stream; every value is a SHA-256 of an extension of it ----
 *   stream_0         = "zkdl-mi355x/v3" zero-padded to 56 bytes || u64le(seed)
 *   absorb(label, m) : stream <- stream || u8(|label|) || label || u64le(|m|) || m
 *   challenge()      : c = int_le(SHA256(stream || 0xF0 || u32le(0)) || SHA256(stream || 0xF1 || u32le(0))) mod r,
 *                      then stream <- stream || 0xF2 || zeros up to the next multiple of 64 */
static void transcript_init(sha_ctx* t, uint64_t seed) {
    static const char dom[] = "zkdl-mi355x/v3";
    uint8_t blk[64];
    memset(blk, 0, sizeof blk);
    memcpy(blk, dom, sizeof dom - 1);
    for (int i = 0; i < 8; ++i) blk[56 + i] = (uint8_t)(seed >> (8 * i));
    sha_init(t);
    sha_update(t, blk, 64);
}

static void transcript_absorb(sha_ctx* t, const char* label, const uint8_t* data, uint64_t n) {
    uint8_t ll = (uint8_t)strlen(label), lenb[8];
    sha_update(t, &ll, 1);
    sha_update(t, (const uint8_t*)label, ll);
    for (int i = 0; i < 8; ++i) lenb[i] = (uint8_t)(n >> (8 * i));
    sha_update(t, lenb, 8);
    sha_update(t, data, n);
}

static fe transcript_challenge(sha_ctx* t) {
    uint8_t wide[64];
    for (int j = 0; j < 2; ++j) {
        sha_ctx f = *t;
        uint8_t tail[5] = {(uint8_t)(0xF0 + j), 0, 0, 0, 0};
        sha_update(&f, tail, 5);
        sha_final(&f, wide + 32 * j);
    }
    uint64_t x[8];
    for (int i = 0; i < 8; ++i) {
        uint64_t w = 0;
        for (int b = 7; b >= 0; --b) w = (w << 8) | wide[8 * i + b];
        x[i] = w;
    }
    fe c = reduce512(x);
    uint8_t tag = 0xF2, zero = 0;
    sha_update(t, &tag, 1);
    while (t->fill != 0) sha_update(t, &zero, 1);
    return c;
}

/* ---- exported ---- */
int zko_fe_mul(const uint8_t a[32], const uint8_t b[32], uint8_t out[32]) {
    init_mu();
    fe_store(fe_mul(fe_load(a), fe_load(b)), out);
    return 0;
}

int zko_fe_add(const uint8_t a[32], const uint8_t b[32], uint8_t out[32]) {
    fe_store(fe_add(fe_load(a), fe_load(b)), out);
    return 0;
}

int zko_fe_sub(const uint8_t a[32], const uint8_t b[32], uint8_t out[32]) {
    fe_store(fe_sub(fe_load(a), fe_load(b)), out);
    return 0;
}

int zko_sha256(const uint8_t* data, uint64_t n, uint8_t out[32]) {
    sha_ctx c;
    sha_init(&c);
    sha_update(&c, data, n);
    sha_final(&c, out);
    return 0;
}

/* out[o, i] = sum_a beta~(u, a) T[o, a, i]; src: O*A*I elements of 32 bytes, point: log2(A) elements,
 * out: O*I elements.  A must be a power of two. */
int zko_partial_eval(const uint8_t* src, uint64_t O, uint64_t A, uint64_t I, const uint8_t* point, uint8_t* out) {
    init_mu();
    int la = 0;
    while (((uint64_t)1 << la) < A) ++la;
    if (((uint64_t)1 << la) != A) return -1;
    fe* beta = (fe*)malloc(sizeof(fe) * A);
    if (!beta) return -2;
    for (uint64_t a = 0; a < A; ++a) {
        fe w = fe_one();
        for (int k = 0; k < la; ++k) {
            fe u = fe_load(point + 32 * k);
            int bit = (int)((a >> (la - 1 - k)) & 1); /* coordinate 0 = most significant bit */
            w = fe_mul(w, bit ? u : fe_sub(fe_one(), u));
        }
        beta[a] = w;
    }
#pragma omp parallel for collapse(2) schedule(static)
    for (uint64_t o = 0; o < O; ++o) {
        for (uint64_t i = 0; i < I; ++i) {
            fe acc = fe_zero();
            for (uint64_t a = 0; a < A; ++a)
                acc = fe_add(acc, fe_mul(beta[a], fe_load(src + 32 * ((o * A + a) * I + i))));
            fe_store(acc, out + 32 * (o * I + i));
        }
    }
    free(beta);
    return 0;
}

/* Product sumcheck over K tables of n = 2^d elements (32 canonical bytes each), transcript
 * seeded with `seed` and started with the header "sumcheck_product" (K, d).
 * proof: "ZKSC", u32 n_finals = K, u32 degree = K, u32 rounds = d, claim_0, d x (K+1) evaluations,
 * K finals (capacity 16 + 32 (1 + d (K+1) + K) bytes).  chal_out: d elements.  digest: SHA-256 of the stream. */
int zko_product_prove(const uint8_t* const* tables, int K, uint64_t n, uint64_t seed, uint8_t* proof,
                      uint8_t* chal_out, uint8_t digest[32]) {
    init_mu();
    if (K < 1 || K > 3) return -1;
    int d = 0;
    while (((uint64_t)1 << d) < n) ++d;
    if (((uint64_t)1 << d) != n) return -1;
    fe* T[3] = {0, 0, 0};
    for (int k = 0; k < K; ++k) {
        T[k] = (fe*)malloc(sizeof(fe) * n);
        if (!T[k]) return -2;
#pragma omp parallel for schedule(static)
        for (uint64_t b = 0; b < n; ++b) T[k][b] = fe_load(tables[k] + 32 * b);
    }
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
    fe* part = (fe*)malloc(sizeof(fe) * (size_t)nthreads * 4);

    sha_ctx ts;
    transcript_init(&ts, seed);
    uint8_t hdr[8];
    uint32_t hw[2] = {(uint32_t)K, (uint32_t)d};
    for (int i = 0; i < 2; ++i)
        for (int b = 0; b < 4; ++b) hdr[4 * i + b] = (uint8_t)(hw[i] >> (8 * b));
    transcript_absorb(&ts, "sumcheck_product", hdr, 8);

    /* claim_0 = sum over the hypercube of the product */
    for (int t = 0; t < nthreads * 4; ++t) part[t] = fe_zero();
#pragma omp parallel
    {
        int me = 0;
#ifdef _OPENMP
        me = omp_get_thread_num();
#endif
        fe acc = fe_zero();
#pragma omp for schedule(static)
        for (uint64_t b = 0; b < n; ++b) {
            fe p = T[0][b];
            for (int k = 1; k < K; ++k) p = fe_mul(p, T[k][b]);
            acc = fe_add(acc, p);
        }
        part[me * 4] = acc;
    }
    fe claim = fe_zero();
    for (int t = 0; t < nthreads; ++t) claim = fe_add(claim, part[t * 4]);

    uint8_t* w = proof;
    const uint32_t head[4] = {0x43534B5Au, (uint32_t)K, (uint32_t)K, (uint32_t)d};
    for (int i = 0; i < 4; ++i)
        for (int b = 0; b < 4; ++b) *w++ = (uint8_t)(head[i] >> (8 * b));
    fe_store(claim, w);
    transcript_absorb(&ts, "c", w, 32);
    w += 32;

    uint64_t len = n;
    for (int round = 0; round < d; ++round) {
        const uint64_t half = len / 2;
        for (int t = 0; t < nthreads * 4; ++t) part[t] = fe_zero();
#pragma omp parallel
        {
            int me = 0;
#ifdef _OPENMP
            me = omp_get_thread_num();
#endif
            fe acc[4] = {fe_zero(), fe_zero(), fe_zero(), fe_zero()};
#pragma omp for schedule(static)
            for (uint64_t b = 0; b < half; ++b) {
                fe e[3], dlt[3];
                for (int k = 0; k < K; ++k) {
                    e[k] = T[k][b];
                    dlt[k] = fe_sub(T[k][b + half], T[k][b]);
                }
                for (int x = 0; x <= K; ++x) { /* e[k] = lo + x (hi - lo) */
                    fe p = e[0];
                    for (int k = 1; k < K; ++k) p = fe_mul(p, e[k]);
                    acc[x] = fe_add(acc[x], p);
                    for (int k = 0; k < K; ++k) e[k] = fe_add(e[k], dlt[k]);
                }
            }
            for (int x = 0; x <= K; ++x) part[me * 4 + x] = acc[x];
        }
        fe g[4];
        for (int x = 0; x <= K; ++x) {
            g[x] = fe_zero();
            for (int t = 0; t < nthreads; ++t) g[x] = fe_add(g[x], part[t * 4 + x]);
        }
        /* round check of Sec. 2.2 */
        if (mp_cmp(fe_add(g[0], g[1]).l, claim.l, 4) != 0) return -3;
        /* the transcript takes g(0), g(2), .., g(K): g(1) is fixed by the check above */
        uint8_t msg[96];
        int nm = 0;
        for (int x = 0; x <= K; ++x) {
            fe_store(g[x], w + 32 * x);
            if (x != 1) fe_store(g[x], msg + 32 * nm++);
        }
        w += 32 * (K + 1);
        transcript_absorb(&ts, "g", msg, 32 * (uint64_t)nm);
        fe v = transcript_challenge(&ts);
        fe_store(v, chal_out + 32 * round);
        /* fold every table; next claim g(v) by Lagrange interpolation on the nodes 0..K:
         * sum_k g(k) prod_{j != k} (v - j) / (k - j) */
#pragma omp parallel for schedule(static)
        for (uint64_t b = 0; b < half; ++b)
            for (int k = 0; k < K; ++k) T[k][b] = fe_add(T[k][b], fe_mul(v, fe_sub(T[k][b + half], T[k][b])));
        {
            fe next = fe_zero();
            for (int k = 0; k <= K; ++k) {
                fe num = g[k];
                int64_t den = 1;
                for (int j = 0; j <= K; ++j) {
                    if (j == k) continue;
                    fe jj = {{(uint64_t)j, 0, 0, 0}};
                    num = fe_mul(num, fe_sub(v, jj));
                    den *= (k - j);
                }
                /* divide by the small integer den = prod_{j != k} (k - j): multiply by its inverse */
                fe dfe;
                if (den > 0) {
                    fe t = {{(uint64_t)den, 0, 0, 0}};
                    dfe = t;
                } else {
                    fe t = {{(uint64_t)(-den), 0, 0, 0}};
                    dfe = fe_sub(fe_zero(), t);
                }
                /* inverse by Fermat: dfe^(r-2) */
                fe inv = fe_one(), base = dfe;
                uint64_t ex[4] = {MOD[0] - 2, MOD[1], MOD[2], MOD[3]};
                for (int bit = 0; bit < 256; ++bit) {
                    if ((ex[bit / 64] >> (bit % 64)) & 1) inv = fe_mul(inv, base);
                    base = fe_mul(base, base);
                }
                next = fe_add(next, fe_mul(num, inv));
            }
            claim = next;
        }
        len = half;
    }
    uint8_t fin[96];
    fe prod = fe_one();
    for (int k = 0; k < K; ++k) {
        fe_store(T[k][0], w + 32 * k);
        fe_store(T[k][0], fin + 32 * k);
        prod = fe_mul(prod, T[k][0]);
    }
    transcript_absorb(&ts, "f", fin, 32 * (uint64_t)K);
    /* the final claim equals the product of the tables' evaluations at the challenge point */
    if (mp_cmp(prod.l, claim.l, 4) != 0) return -4;
    sha_final(&ts, digest);
    for (int k = 0; k < K; ++k) free(T[k]);
    free(part);
    return 0;
}

/* ==========================================================================================
 * Second part: the protocol provers at full size (matrix product, zkReLU, the aggregated
 * window and its linked form), so that the largest configurations have an oracle PROVER and not
 * only a verifier.  Written from the paper and from the Python-integer tier's statement of the
 * same steps (oracle/protocols.py), which stays the parity authority: tests/test_oracle_c.py
 * compares every function below byte for byte with it on small inputs.
 *
 * One difference in bookkeeping, none in arithmetic: a table of the sumcheck that depends on
 * only some of the variables (beta~(w, n) in Eq. exm-matmul-batched does not depend on i; the
 * recomposition vectors of App. A do not depend on the row index) is kept at its own size
 * together with the range [lo, hi) of variables it depends on, and read as T[b] through that
 * range (vt_get) - the same value the Python tier reads from its repeated / tiled copy.
 * Binding a variable outside the range leaves such a table as it is (lo + v (hi - lo), lo = hi).
 * ========================================================================================== */
#include <stdio.h>

#define ZKO_EARG (-1)
#define ZKO_ENOMEM (-2)
#define ZKO_ECHECK (-3)  /* one of the prover's own consistency checks failed */
#define ZKO_ESMALL (-4)  /* output buffer too small */
#define ZKO_ERANGE (-5)  /* a zkReLU input is not a (Q+R)-bit signed integer */

static void (*g_progress)(const char* what, int round, int rounds) = 0;

void zko_set_progress(void (*cb)(const char*, int, int)) { g_progress = cb; }

int zko_set_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}

static int max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int my_thread(void) {
#ifdef _OPENMP
    return omp_get_thread_num();
#else
    return 0;
#endif
}

/* ---- small field helpers ---- */
static fe fe_from_u64(uint64_t x) {
    fe o = {{x, 0, 0, 0}};
    return o;
}

static fe fe_neg(fe a) { return fe_sub(fe_zero(), a); }

static fe fe_from_i64(int64_t x) { /* the signed integer x as x mod r (Sec. 2.2: negatives are r - |x|) */
    if (x >= 0) return fe_from_u64((uint64_t)x);
    return fe_neg(fe_from_u64((uint64_t)0 - (uint64_t)x));
}

static int fe_eq(fe a, fe b) { return mp_cmp(a.l, b.l, 4) == 0; }

static fe fe_inv(fe a) { /* a^(r-2) */
    fe inv = fe_one(), base = a;
    uint64_t ex[4] = {MOD[0] - 2, MOD[1], MOD[2], MOD[3]};
    for (int bit = 0; bit < 256; ++bit) {
        if ((ex[bit / 64] >> (bit % 64)) & 1) inv = fe_mul(inv, base);
        base = fe_mul(base, base);
    }
    return inv;
}

static int ilog2_u64(uint64_t n) { /* -1 if n is no power of two */
    int d = 0;
    if (n == 0) return -1;
    while (((uint64_t)1 << d) < n) ++d;
    return (((uint64_t)1 << d) == n) ? d : -1;
}

/* ---- output buffer ---- */
typedef struct {
    uint8_t* p;
    size_t cap, len;
} wbuf;

static void wb_bytes(wbuf* w, const void* src, size_t n) {
    if (w->len + n <= w->cap) memcpy(w->p + w->len, src, n);
    w->len += n; /* keeps counting: the caller learns the size needed */
}

static void wb_u32(wbuf* w, uint32_t x) {
    uint8_t b[4] = {(uint8_t)x, (uint8_t)(x >> 8), (uint8_t)(x >> 16), (uint8_t)(x >> 24)};
    wb_bytes(w, b, 4);
}

static void wb_fe(wbuf* w, fe a) {
    uint8_t b[32];
    fe_store(a, b);
    wb_bytes(w, b, 32);
}

/* ---- transcript object: the stream plus a record of every challenge drawn ---- */
typedef struct {
    sha_ctx s;
    fe* chal;
    size_t nchal, cap;
} zko_ts;

static int ts_record(zko_ts* t, fe c) {
    if (t->nchal == t->cap) {
        size_t nc = t->cap ? 2 * t->cap : 256;
        fe* p = (fe*)realloc(t->chal, nc * sizeof(fe));
        if (!p) return ZKO_ENOMEM;
        t->chal = p;
        t->cap = nc;
    }
    t->chal[t->nchal++] = c;
    return 0;
}

static void ts_absorb_fe(zko_ts* t, const char* label, const fe* e, int n) {
    uint8_t* buf = (uint8_t*)malloc(32 * (size_t)(n > 0 ? n : 1));
    for (int i = 0; i < n; ++i) fe_store(e[i], buf + 32 * i);
    transcript_absorb(&t->s, label, buf, 32 * (uint64_t)n);
    free(buf);
}

static void ts_absorb_u32(zko_ts* t, const char* label, const uint32_t* w, int n) {
    uint8_t buf[4 * 16];
    for (int i = 0; i < n; ++i)
        for (int b = 0; b < 4; ++b) buf[4 * i + b] = (uint8_t)(w[i] >> (8 * b));
    transcript_absorb(&t->s, label, buf, 4 * (uint64_t)n);
}

/* challenges(n): c_i = int_le(SHA256(stream || 0xF0 || u32le(i)) || SHA256(stream || 0xF1 || u32le(i))) mod r,
 * then stream <- stream || 0xF2 || zeros up to the next multiple of 64; n = 0 does nothing */
static int ts_draw(zko_ts* t, int n, fe* out) {
    for (int i = 0; i < n; ++i) {
        uint8_t wide[64];
        for (int j = 0; j < 2; ++j) {
            sha_ctx f = t->s;
            uint8_t tail[5] = {(uint8_t)(0xF0 + j), (uint8_t)i, (uint8_t)(i >> 8), (uint8_t)(i >> 16), (uint8_t)(i >> 24)};
            sha_update(&f, tail, 5);
            sha_final(&f, wide + 32 * j);
        }
        uint64_t x[8];
        for (int k = 0; k < 8; ++k) {
            uint64_t w = 0;
            for (int b = 7; b >= 0; --b) w = (w << 8) | wide[8 * k + b];
            x[k] = w;
        }
        out[i] = reduce512(x);
        int rc = ts_record(t, out[i]);
        if (rc) return rc;
    }
    if (n > 0) {
        uint8_t tag = 0xF2, zero = 0;
        sha_update(&t->s, &tag, 1);
        while (t->s.fill != 0) sha_update(&t->s, &zero, 1);
    }
    return 0;
}

zko_ts* zko_ts_new(uint64_t seed) {
    init_mu();
    zko_ts* t = (zko_ts*)calloc(1, sizeof(zko_ts));
    if (!t) return 0;
    transcript_init(&t->s, seed);
    return t;
}

void zko_ts_free(zko_ts* t) {
    if (t) {
        free(t->chal);
        free(t);
    }
}

int zko_ts_absorb(zko_ts* t, const char* label, const uint8_t* data, uint64_t n) {
    if (!t || !label || strlen(label) > 32) return ZKO_EARG;
    transcript_absorb(&t->s, label, data, n);
    return 0;
}

int zko_ts_draw(zko_ts* t, int n, uint8_t* out) { /* out: n x 32 bytes */
    fe* c = (fe*)malloc(sizeof(fe) * (size_t)(n > 0 ? n : 1));
    int rc = ts_draw(t, n, c);
    for (int i = 0; i < n && !rc; ++i) fe_store(c[i], out + 32 * i);
    free(c);
    return rc;
}

int zko_ts_digest(const zko_ts* t, uint8_t out[32]) {
    sha_final(&t->s, out);
    return 0;
}

uint64_t zko_ts_nchal(const zko_ts* t) { return t->nchal; }

int zko_ts_challenges(const zko_ts* t, uint8_t* out) { /* every challenge drawn so far, in order */
    for (size_t i = 0; i < t->nchal; ++i) fe_store(t->chal[i], out + 32 * i);
    return 0;
}

/* ---- beta~(u, .) as a table: entry b = prod_k (u_k b_k + (1 - u_k)(1 - b_k)), coordinate 0 the most
 * significant bit of b (Sec. 2.2).  Built coordinate by coordinate from the last one: the table over
 * (u_k, .., u_{m-1}) is (1 - u_k) times the table over (u_{k+1}, ..) followed by u_k times it. ---- */
static fe* beta_table(const fe* u, int m) {
    uint64_t n = (uint64_t)1 << m;
    fe* t = (fe*)malloc(sizeof(fe) * n);
    if (!t) return 0;
    t[0] = fe_one();
    uint64_t len = 1;
    for (int k = m - 1; k >= 0; --k) {
        fe uk = u[k], nk = fe_sub(fe_one(), u[k]);
#pragma omp parallel for schedule(static) if (len >= 4096)
        for (uint64_t b = 0; b < len; ++b) {
            fe e = t[b];
            t[len + b] = fe_mul(e, uk);
            t[b] = fe_mul(e, nk);
        }
        len *= 2;
    }
    return t;
}

/* out[o, i] = sum_a beta~(point, a) src[o, a, i]  (Eq. multilinear-extension on one axis) */
static int partial_eval_fe(const fe* src, uint64_t O, uint64_t A, uint64_t I, const fe* point, fe* out) {
    int la = ilog2_u64(A);
    if (la < 0) return ZKO_EARG;
    fe* beta = beta_table(point, la);
    if (!beta) return ZKO_ENOMEM;
#pragma omp parallel for collapse(2) schedule(static)
    for (uint64_t o = 0; o < O; ++o) {
        for (uint64_t i = 0; i < I; ++i) {
            fe acc = fe_zero();
            for (uint64_t a = 0; a < A; ++a) acc = fe_add(acc, fe_mul(beta[a], src[(o * A + a) * I + i]));
            out[o * I + i] = acc;
        }
    }
    free(beta);
    return 0;
}

/* S~(u) = sum_b S(b) beta~(u, b) */
static int mle_eval_fe(const fe* table, int m, const fe* u, fe* out) {
    return partial_eval_fe(table, 1, (uint64_t)1 << m, 1, u, out);
}

/* value at v of the polynomial of degree < n through (k, ys[k]), k = 0..n-1 */
static fe lagrange_eval(const fe* ys, int n, fe v) {
    fe acc = fe_zero();
    for (int k = 0; k < n; ++k) {
        fe num = fe_one(), den = fe_one();
        for (int j = 0; j < n; ++j) {
            if (j == k) continue;
            num = fe_mul(num, fe_sub(v, fe_from_u64((uint64_t)j)));
            den = fe_mul(den, fe_from_i64((int64_t)k - (int64_t)j));
        }
        acc = fe_add(acc, fe_mul(fe_mul(ys[k], num), fe_inv(den)));
    }
    return acc;
}

/* ---- the textbook sumcheck prover (Sec. 2.2; round structure of App. B) for
 *      sum_b F(b),  F = sum_terms coef * prod_k T_k,  every T_k multilinear in (some of) d variables ---- */
#define SC_MAX_TABLES 10
#define SC_MAX_TERMS 8
#define SC_MAX_EVALS 4

typedef struct {
    fe* data;   /* 2^(hi - max(lo, t)) entries at round t */
    int lo, hi; /* the table depends on variables lo .. hi-1 of the d variables */
} vtab;

typedef struct {
    fe coef;
    int nfac;
    int fac[4];
} scterm;

typedef void (*sc_report_fn)(const fe* all, fe* out);

/* T[b] at round t (variables t .. d-1 remain; b has d - t bits, variable t the most significant) */
static fe vt_get(const vtab* T, int t, int d, uint64_t b) {
    if (t >= T->hi) return T->data[0];
    uint64_t idx = b >> (d - T->hi);
    if (t < T->lo) idx &= (((uint64_t)1 << (T->hi - T->lo)) - 1);
    return T->data[idx];
}

/* sum over the terms of coef * (sum of the products), from per-term sums */
static fe combine_terms(const scterm* terms, int nterms, const fe* sums) {
    fe total = fe_zero();
    for (int j = 0; j < nterms; ++j) total = fe_add(total, fe_mul(terms[j].coef, sums[j]));
    return total;
}

/* Writes one SC block ("ZKSC", n_finals, degree, rounds, claim_0, rounds x (degree+1) evaluations,
 * finals).  vs: the d challenges; finals_all: every table's last value; the tables are consumed. */
static int sc_prove(vtab* T, int nt, const scterm* terms, int nterms, int degree, int d, zko_ts* ts,
                    int absorb_claim, sc_report_fn report, int n_report, wbuf* wb, fe* vs, fe* finals_all,
                    fe* claim0_out, fe* finals_out, const char* what) {
    if (nt > SC_MAX_TABLES || nterms > SC_MAX_TERMS || degree + 1 > SC_MAX_EVALS) return ZKO_EARG;
    const int nthreads = max_threads();
    const int ne = degree + 1;
    fe* part = (fe*)malloc(sizeof(fe) * (size_t)nthreads * SC_MAX_TERMS * SC_MAX_EVALS);
    if (!part) return ZKO_ENOMEM;
#define PART(th, j, x) part[((size_t)(th) * SC_MAX_TERMS + (j)) * SC_MAX_EVALS + (x)]

    /* claim_0 = sum over the hypercube */
    for (int i = 0; i < nthreads * SC_MAX_TERMS * SC_MAX_EVALS; ++i) part[i] = fe_zero();
    const uint64_t n = (uint64_t)1 << d;
#pragma omp parallel
    {
        fe acc[SC_MAX_TERMS];
        for (int j = 0; j < nterms; ++j) acc[j] = fe_zero();
#pragma omp for schedule(static)
        for (uint64_t b = 0; b < n; ++b) {
            fe e[SC_MAX_TABLES];
            for (int k = 0; k < nt; ++k) e[k] = vt_get(&T[k], 0, d, b);
            for (int j = 0; j < nterms; ++j) {
                fe p = e[terms[j].fac[0]];
                for (int f = 1; f < terms[j].nfac; ++f) p = fe_mul(p, e[terms[j].fac[f]]);
                acc[j] = fe_add(acc[j], p);
            }
        }
        for (int j = 0; j < nterms; ++j) PART(my_thread(), j, 0) = acc[j];
    }
    fe sums[SC_MAX_TERMS];
    for (int j = 0; j < nterms; ++j) {
        sums[j] = fe_zero();
        for (int th = 0; th < nthreads; ++th) sums[j] = fe_add(sums[j], PART(th, j, 0));
    }
    fe claim = combine_terms(terms, nterms, sums);
    if (claim0_out) *claim0_out = claim;
    wb_u32(wb, 0x43534B5Au);
    wb_u32(wb, (uint32_t)n_report);
    wb_u32(wb, (uint32_t)degree);
    wb_u32(wb, (uint32_t)d);
    wb_fe(wb, claim);
    if (absorb_claim) ts_absorb_fe(ts, "c", &claim, 1);

    for (int t = 0; t < d; ++t) {
        if (g_progress) g_progress(what, t, d);
        const uint64_t half = (uint64_t)1 << (d - t - 1);
        for (int i = 0; i < nthreads * SC_MAX_TERMS * SC_MAX_EVALS; ++i) part[i] = fe_zero();
#pragma omp parallel
        {
            fe acc[SC_MAX_TERMS][SC_MAX_EVALS];
            for (int j = 0; j < nterms; ++j)
                for (int x = 0; x < ne; ++x) acc[j][x] = fe_zero();
#pragma omp for schedule(static)
            for (uint64_t b = 0; b < half; ++b) {
                fe e[SC_MAX_TABLES], dlt[SC_MAX_TABLES];
                for (int k = 0; k < nt; ++k) {
                    e[k] = vt_get(&T[k], t, d, b);
                    dlt[k] = fe_sub(vt_get(&T[k], t, d, b + half), e[k]);
                }
                for (int x = 0; x < ne; ++x) { /* e[k] = lo + x (hi - lo) */
                    for (int j = 0; j < nterms; ++j) {
                        fe p = e[terms[j].fac[0]];
                        for (int f = 1; f < terms[j].nfac; ++f) p = fe_mul(p, e[terms[j].fac[f]]);
                        acc[j][x] = fe_add(acc[j][x], p);
                    }
                    for (int k = 0; k < nt; ++k) e[k] = fe_add(e[k], dlt[k]);
                }
            }
            for (int j = 0; j < nterms; ++j)
                for (int x = 0; x < ne; ++x) PART(my_thread(), j, x) = acc[j][x];
        }
        fe g[SC_MAX_EVALS];
        for (int x = 0; x < ne; ++x) {
            for (int j = 0; j < nterms; ++j) {
                sums[j] = fe_zero();
                for (int th = 0; th < nthreads; ++th) sums[j] = fe_add(sums[j], PART(th, j, x));
            }
            g[x] = combine_terms(terms, nterms, sums);
        }
        /* the round check of Sec. 2.2 */
        if (!fe_eq(fe_add(g[0], g[1]), claim)) {
            free(part);
            return ZKO_ECHECK;
        }
        /* the transcript takes g(0), g(2), .., g(degree): g(1) is fixed by the check above */
        fe msg[SC_MAX_EVALS];
        int nm = 0;
        for (int x = 0; x < ne; ++x) {
            wb_fe(wb, g[x]);
            if (x != 1) msg[nm++] = g[x];
        }
        ts_absorb_fe(ts, "g", msg, nm);
        fe v;
        int rc = ts_draw(ts, 1, &v);
        if (rc) {
            free(part);
            return rc;
        }
        vs[t] = v;
        /* bind variable t: T'[b] = T[b] + v (T[b + half'] - T[b]) on every table that depends on it */
        for (int k = 0; k < nt; ++k) {
            if (t < T[k].lo || t >= T[k].hi) continue;
            const uint64_t h = (uint64_t)1 << (T[k].hi - t - 1);
            fe* data = T[k].data;
#pragma omp parallel for schedule(static) if (h >= 1024)
            for (uint64_t b = 0; b < h; ++b) data[b] = fe_add(data[b], fe_mul(v, fe_sub(data[b + h], data[b])));
        }
        claim = lagrange_eval(g, ne, v);
    }
    for (int k = 0; k < nt; ++k) finals_all[k] = T[k].data[0];
    fe rep[SC_MAX_TABLES];
    if (report) {
        report(finals_all, rep);
    } else {
        for (int k = 0; k < nt; ++k) rep[k] = finals_all[k];
    }
    for (int k = 0; k < n_report; ++k) {
        wb_fe(wb, rep[k]);
        if (finals_out) finals_out[k] = rep[k];
    }
    ts_absorb_fe(ts, "f", rep, n_report);
    /* the last claim equals F at the challenge point */
    for (int j = 0; j < nterms; ++j) {
        fe p = finals_all[terms[j].fac[0]];
        for (int f = 1; f < terms[j].nfac; ++f) p = fe_mul(p, finals_all[terms[j].fac[f]]);
        sums[j] = p;
    }
    free(part);
#undef PART
    if (!fe_eq(combine_terms(terms, nterms, sums), claim)) return ZKO_ECHECK;
    return 0;
}

static scterm product_term(int k) {
    scterm t;
    t.coef = fe_one();
    t.nfac = k;
    for (int i = 0; i < k; ++i) t.fac[i] = i;
    return t;
}

/* ---- batched matrix product (Eq. exm-matmul-batched) ----
 * Y[n] = X0[n] X1[n], X0 [N, D1, D2], X1 [N, D2, D3]:
 *   Y~(w, u0, u1) = sum_{n, i} beta~(w, n) X0~(n, u0, i) X1~(n, i, u1).
 * Header "sumcheck_matmul" (N, D1, D2, D3); one draw (w, u0, u1); the sumcheck over (n, i) with the
 * three tables beta~(w, n), X0~(n, u0, i), X1~(n, i, u1), degree 3. */
typedef struct {
    int ln, l1, l2, l3;
    fe w[32], u0[32], u1[32], v[64];
    fe claim0, finals[3];
} mm_info;

static int matmul_core(const fe* x0, const fe* x1, uint64_t n, uint64_t d1, uint64_t d2, uint64_t d3, zko_ts* ts,
                       wbuf* wb, mm_info* info, const char* what) {
    int ln = ilog2_u64(n), l1 = ilog2_u64(d1), l2 = ilog2_u64(d2), l3 = ilog2_u64(d3);
    if (ln < 0 || l1 < 0 || l2 < 0 || l3 < 0 || ln > 32 || l1 > 32 || l3 > 32 || ln + l2 > 64) return ZKO_EARG;
    uint32_t hdr[4] = {(uint32_t)n, (uint32_t)d1, (uint32_t)d2, (uint32_t)d3};
    ts_absorb_u32(ts, "sumcheck_matmul", hdr, 4);
    fe pt[96];
    int rc = ts_draw(ts, ln + l1 + l3, pt);
    if (rc) return rc;
    info->ln = ln; info->l1 = l1; info->l2 = l2; info->l3 = l3;
    for (int k = 0; k < ln; ++k) info->w[k] = pt[k];
    for (int k = 0; k < l1; ++k) info->u0[k] = pt[ln + k];
    for (int k = 0; k < l3; ++k) info->u1[k] = pt[ln + l1 + k];
    fe* t0 = (fe*)malloc(sizeof(fe) * n * d2);
    fe* t1 = (fe*)malloc(sizeof(fe) * n * d2);
    fe* tb = beta_table(info->w, ln);
    if (!t0 || !t1 || !tb) return ZKO_ENOMEM;
    rc = partial_eval_fe(x0, n, d1, d2, info->u0, t0);          /* X0~(n, u0, i) */
    if (!rc) rc = partial_eval_fe(x1, n * d2, d3, 1, info->u1, t1); /* X1~(n, i, u1) */
    if (!rc) {
        vtab T[3] = {{tb, 0, ln}, {t0, 0, ln + l2}, {t1, 0, ln + l2}};
        scterm term = product_term(3);
        fe all[3];
        rc = sc_prove(T, 3, &term, 1, 3, ln + l2, ts, 1, 0, 3, wb, info->v, all, &info->claim0, info->finals, what);
    }
    free(t0);
    free(t1);
    free(tb);
    return rc;
}

/* ---- batched matrix product, optimized aggregated protocol (App. B, Protocol tensor-op-aggr-optimized) ----
 * Stack rounds t = 0 .. log N - 1: the prover sends, at x = 0, 1, 2,
 *   f_t(x) = sum_{n'} beta~(w_[t+1:], n') sum_i X0~(v_<t, x, n', u0, i) X1~(v_<t, x, n', i, u1),
 * the round polynomial without its factor beta~(w_t, x); the verifier's check is
 * (1 - w_t) f_t(0) + w_t f_t(1) = claim, the next claim f_t(v_t).  Then the sumcheck of the single
 * product sum_i X0~(v, u0, i) X1~(v, i, u1) (K = 2, degree 2, claim_0 not absorbed again).
 * Header "sumcheck_matmul_ft" (N, D1, D2, D3); one draw (w, u0, u1); "c" claim_0; per stack round "f"
 * (three evaluations) and a draw.  Proof: "ZKSF", log N, log D2, 0, claim_0, log N x 3 evaluations, SC block. */
static int matmul_ft_core(const fe* x0, const fe* x1, uint64_t n, uint64_t d1, uint64_t d2, uint64_t d3, zko_ts* ts,
                          wbuf* wb, mm_info* info, const char* what) {
    int ln = ilog2_u64(n), l1 = ilog2_u64(d1), l2 = ilog2_u64(d2), l3 = ilog2_u64(d3);
    if (ln < 0 || l1 < 0 || l2 < 0 || l3 < 0 || ln > 32 || l1 > 32 || l3 > 32 || ln + l2 > 64) return ZKO_EARG;
    uint32_t hdr[4] = {(uint32_t)n, (uint32_t)d1, (uint32_t)d2, (uint32_t)d3};
    ts_absorb_u32(ts, "sumcheck_matmul_ft", hdr, 4);
    fe pt[96];
    int rc = ts_draw(ts, ln + l1 + l3, pt);
    if (rc) return rc;
    info->ln = ln; info->l1 = l1; info->l2 = l2; info->l3 = l3;
    for (int k = 0; k < ln; ++k) info->w[k] = pt[k];
    for (int k = 0; k < l1; ++k) info->u0[k] = pt[ln + k];
    for (int k = 0; k < l3; ++k) info->u1[k] = pt[ln + l1 + k];
    fe* t0 = (fe*)malloc(sizeof(fe) * n * d2);
    fe* t1 = (fe*)malloc(sizeof(fe) * n * d2);
    if (!t0 || !t1) return ZKO_ENOMEM;
    rc = partial_eval_fe(x0, n, d1, d2, info->u0, t0);
    if (!rc) rc = partial_eval_fe(x1, n * d2, d3, 1, info->u1, t1);
    if (rc) return rc;
    const int nthreads = max_threads();
    fe* part = (fe*)malloc(sizeof(fe) * (size_t)nthreads * 4);
    if (!part) return ZKO_ENOMEM;
    /* claim_0 = sum_n beta~(w, n) sum_i T0[n, i] T1[n, i] = Y~(w, u0, u1) */
    fe* bw = beta_table(info->w, ln);
    if (!bw) return ZKO_ENOMEM;
    fe claim = fe_zero();
    for (uint64_t row = 0; row < n; ++row) {
        fe dot = fe_zero();
        for (uint64_t i = 0; i < d2; ++i) dot = fe_add(dot, fe_mul(t0[row * d2 + i], t1[row * d2 + i]));
        claim = fe_add(claim, fe_mul(bw[row], dot));
    }
    free(bw);
    info->claim0 = claim;
    wb_u32(wb, 0x46534B5Au);
    wb_u32(wb, (uint32_t)ln);
    wb_u32(wb, (uint32_t)l2);
    wb_u32(wb, 0);
    wb_fe(wb, claim);
    ts_absorb_fe(ts, "c", &claim, 1);
    uint64_t rows = n;
    for (int t = 0; t < ln; ++t) {
        if (g_progress) g_progress(what, t, ln);
        const uint64_t half = rows / 2;
        fe* bs = beta_table(info->w + t + 1, ln - t - 1); /* beta~(w_[t+1:], n'), half entries */
        if (!bs) return ZKO_ENOMEM;
        for (int i = 0; i < nthreads * 4; ++i) part[i] = fe_zero();
#pragma omp parallel
        {
            fe acc[3] = {fe_zero(), fe_zero(), fe_zero()};
#pragma omp for schedule(static)
            for (uint64_t row = 0; row < half; ++row) {
                fe dot[3] = {fe_zero(), fe_zero(), fe_zero()};
                for (uint64_t i = 0; i < d2; ++i) {
                    fe a = t0[row * d2 + i], b = t1[row * d2 + i];
                    const fe da = fe_sub(t0[(row + half) * d2 + i], a), db = fe_sub(t1[(row + half) * d2 + i], b);
                    for (int x = 0; x < 3; ++x) { /* a = lo + x (hi - lo) */
                        dot[x] = fe_add(dot[x], fe_mul(a, b));
                        a = fe_add(a, da);
                        b = fe_add(b, db);
                    }
                }
                for (int x = 0; x < 3; ++x) acc[x] = fe_add(acc[x], fe_mul(bs[row], dot[x]));
            }
            for (int x = 0; x < 3; ++x) part[my_thread() * 4 + x] = acc[x];
        }
        free(bs);
        fe f[3];
        for (int x = 0; x < 3; ++x) {
            f[x] = fe_zero();
            for (int th = 0; th < nthreads; ++th) f[x] = fe_add(f[x], part[th * 4 + x]);
        }
        /* g_t(x) = beta~(w_t, x) f_t(x): g_t(0) + g_t(1) = (1 - w_t) f_t(0) + w_t f_t(1) = claim */
        fe chk = fe_add(fe_mul(fe_sub(fe_one(), info->w[t]), f[0]), fe_mul(info->w[t], f[1]));
        if (!fe_eq(chk, claim)) return ZKO_ECHECK;
        for (int x = 0; x < 3; ++x) wb_fe(wb, f[x]);
        ts_absorb_fe(ts, "f", f, 3);
        fe v;
        rc = ts_draw(ts, 1, &v);
        if (rc) return rc;
        info->v[t] = v;
#pragma omp parallel for schedule(static)
        for (uint64_t b = 0; b < half * d2; ++b) {
            t0[b] = fe_add(t0[b], fe_mul(v, fe_sub(t0[b + half * d2], t0[b])));
            t1[b] = fe_add(t1[b], fe_mul(v, fe_sub(t1[b + half * d2], t1[b])));
        }
        claim = lagrange_eval(f, 3, v);
        rows = half;
    }
    free(part);
    vtab T[2] = {{t0, 0, l2}, {t1, 0, l2}};
    scterm term = product_term(2);
    fe all[2], inner0;
    rc = sc_prove(T, 2, &term, 1, 2, l2, ts, 0, 0, 2, wb, info->v + ln, all, &inner0, info->finals, what);
    free(t0);
    free(t1);
    if (rc) return rc;
    if (!fe_eq(inner0, claim)) return ZKO_ECHECK; /* the single-product sumcheck starts at f_{n-1}(v_{n-1}) */
    return 0;
}

/* ---- batched Hadamard product (Eq. exm-hadamard-batched): Y~(p) = sum_b beta~(p, b) X0(b) X1(b) ---- */
static int hadamard_core(const fe* x0, const fe* x1, int d, zko_ts* ts, wbuf* wb) {
    if (d < 0 || d > 40) return ZKO_EARG;
    uint32_t hdr[1] = {(uint32_t)d};
    ts_absorb_u32(ts, "sumcheck_hadamard", hdr, 1);
    fe p[64], vs[64], all[3];
    int rc = ts_draw(ts, d, p);
    if (rc) return rc;
    uint64_t n = (uint64_t)1 << d;
    fe* tb = beta_table(p, d);
    fe* a = (fe*)malloc(sizeof(fe) * n);
    fe* b = (fe*)malloc(sizeof(fe) * n);
    if (!tb || !a || !b) return ZKO_ENOMEM;
    memcpy(a, x0, sizeof(fe) * n);
    memcpy(b, x1, sizeof(fe) * n);
    vtab T[3] = {{tb, 0, d}, {a, 0, d}, {b, 0, d}};
    scterm term = product_term(3);
    rc = sc_prove(T, 3, &term, 1, 3, d, ts, 1, 0, 3, wb, vs, all, 0, 0, "hadamard");
    free(tb);
    free(a);
    free(b);
    return rc;
}

/* ---- zkReLU (Sec. 3.1, App. A) ---- */
typedef struct {
    int li, lj, mode;
    fe u[4][40]; /* u_Z, u_A, u_GA, u_GZ */
    fe c_in[4];
    fe v[64];    /* the li + lj challenges of the combined sumcheck */
    fe finals[3];
    fe vm[8];    /* the 1 + lj challenges of the merge */
    fe merge_finals[2];
} zk_info;

static void zk_report(const fe* all, fe* out) { /* aux~(0,v,w), aux~(1,v,w), aux~(0,v,Q+R-1) = 1 - (1 - sign)~(v) */
    out[0] = all[5];
    out[1] = all[6];
    out[2] = fe_sub(fe_one(), all[7]);
}

/* s_{Q+R} and s', zero-padded to J entries (Sec. 3.1; App. A): s_B = (1, 2, .., 2^(B-2), -2^(B-1));
 * s' picks the rescaled value aux[R:Q+R] . s_Q + aux[R-1] = (0^(R-1), 1, 1, 2, .., 2^(Q-2), -2^(Q-1)). */
static void recomposition_vectors(int q, int rb, int J, __int128* s, __int128* sp) {
    int b = q + rb;
    for (int j = 0; j < J; ++j) s[j] = sp[j] = 0;
    for (int j = 0; j < b - 1; ++j) s[j] = (__int128)1 << j;
    s[b - 1] = -((__int128)1 << (b - 1));
    sp[rb - 1] = 1;
    for (int j = rb; j < b - 1; ++j) sp[j] = (__int128)1 << (j - rb);
    sp[b - 1] = -((__int128)1 << (q - 1));
}

static fe fe_from_i128(__int128 x) { /* |x| < 2^64 here */
    if (x >= 0) return fe_from_u64((uint64_t)x);
    return fe_neg(fe_from_u64((uint64_t)(-x)));
}

static int zkrelu_core(const int64_t* z, const int64_t* ga_in, uint64_t D, int q, int rb, zko_ts* ts,
                       const fe* points, int bind_points, wbuf* wb, zk_info* info) {
    const int li = ilog2_u64(D);
    const int b = q + rb;
    if (li < 0 || li > 40 || rb < 1 || q < 1 || b > 64) return ZKO_EARG;
    int lj = 0;
    while ((1 << lj) < b) ++lj;
    const int J = 1 << lj;
    const int has_ga = ga_in != 0;
    int rc = 0;
    int64_t* ga = (int64_t*)calloc(D, sizeof(int64_t)); /* G_A = 0 stands for the forward-only use */
    if (!ga) return ZKO_ENOMEM;
    if (has_ga) memcpy(ga, ga_in, sizeof(int64_t) * D);
    /* Theorem completeness: Z and G_A are (Q+R)-bit signed integers */
    if (b < 64) {
        const int64_t lim = (int64_t)1 << (b - 1);
        for (uint64_t i = 0; i < D; ++i)
            if (z[i] < -lim || z[i] >= lim || ga[i] < -lim || ga[i] >= lim) {
                free(ga);
                return ZKO_ERANGE;
            }
    }
    __int128 s[64], sp[64];
    recomposition_vectors(q, rb, J, s, sp);
    const uint64_t n = D * (uint64_t)J;

    /* aux(k, i, j) = bit j of the two's-complement value (Eqs. aux-Z, aux-GA), zero columns up to J;
     * the tensors recomposed from it (Sec. 3.1): Z, Z', sign, A = (1 - sign) Z', G_A, G_A', G_Z */
    fe* aux0 = (fe*)malloc(sizeof(fe) * n);
    fe* aux1 = (fe*)malloc(sizeof(fe) * n);
    fe* Zf = (fe*)malloc(sizeof(fe) * D);
    fe* Af = (fe*)malloc(sizeof(fe) * D);
    fe* GAf = (fe*)malloc(sizeof(fe) * D);
    fe* GZf = (fe*)malloc(sizeof(fe) * D);
    fe* oms = (fe*)malloc(sizeof(fe) * D); /* 1 - aux(0, i, Q+R-1) */
    if (!aux0 || !aux1 || !Zf || !Af || !GAf || !GZf || !oms) return ZKO_ENOMEM;
#pragma omp parallel for schedule(static)
    for (uint64_t i = 0; i < D; ++i) {
        const uint64_t zb = (uint64_t)z[i], gb = (uint64_t)ga[i];
        __int128 z_rec = 0, zp = 0, g_rec = 0, gp = 0;
        for (int j = 0; j < J; ++j) {
            const int b0 = j < b ? (int)((zb >> j) & 1) : 0;
            const int b1 = j < b ? (int)((gb >> j) & 1) : 0;
            aux0[i * J + j] = fe_from_u64((uint64_t)b0);
            aux1[i * J + j] = fe_from_u64((uint64_t)b1);
            if (b0) { z_rec += s[j]; zp += sp[j]; }
            if (b1) { g_rec += s[j]; gp += sp[j]; }
        }
        const int sgn = (int)((zb >> (b - 1)) & 1);
        Zf[i] = fe_from_i128(z_rec);
        GAf[i] = fe_from_i128(g_rec);
        Af[i] = sgn ? fe_zero() : fe_from_i128(zp);
        GZf[i] = sgn ? fe_zero() : fe_from_i128(gp);
        oms[i] = fe_from_u64((uint64_t)(1 - sgn));
    }

    /* header and points */
    fe u_bin[64];
    if (!points) {
        uint32_t hdr[4] = {(uint32_t)li, (uint32_t)q, (uint32_t)rb, (uint32_t)has_ga};
        ts_absorb_u32(ts, "zkrelu", hdr, 4);
        fe* pt = (fe*)malloc(sizeof(fe) * (size_t)(5 * li + lj + 1));
        rc = ts_draw(ts, 5 * li + lj, pt);
        if (rc) return rc;
        for (int k = 0; k < 4; ++k)
            for (int c = 0; c < li; ++c) info->u[k][c] = pt[k * li + c];
        for (int c = 0; c < li + lj; ++c) u_bin[c] = pt[4 * li + c];
        free(pt);
        info->mode = 0;
    } else {
        info->mode = bind_points ? 1 : 2;
        uint32_t hdr[5] = {(uint32_t)li, (uint32_t)q, (uint32_t)rb, (uint32_t)has_ga, (uint32_t)info->mode};
        ts_absorb_u32(ts, "zkrelu_at", hdr, 5);
        for (int k = 0; k < 4; ++k)
            for (int c = 0; c < li; ++c) info->u[k][c] = points[k * li + c];
        if (bind_points) { /* SHA-256 of the four points, 32 bytes little-endian per coordinate */
            sha_ctx h;
            sha_init(&h);
            for (int k = 0; k < 4; ++k)
                for (int c = 0; c < li; ++c) {
                    uint8_t e[32];
                    fe_store(info->u[k][c], e);
                    sha_update(&h, e, 32);
                }
            uint8_t dg[32];
            sha_final(&h, dg);
            transcript_absorb(&ts->s, "u", dg, 32);
        }
        rc = ts_draw(ts, li + lj, u_bin);
        if (rc) return rc;
    }
    info->li = li;
    info->lj = lj;

    /* the four input claims Z~(u_Z), A~(u_A), G_A~(u_GA), G_Z~(u_GZ) */
    const fe* inputs[4] = {Zf, Af, GAf, GZf};
    for (int k = 0; k < 4; ++k) {
        rc = mle_eval_fe(inputs[k], li, info->u[k], &info->c_in[k]);
        if (rc) return rc;
    }
    ts_absorb_fe(ts, "c", info->c_in, 4);
    fe rr[2];
    rc = ts_draw(ts, 2, rr);
    if (rc) return rc;
    const fe r = rr[0], rp = rr[1], r2 = fe_mul(rr[0], rr[0]);

    /* the ten tables of the combined sumcheck over (i, j), i first */
    fe* sj = (fe*)malloc(sizeof(fe) * J);
    fe* spj = (fe*)malloc(sizeof(fe) * J);
    for (int j = 0; j < J; ++j) {
        sj[j] = fe_from_i128(s[j]);
        spj[j] = fe_from_i128(sp[j]);
    }
    fe* bt[4];
    for (int k = 0; k < 4; ++k) {
        bt[k] = beta_table(info->u[k], li);
        if (!bt[k]) return ZKO_ENOMEM;
    }
    fe* bbin = beta_table(u_bin, li + lj);
    if (!bbin) return ZKO_ENOMEM;
    const int d = li + lj;
    vtab T[10] = {
        {bt[0], 0, li}, {bt[1], 0, li}, {bt[2], 0, li}, {bt[3], 0, li}, /* beta~(u_Z, i) .. beta~(u_GZ, i) */
        {bbin, 0, d},                                                  /* beta~(u_bin, (i, j)) */
        {aux0, 0, d}, {aux1, 0, d},                                    /* aux(0, i, j), aux(1, i, j) */
        {oms, 0, li},                                                  /* 1 - aux(0, i, Q+R-1) */
        {sj, li, d}, {spj, li, d},                                     /* s_{Q+R}(j), s'(j) */
    };
    /* the six equations of App. A with weights r^2, r, 1, r'r^2, r'r, r' (binarity as a^2 - a) */
    const fe minus1 = fe_neg(fe_one());
    scterm terms[8] = {
        {r2, 3, {0, 5, 8, 0}},
        {r, 4, {1, 7, 5, 9}},
        {fe_one(), 3, {4, 5, 5, 0}},
        {minus1, 2, {4, 5, 0, 0}},
        {fe_mul(rp, r2), 3, {2, 6, 8, 0}},
        {fe_mul(rp, r), 4, {3, 7, 6, 9}},
        {rp, 3, {4, 6, 6, 0}},
        {fe_neg(rp), 2, {4, 6, 0, 0}},
    };
    /* proof header and the claims go out before the SC blocks */
    wb_u32(wb, 0x4C524B5Au);
    wb_u32(wb, (uint32_t)li);
    wb_u32(wb, (uint32_t)q);
    wb_u32(wb, (uint32_t)rb);
    wb_u32(wb, (uint32_t)has_ga);
    wb_u32(wb, (uint32_t)info->mode);
    wb_u32(wb, 0);
    wb_u32(wb, 0);
    for (int k = 0; k < 4; ++k) wb_fe(wb, info->c_in[k]);
    fe all[10], claim0;
    rc = sc_prove(T, 10, terms, 8, 3, d, ts, 0, zk_report, 3, wb, info->v, all, &claim0, info->finals, "zkrelu");
    free(bbin);
    free(aux0);
    free(aux1);
    for (int k = 0; k < 4; ++k) free(bt[k]);
    free(Zf); free(Af); free(GAf); free(GZf); free(oms);
    if (rc) return rc;
    /* the combined claim is the weighted sum of the input claims */
    fe expect0 = fe_add(fe_add(fe_mul(r2, info->c_in[0]), fe_mul(r, info->c_in[1])),
                        fe_add(fe_mul(fe_mul(rp, r2), info->c_in[2]), fe_mul(fe_mul(rp, r), info->c_in[3])));
    if (!fe_eq(claim0, expect0)) return ZKO_ECHECK;

    /* merge of the three claims on aux: M[k, j] = aux~(k, v, j) = sum_i beta~(v, i) aux(k, i, j) */
    const fe* v_i = info->v;
    const fe* wbar = info->v + li;
    fe* bv = beta_table(v_i, li);
    fe* M = (fe*)malloc(sizeof(fe) * 2 * J);
    if (!bv || !M) return ZKO_ENOMEM;
#pragma omp parallel for schedule(static)
    for (int kj = 0; kj < 2 * J; ++kj) {
        const int k = kj / J, j = kj % J;
        const int64_t* src = k ? ga : z;
        fe acc = fe_zero();
        if (j < b)
            for (uint64_t i = 0; i < D; ++i)
                if (((uint64_t)src[i] >> j) & 1) acc = fe_add(acc, bv[i]);
        M[kj] = acc;
    }
    free(bv);
    fe chk;
    rc = mle_eval_fe(M, lj, wbar, &chk);
    if (rc || !fe_eq(chk, info->finals[0])) return rc ? rc : ZKO_ECHECK;
    rc = mle_eval_fe(M + J, lj, wbar, &chk);
    if (rc || !fe_eq(chk, info->finals[1])) return rc ? rc : ZKO_ECHECK;
    if (!fe_eq(M[b - 1], info->finals[2])) return ZKO_ECHECK;
    fe rho[3];
    rc = ts_draw(ts, 3, rho);
    if (rc) return rc;
    /* E = rho0 beta~((0, wbar), .) + rho1 beta~((1, wbar), .) + rho2 beta~((0, e_{Q+R-1}), .) */
    fe p0[8], p1[8], p2[8];
    p0[0] = fe_zero();
    p1[0] = fe_one();
    p2[0] = fe_zero();
    for (int c = 0; c < lj; ++c) {
        p0[1 + c] = wbar[c];
        p1[1 + c] = wbar[c];
        p2[1 + c] = fe_from_u64((uint64_t)(((b - 1) >> (lj - 1 - c)) & 1));
    }
    fe* e0 = beta_table(p0, 1 + lj);
    fe* e1 = beta_table(p1, 1 + lj);
    fe* e2 = beta_table(p2, 1 + lj);
    fe* E = (fe*)malloc(sizeof(fe) * 2 * J);
    for (int x = 0; x < 2 * J; ++x)
        E[x] = fe_add(fe_add(fe_mul(rho[0], e0[x]), fe_mul(rho[1], e1[x])), fe_mul(rho[2], e2[x]));
    free(e0); free(e1); free(e2);
    vtab TM[2] = {{M, 0, 1 + lj}, {E, 0, 1 + lj}};
    scterm mt = product_term(2);
    fe mall[2], mclaim0;
    rc = sc_prove(TM, 2, &mt, 1, 2, 1 + lj, ts, 0, 0, 2, wb, info->vm, mall, &mclaim0, info->merge_finals, "zkrelu-merge");
    free(M);
    free(E);
    free(sj);
    free(spj);
    free(ga);
    if (rc) return rc;
    fe em = fe_add(fe_add(fe_mul(rho[0], info->finals[0]), fe_mul(rho[1], info->finals[1])), fe_mul(rho[2], info->finals[2]));
    if (!fe_eq(mclaim0, em)) return ZKO_ECHECK;
    return 0;
}

/* ---- re-indexing of stacked tensors (Sec. 4, Eq. sc-reindex) ---- */
typedef struct {
    fe claims[8], r[8], v[40];
    fe claim0, finals[2]; /* P~(v), X~(v, u) */
} ri_info;

static int reindex_core(const fe* x, uint64_t n, uint64_t d, int K, const int32_t* const* maps, const uint64_t* map_len,
                        const fe* const* points, const fe* u, zko_ts* ts, int bind_statement, wbuf* wb, ri_info* info) {
    const int ln = ilog2_u64(n), ld = ilog2_u64(d);
    if (ln < 0 || ld < 0 || ln > 40 || K < 1 || K > 8) return ZKO_EARG;
    int lm[8];
    for (int k = 0; k < K; ++k) {
        lm[k] = ilog2_u64(map_len[k]);
        if (lm[k] < 0) return ZKO_EARG;
        for (uint64_t j = 0; j < map_len[k]; ++j)
            if (maps[k][j] < -1 || (int64_t)maps[k][j] >= (int64_t)n) return ZKO_EARG;
    }
    if (bind_statement) { /* digest of the public part of the statement: shapes, index maps, points */
        sha_ctx h;
        sha_init(&h);
        uint8_t w4[4];
        uint32_t hd[3] = {(uint32_t)n, (uint32_t)d, (uint32_t)K};
        for (int i = 0; i < 3; ++i) {
            for (int b = 0; b < 4; ++b) w4[b] = (uint8_t)(hd[i] >> (8 * b));
            sha_update(&h, w4, 4);
        }
        for (int k = 0; k < K; ++k) {
            uint32_t l = (uint32_t)map_len[k];
            for (int b = 0; b < 4; ++b) w4[b] = (uint8_t)(l >> (8 * b));
            sha_update(&h, w4, 4);
            for (uint64_t j = 0; j < map_len[k]; ++j) {
                uint32_t e = (uint32_t)maps[k][j];
                for (int b = 0; b < 4; ++b) w4[b] = (uint8_t)(e >> (8 * b));
                sha_update(&h, w4, 4);
            }
        }
        uint8_t e32[32];
        for (int k = 0; k < K; ++k)
            for (int c = 0; c < lm[k]; ++c) {
                fe_store(points[k][c], e32);
                sha_update(&h, e32, 32);
            }
        for (int c = 0; c < ld; ++c) {
            fe_store(u[c], e32);
            sha_update(&h, e32, 32);
        }
        uint8_t dg[32];
        sha_final(&h, dg);
        transcript_absorb(&ts->s, "reindex", dg, 32);
    } else {
        uint32_t hd[3] = {(uint32_t)n, (uint32_t)d, (uint32_t)K};
        ts_absorb_u32(ts, "reindex", hd, 3);
    }
    fe* t = (fe*)malloc(sizeof(fe) * n); /* X~(i, u) for every stack index i */
    fe* p = (fe*)malloc(sizeof(fe) * n);
    if (!t || !p) return ZKO_ENOMEM;
    int rc = partial_eval_fe(x, n, d, 1, u, t);
    if (rc) return rc;
    fe* bk[8];
    for (int k = 0; k < K; ++k) { /* X_k~(u_k, u) = sum_j beta~(u_k, j) X~(maps[k][j], u) */
        bk[k] = beta_table(points[k], lm[k]);
        if (!bk[k]) return ZKO_ENOMEM;
        fe acc = fe_zero();
        for (uint64_t j = 0; j < map_len[k]; ++j)
            if (maps[k][j] >= 0) acc = fe_add(acc, fe_mul(bk[k][j], t[maps[k][j]]));
        info->claims[k] = acc;
    }
    ts_absorb_fe(ts, "c", info->claims, K);
    rc = ts_draw(ts, K, info->r);
    if (rc) return rc;
    /* P[i] = sum_k r_k sum_{j : maps[k][j] = i} beta~(u_k, j) */
    for (uint64_t i = 0; i < n; ++i) p[i] = fe_zero();
    for (int k = 0; k < K; ++k) {
        for (uint64_t j = 0; j < map_len[k]; ++j)
            if (maps[k][j] >= 0) p[maps[k][j]] = fe_add(p[maps[k][j]], fe_mul(info->r[k], bk[k][j]));
        free(bk[k]);
    }
    wb_u32(wb, 0x49524B5Au);
    wb_u32(wb, (uint32_t)n);
    wb_u32(wb, (uint32_t)d);
    wb_u32(wb, (uint32_t)K);
    for (int k = 0; k < K; ++k) wb_fe(wb, info->claims[k]);
    vtab T[2] = {{p, 0, ln}, {t, 0, ln}};
    scterm term = product_term(2);
    fe all[2];
    rc = sc_prove(T, 2, &term, 1, 2, ln, ts, 1, 0, 2, wb, info->v, all, &info->claim0, info->finals, "reindex");
    free(t);
    free(p);
    if (rc) return rc;
    fe expect = fe_zero();
    for (int k = 0; k < K; ++k) expect = fe_add(expect, fe_mul(info->r[k], info->claims[k]));
    if (!fe_eq(expect, info->claim0)) return ZKO_ECHECK;
    return 0;
}

/* ---- K claims X~(s_k, q_k) on a stack X [N, D] -> one claim X~(v_n, v), on tables of D entries
 *      (the identity behind Eq. sc-reindex used twice; steps as in the Python tier's stack_merge_prove) ---- */
typedef struct {
    fe claims[8], r[8];
    fe rho[4], v[40], vn[40];
    fe inner_finals[2], outer_finals[2];
} ms_info;

static int stack_merge_core(const fe* x, uint64_t n, uint64_t d, int K, const fe* const* points, zko_ts* ts,
                            int bind_statement, wbuf* wb, ms_info* info) {
    const int ln = ilog2_u64(n), ld = ilog2_u64(d);
    if (ln < 0 || ld < 0 || ln > 40 || ld > 40 || K < 1 || K > 8) return ZKO_EARG;
    if (bind_statement) {
        sha_ctx h;
        sha_init(&h);
        uint8_t w4[4], e32[32];
        uint32_t hd[3] = {(uint32_t)n, (uint32_t)d, (uint32_t)K};
        for (int i = 0; i < 3; ++i) {
            for (int b = 0; b < 4; ++b) w4[b] = (uint8_t)(hd[i] >> (8 * b));
            sha_update(&h, w4, 4);
        }
        for (int k = 0; k < K; ++k)
            for (int c = 0; c < ln + ld; ++c) {
                fe_store(points[k][c], e32);
                sha_update(&h, e32, 32);
            }
        uint8_t dg[32];
        sha_final(&h, dg);
        transcript_absorb(&ts->s, "merge_stack", dg, 32);
    } else {
        uint32_t hd[3] = {(uint32_t)n, (uint32_t)d, (uint32_t)K};
        ts_absorb_u32(ts, "merge_stack", hd, 3);
    }
    int lk = 0;
    while ((1 << lk) < K) ++lk;
    const uint64_t kpad = (uint64_t)1 << lk;
    fe* Tt = (fe*)calloc(kpad * d, sizeof(fe)); /* T[k, x] = X~(s_k, x), zero rows up to a power of two */
    fe* Et = (fe*)calloc(kpad * d, sizeof(fe)); /* E[k, x] = r_k beta~(q_k, x) */
    if (!Tt || !Et) return ZKO_ENOMEM;
    int rc;
    for (int k = 0; k < K; ++k) {
        rc = partial_eval_fe(x, 1, n, d, points[k], Tt + (uint64_t)k * d);
        if (rc) return rc;
        rc = mle_eval_fe(Tt + (uint64_t)k * d, ld, points[k] + ln, &info->claims[k]);
        if (rc) return rc;
    }
    ts_absorb_fe(ts, "c", info->claims, K);
    rc = ts_draw(ts, K, info->r);
    if (rc) return rc;
    for (int k = 0; k < K; ++k) {
        fe* bq = beta_table(points[k] + ln, ld);
        if (!bq) return ZKO_ENOMEM;
        for (uint64_t xx = 0; xx < d; ++xx) Et[(uint64_t)k * d + xx] = fe_mul(info->r[k], bq[xx]);
        free(bq);
    }
    wb_u32(wb, 0x534D4B5Au);
    wb_u32(wb, (uint32_t)n);
    wb_u32(wb, (uint32_t)d);
    wb_u32(wb, (uint32_t)K);
    for (int k = 0; k < K; ++k) wb_fe(wb, info->claims[k]);
    vtab TI[2] = {{Et, 0, lk + ld}, {Tt, 0, lk + ld}};
    scterm term = product_term(2);
    fe all[2], vs[48], claim0;
    rc = sc_prove(TI, 2, &term, 1, 2, lk + ld, ts, 1, 0, 2, wb, vs, all, &claim0, info->inner_finals, "merge-inner");
    free(Tt);
    free(Et);
    if (rc) return rc;
    fe expect = fe_zero();
    for (int k = 0; k < K; ++k) expect = fe_add(expect, fe_mul(info->r[k], info->claims[k]));
    if (!fe_eq(expect, claim0)) return ZKO_ECHECK;
    for (int c = 0; c < lk; ++c) info->rho[c] = vs[c];
    for (int c = 0; c < ld; ++c) info->v[c] = vs[lk + c];
    /* Eq. sc-reindex over the stack index: T~(rho, v) = sum_i Pn[i] X~(i, v),
     * Pn[i] = sum_k beta~(rho, k) beta~(s_k, i) */
    fe* brho = beta_table(info->rho, lk);
    fe* pn = (fe*)malloc(sizeof(fe) * n);
    fe* tn = (fe*)malloc(sizeof(fe) * n);
    if (!brho || !pn || !tn) return ZKO_ENOMEM;
    for (uint64_t i = 0; i < n; ++i) pn[i] = fe_zero();
    for (int k = 0; k < K; ++k) {
        fe* bs = beta_table(points[k], ln);
        if (!bs) return ZKO_ENOMEM;
        for (uint64_t i = 0; i < n; ++i) pn[i] = fe_add(pn[i], fe_mul(brho[k], bs[i]));
        free(bs);
    }
    free(brho);
    rc = partial_eval_fe(x, n, d, 1, info->v, tn);
    if (rc) return rc;
    vtab TO[2] = {{pn, 0, ln}, {tn, 0, ln}};
    rc = sc_prove(TO, 2, &term, 1, 2, ln, ts, 1, 0, 2, wb, info->vn, all, &claim0, info->outer_finals, "merge-outer");
    free(pn);
    free(tn);
    if (rc) return rc;
    if (!fe_eq(claim0, info->inner_finals[1])) return ZKO_ECHECK;
    return 0;
}

/* ---- one aggregation window of an L-layer FCNN (Sec. 5, Example FCNN; Protocol zkdl, sumcheck line) ---- */

/* integer stack [n, rows, cols] as field elements; with n_layers > 0 slot (t, l) takes slot (t, l+1) and
 * the last layer's slot of every step is zero; with transpose the matrices are stored transposed */
static fe* stack_fe(const int32_t* src, uint64_t n, uint64_t rows, uint64_t cols, int n_layers, int transpose) {
    fe* out = (fe*)malloc(sizeof(fe) * n * rows * cols);
    if (!out) return 0;
#pragma omp parallel for schedule(static)
    for (uint64_t k = 0; k < n; ++k) {
        const int zero = n_layers > 0 && (k % (uint64_t)n_layers) == (uint64_t)n_layers - 1;
        const int32_t* m = src + (n_layers > 0 ? k + 1 : k) * rows * cols;
        for (uint64_t a = 0; a < rows; ++a)
            for (uint64_t c = 0; c < cols; ++c) {
                fe v = zero ? fe_zero() : fe_from_i64(m[a * cols + c]);
                if (transpose) out[(k * cols + c) * rows + a] = v;
                else out[(k * rows + a) * cols + c] = v;
            }
    }
    return out;
}

typedef struct {
    uint32_t L, B, width, T, Q, R;
    const int32_t *A, *W, *GZ;
    const int64_t *Zr, *GA;
} zko_witness;

/* the three matmul families: forward Z = A W; gradA G_A = G_Z^(l+1) W^(l+1)T; gradW G_W = A^T G_Z */
static int aggregate_matmuls(const zko_witness* w, zko_ts* ts, wbuf* wb, mm_info mm[3], fe** a_out, fe** w_out, fe** gz_out,
                             int ft) {
    const uint64_t n = (uint64_t)w->L * w->T, B = w->B, wd = w->width;
    int (*const matmul)(const fe*, const fe*, uint64_t, uint64_t, uint64_t, uint64_t, zko_ts*, wbuf*, mm_info*,
                        const char*) = ft ? matmul_ft_core : matmul_core;
    fe* a = stack_fe(w->A, n, B, wd, 0, 0);
    fe* ww = stack_fe(w->W, n, wd, wd, 0, 0);
    if (!a || !ww) return ZKO_ENOMEM;
    int rc = matmul(a, ww, n, B, wd, wd, ts, wb, &mm[0], "forward");
    if (rc) return rc;
    fe* gz_next = stack_fe(w->GZ, n, B, wd, (int)w->L, 0);
    fe* wt_next = stack_fe(w->W, n, wd, wd, (int)w->L, 1);
    if (!gz_next || !wt_next) return ZKO_ENOMEM;
    rc = matmul(gz_next, wt_next, n, B, wd, wd, ts, wb, &mm[1], "gradA");
    free(gz_next);
    free(wt_next);
    if (rc) return rc;
    fe* a_t = stack_fe(w->A, n, B, wd, 0, 1);
    fe* gz = stack_fe(w->GZ, n, B, wd, 0, 0);
    if (!a_t || !gz) return ZKO_ENOMEM;
    rc = matmul(a_t, gz, n, wd, B, wd, ts, wb, &mm[2], "gradW");
    free(a_t);
    if (a_out) *a_out = a; else free(a);
    if (w_out) *w_out = ww; else free(ww);
    if (gz_out) *gz_out = gz; else free(gz);
    return rc;
}

static void aggregate_header(const zko_witness* w, zko_ts* ts, wbuf* wb, const char* label, uint32_t magic) {
    uint32_t hdr[6] = {w->L, w->B, w->width, w->T, w->Q, w->R};
    ts_absorb_u32(ts, label, hdr, 6);
    wb_u32(wb, magic);
    for (int i = 0; i < 6; ++i) wb_u32(wb, hdr[i]);
    wb_u32(wb, 0);
}

static int witness_ok(const zko_witness* w) {
    if (!w || !w->A || !w->W || !w->GZ || !w->Zr || !w->GA) return 0;
    return ilog2_u64(w->L) >= 0 && ilog2_u64(w->B) >= 0 && ilog2_u64(w->width) >= 0 && ilog2_u64(w->T) >= 0;
}

int zko_aggregate_prove(const zko_witness* w, zko_ts* ts, uint8_t* proof, uint64_t cap, uint64_t* proof_len) {
    init_mu();
    if (!witness_ok(w) || !ts) return ZKO_EARG;
    wbuf wb = {proof, (size_t)cap, 0};
    aggregate_header(w, ts, &wb, "aggregate", 0x47414B5Au);
    mm_info mm[3];
    int rc = aggregate_matmuls(w, ts, &wb, mm, 0, 0, 0, 0);
    if (rc) return rc;
    zk_info zi;
    const uint64_t D = (uint64_t)w->L * w->T * w->B * w->width;
    rc = zkrelu_core(w->Zr, w->GA, D, (int)w->Q, (int)w->R, ts, 0, 1, &wb, &zi);
    if (rc) return rc;
    *proof_len = wb.len;
    return wb.len <= wb.cap ? 0 : ZKO_ESMALL;
}

/* the same window with the matrix-product families in the optimized aggregated form (f_t for the stack rounds) */
int zko_aggregate_ft_prove(const zko_witness* w, zko_ts* ts, uint8_t* proof, uint64_t cap, uint64_t* proof_len) {
    init_mu();
    if (!witness_ok(w) || !ts) return ZKO_EARG;
    wbuf wb = {proof, (size_t)cap, 0};
    aggregate_header(w, ts, &wb, "aggregate_ft", 0x46414B5Au);
    mm_info mm[3];
    int rc = aggregate_matmuls(w, ts, &wb, mm, 0, 0, 0, 1);
    if (rc) return rc;
    zk_info zi;
    const uint64_t D = (uint64_t)w->L * w->T * w->B * w->width;
    rc = zkrelu_core(w->Zr, w->GA, D, (int)w->Q, (int)w->R, ts, 0, 1, &wb, &zi);
    if (rc) return rc;
    *proof_len = wb.len;
    return wb.len <= wb.cap ? 0 : ZKO_ESMALL;
}

/* the same window with the claims linked (Sec. 3.2; Sec. 4, Eq. sc-reindex; Protocol zkdl): steps 1-5 of
 * the Python tier's aggregate_linked_prove */
int zko_aggregate_linked_prove(const zko_witness* w, zko_ts* ts, uint8_t* proof, uint64_t cap, uint64_t* proof_len) {
    init_mu();
    if (!witness_ok(w) || !ts) return ZKO_EARG;
    wbuf wb = {proof, (size_t)cap, 0};
    aggregate_header(w, ts, &wb, "aggregate_linked", 0x4C414B5Au);
    mm_info mm[3];
    fe *a = 0, *ww = 0, *gz = 0;
    int rc = aggregate_matmuls(w, ts, &wb, mm, &a, &ww, &gz, 0);
    if (rc) return rc;
    const uint64_t n = (uint64_t)w->L * w->T, B = w->B, wd = w->width;
    const int ln = ilog2_u64(n), lb = ilog2_u64(B), lw = ilog2_u64(wd);
    const mm_info *f = &mm[0], *g = &mm[1], *h = &mm[2];
    /* zkReLU at u_Z = point of forward's claim_0, u_A = point of its final on A, u_GA = point of gradA's
     * claim_0, u_GZ = point of gradW's final on G_Z */
    const int li = ln + lb + lw;
    fe* pts = (fe*)malloc(sizeof(fe) * 4 * (size_t)li);
    {
        fe* p = pts;
        for (int c = 0; c < ln; ++c) *p++ = f->w[c];
        for (int c = 0; c < lb; ++c) *p++ = f->u0[c];
        for (int c = 0; c < lw; ++c) *p++ = f->u1[c];
        for (int c = 0; c < ln; ++c) *p++ = f->v[c];
        for (int c = 0; c < lb; ++c) *p++ = f->u0[c];
        for (int c = 0; c < lw; ++c) *p++ = f->v[ln + c];
        for (int c = 0; c < ln; ++c) *p++ = g->w[c];
        for (int c = 0; c < lb; ++c) *p++ = g->u0[c];
        for (int c = 0; c < lw; ++c) *p++ = g->u1[c];
        for (int c = 0; c < ln; ++c) *p++ = h->v[c];
        for (int c = 0; c < lb; ++c) *p++ = h->v[ln + c];
        for (int c = 0; c < lw; ++c) *p++ = h->u1[c];
    }
    zk_info zi;
    rc = zkrelu_core(w->Zr, w->GA, n * B * wd, (int)w->Q, (int)w->R, ts, pts, 0, &wb, &zi);
    free(pts);
    if (rc) return rc;
    if (!fe_eq(zi.c_in[2], g->claim0)) return ZKO_ECHECK; /* G_A of the witness is gradA's product */
    /* index maps: the stack itself, and the stack whose slot (t, l) is slot (t, l+1) */
    int32_t* ident = (int32_t*)malloc(sizeof(int32_t) * n);
    int32_t* down = (int32_t*)malloc(sizeof(int32_t) * n);
    for (uint64_t j = 0; j < n; ++j) {
        ident[j] = (int32_t)j;
        down[j] = (j % w->L != (uint64_t)w->L - 1) ? (int32_t)(j + 1) : -1;
    }
    fe u[64];
    ri_info ra, rg, rw;
    {   /* re-indexing on A: A itself (forward's final) and the shifted stack (c_A), at forward's stack point */
        const int32_t* maps[2] = {ident, down};
        const uint64_t mlen[2] = {n, n};
        const fe* mp[2] = {f->v, f->v};
        for (int c = 0; c < lb; ++c) u[c] = f->u0[c];
        for (int c = 0; c < lw; ++c) u[lb + c] = f->v[ln + c];
        rc = reindex_core(a, n, B * wd, 2, maps, mlen, mp, u, ts, 0, &wb, &ra);
        if (rc) return rc;
        if (!fe_eq(ra.claims[0], f->finals[1]) || !fe_eq(ra.claims[1], zi.c_in[1])) return ZKO_ECHECK;
    }
    {   /* re-indexing on G_Z and on W, the shifted sub-stack alone, at gradA's stack point */
        const int32_t* maps[1] = {down};
        const uint64_t mlen[1] = {n};
        const fe* mp[1] = {g->v};
        for (int c = 0; c < lb; ++c) u[c] = g->u0[c];
        for (int c = 0; c < lw; ++c) u[lb + c] = g->v[ln + c];
        rc = reindex_core(gz, n, B * wd, 1, maps, mlen, mp, u, ts, 0, &wb, &rg);
        if (rc) return rc;
        if (!fe_eq(rg.claims[0], g->finals[1])) return ZKO_ECHECK;
        for (int c = 0; c < lw; ++c) u[c] = g->u1[c];
        for (int c = 0; c < lw; ++c) u[lw + c] = g->v[ln + c];
        rc = reindex_core(ww, n, wd * wd, 1, maps, mlen, mp, u, ts, 0, &wb, &rw);
        if (rc) return rc;
        if (!fe_eq(rw.claims[0], g->finals[2])) return ZKO_ECHECK;
    }
    ms_info ma, mw;
    fe p0[96], p1[96];
    {   /* the two claims on A: (re-indexing's v, u0, v_i of forward) and gradW's final on A^T at (v_n, v_i, u0) */
        fe* p = p0;
        for (int c = 0; c < ln; ++c) *p++ = ra.v[c];
        for (int c = 0; c < lb; ++c) *p++ = f->u0[c];
        for (int c = 0; c < lw; ++c) *p++ = f->v[ln + c];
        p = p1;
        for (int c = 0; c < ln; ++c) *p++ = h->v[c];
        for (int c = 0; c < lb; ++c) *p++ = h->v[ln + c];
        for (int c = 0; c < lw; ++c) *p++ = h->u0[c];
        const fe* mp[2] = {p0, p1};
        rc = stack_merge_core(a, n, B * wd, 2, mp, ts, 0, &wb, &ma);
        if (rc) return rc;
        if (!fe_eq(ma.claims[0], ra.finals[1]) || !fe_eq(ma.claims[1], h->finals[1])) return ZKO_ECHECK;
    }
    {   /* the two claims on W: forward's final at (v_n, v_i, u1) and the re-indexing's at (v, u1, v_i of gradA) */
        fe* p = p0;
        for (int c = 0; c < ln; ++c) *p++ = f->v[c];
        for (int c = 0; c < lw; ++c) *p++ = f->v[ln + c];
        for (int c = 0; c < lw; ++c) *p++ = f->u1[c];
        p = p1;
        for (int c = 0; c < ln; ++c) *p++ = rw.v[c];
        for (int c = 0; c < lw; ++c) *p++ = g->u1[c];
        for (int c = 0; c < lw; ++c) *p++ = g->v[ln + c];
        const fe* mp[2] = {p0, p1};
        rc = stack_merge_core(ww, n, wd * wd, 2, mp, ts, 0, &wb, &mw);
        if (rc) return rc;
        if (!fe_eq(mw.claims[0], f->finals[2]) || !fe_eq(mw.claims[1], rw.finals[1])) return ZKO_ECHECK;
    }
    free(ident);
    free(down);
    free(a);
    free(ww);
    free(gz);
    *proof_len = wb.len;
    return wb.len <= wb.cap ? 0 : ZKO_ESMALL;
}

/* ---- exported single protocols (inputs as canonical 32-byte elements, or integers for zkReLU) ---- */
static fe* load_table(const uint8_t* src, uint64_t n) {
    fe* t = (fe*)malloc(sizeof(fe) * (n ? n : 1));
    if (!t) return 0;
#pragma omp parallel for schedule(static)
    for (uint64_t b = 0; b < n; ++b) t[b] = fe_load(src + 32 * b);
    return t;
}

int zko_matmul_prove(const uint8_t* x0, const uint8_t* x1, uint64_t n, uint64_t d1, uint64_t d2, uint64_t d3, zko_ts* ts,
                     uint8_t* proof, uint64_t cap, uint64_t* proof_len) {
    init_mu();
    fe* a = load_table(x0, n * d1 * d2);
    fe* b = load_table(x1, n * d2 * d3);
    if (!a || !b) return ZKO_ENOMEM;
    wbuf wb = {proof, (size_t)cap, 0};
    mm_info info;
    int rc = matmul_core(a, b, n, d1, d2, d3, ts, &wb, &info, "matmul");
    free(a);
    free(b);
    if (rc) return rc;
    *proof_len = wb.len;
    return wb.len <= wb.cap ? 0 : ZKO_ESMALL;
}

int zko_matmul_ft_prove(const uint8_t* x0, const uint8_t* x1, uint64_t n, uint64_t d1, uint64_t d2, uint64_t d3, zko_ts* ts,
                        uint8_t* proof, uint64_t cap, uint64_t* proof_len) {
    init_mu();
    fe* a = load_table(x0, n * d1 * d2);
    fe* b = load_table(x1, n * d2 * d3);
    if (!a || !b) return ZKO_ENOMEM;
    wbuf wb = {proof, (size_t)cap, 0};
    mm_info info;
    int rc = matmul_ft_core(a, b, n, d1, d2, d3, ts, &wb, &info, "matmul_ft");
    free(a);
    free(b);
    if (rc) return rc;
    *proof_len = wb.len;
    return wb.len <= wb.cap ? 0 : ZKO_ESMALL;
}

int zko_hadamard_prove(const uint8_t* x0, const uint8_t* x1, int d, zko_ts* ts, uint8_t* proof, uint64_t cap,
                       uint64_t* proof_len) {
    init_mu();
    if (d < 0 || d > 40) return ZKO_EARG;
    fe* a = load_table(x0, (uint64_t)1 << d);
    fe* b = load_table(x1, (uint64_t)1 << d);
    if (!a || !b) return ZKO_ENOMEM;
    wbuf wb = {proof, (size_t)cap, 0};
    int rc = hadamard_core(a, b, d, ts, &wb);
    free(a);
    free(b);
    if (rc) return rc;
    *proof_len = wb.len;
    return wb.len <= wb.cap ? 0 : ZKO_ESMALL;
}

/* points: NULL (all five points drawn) or 4 log2(D) canonical elements u_Z, u_A, u_GA, u_GZ */
int zko_zkrelu_prove(const int64_t* z, const int64_t* ga, uint64_t D, int q, int rb, const uint8_t* points,
                     int bind_points, zko_ts* ts, uint8_t* proof, uint64_t cap, uint64_t* proof_len) {
    init_mu();
    int li = ilog2_u64(D);
    if (li < 0 || !z || !ts) return ZKO_EARG;
    fe* pts = 0;
    if (points) {
        pts = load_table(points, 4 * (uint64_t)li);
        if (!pts) return ZKO_ENOMEM;
    }
    wbuf wb = {proof, (size_t)cap, 0};
    zk_info info;
    int rc = zkrelu_core(z, ga, D, q, rb, ts, pts, bind_points, &wb, &info);
    free(pts);
    if (rc) return rc;
    *proof_len = wb.len;
    return wb.len <= wb.cap ? 0 : ZKO_ESMALL;
}

/* x: N x D canonical elements; maps / map_len / points (log2 map_len[k] elements each) / u (log2 D) */
int zko_reindex_prove(const uint8_t* x, uint64_t n, uint64_t d, int K, const int32_t* const* maps, const uint64_t* map_len,
                      const uint8_t* const* points, const uint8_t* u, int bind_statement, zko_ts* ts, uint8_t* proof,
                      uint64_t cap, uint64_t* proof_len) {
    init_mu();
    if (K < 1 || K > 8 || ilog2_u64(d) < 0) return ZKO_EARG;
    fe* xx = load_table(x, n * d);
    fe* uu = load_table(u, (uint64_t)ilog2_u64(d));
    fe* pp[8];
    const fe* cp[8];
    for (int k = 0; k < K; ++k) {
        int lm = ilog2_u64(map_len[k]);
        if (lm < 0) return ZKO_EARG;
        pp[k] = load_table(points[k], (uint64_t)lm);
        cp[k] = pp[k];
    }
    wbuf wb = {proof, (size_t)cap, 0};
    ri_info info;
    int rc = reindex_core(xx, n, d, K, maps, map_len, cp, uu, ts, bind_statement, &wb, &info);
    for (int k = 0; k < K; ++k) free(pp[k]);
    free(xx);
    free(uu);
    if (rc) return rc;
    *proof_len = wb.len;
    return wb.len <= wb.cap ? 0 : ZKO_ESMALL;
}

int zko_stack_merge_prove(const uint8_t* x, uint64_t n, uint64_t d, int K, const uint8_t* const* points, int bind_statement,
                          zko_ts* ts, uint8_t* proof, uint64_t cap, uint64_t* proof_len) {
    init_mu();
    int ln = ilog2_u64(n), ld = ilog2_u64(d);
    if (K < 1 || K > 8 || ln < 0 || ld < 0) return ZKO_EARG;
    fe* xx = load_table(x, n * d);
    fe* pp[8];
    const fe* cp[8];
    for (int k = 0; k < K; ++k) {
        pp[k] = load_table(points[k], (uint64_t)(ln + ld));
        cp[k] = pp[k];
    }
    wbuf wb = {proof, (size_t)cap, 0};
    ms_info info;
    int rc = stack_merge_core(xx, n, d, K, cp, ts, bind_statement, &wb, &info);
    for (int k = 0; k < K; ++k) free(pp[k]);
    free(xx);
    if (rc) return rc;
    *proof_len = wb.len;
    return wb.len <= wb.cap ? 0 : ZKO_ESMALL;
}

/* Proof of the parameter update (Sec. 5, Example FCNN, last item; the rounding by zkReLU, Sec. 3.1 and App. A),
 * the steps of the first tier's update_prove in the same order: header, p, Au = ReLU(rescale([G; -G])), the two
 * claims Au~(0, p), Au~(1, p), rho and u_Z, zkReLU at the given points u_A = (rho, p), u_Z. */
int zko_update_prove(const int64_t* gw, uint64_t D, int q, int rb, zko_ts* ts, uint8_t* proof, uint64_t cap,
                     uint64_t* proof_len) {
    init_mu();
    const int ld = ilog2_u64(D);
    if (ld < 0 || ld > 38 || !gw || !ts || q < 1 || rb < 1 || q + rb > 63) return ZKO_EARG;
    const int li = ld + 1;
    const int64_t lim = (int64_t)1 << (q + rb - 1), half = (int64_t)1 << (rb - 1);
    uint32_t hdr[3] = {(uint32_t)ld, (uint32_t)q, (uint32_t)rb};
    ts_absorb_u32(ts, "update", hdr, 3);
    fe p[40];
    ts_draw(ts, ld, p);
    int64_t* zu = (int64_t*)malloc(sizeof(int64_t) * 2 * D);
    fe* au = (fe*)malloc(sizeof(fe) * 2 * D);
    fe* bp = beta_table(p, ld);
    if (!zu || !au || !bp) {
        free(zu);
        free(au);
        free(bp);
        return ZKO_ENOMEM;
    }
    int rc = 0;
    for (uint64_t i = 0; i < D; ++i) {
        if (gw[i] <= -lim || gw[i] >= lim) rc = ZKO_ERANGE; /* -G must be in range as well */
        zu[i] = gw[i];
        zu[D + i] = -gw[i];
    }
    if (!rc) {
        for (uint64_t i = 0; i < 2 * D; ++i) {
            const int64_t zp = (zu[i] + half) >> rb; /* zkReLU's rescaling: round half up */
            au[i] = fe_from_u64(zp > 0 ? (uint64_t)zp : 0);
        }
        fe a[2];
        for (int k = 0; k < 2; ++k) { /* Au~(k, p) = sum_x beta~(p, x) Au[k, x] */
            fe acc = fe_from_u64(0);
            for (uint64_t x = 0; x < D; ++x) acc = fe_add(acc, fe_mul(bp[x], au[(uint64_t)k * D + x]));
            a[k] = acc;
        }
        ts_absorb_fe(ts, "c", a, 2);
        fe drawn[42];
        ts_draw(ts, 1 + li, drawn);
        wbuf wb = {proof, (size_t)cap, 0};
        wb_u32(&wb, 0x50554B5Au); /* "ZKUP" */
        wb_u32(&wb, (uint32_t)ld);
        wb_u32(&wb, (uint32_t)q);
        wb_u32(&wb, (uint32_t)rb);
        for (int k = 0; k < 4; ++k) wb_u32(&wb, 0);
        wb_fe(&wb, a[0]);
        wb_fe(&wb, a[1]);
        fe* four = (fe*)malloc(sizeof(fe) * 4 * (size_t)li);
        if (!four) rc = ZKO_ENOMEM;
        if (!rc) {
            for (int c = 0; c < li; ++c) four[c] = four[2 * li + c] = four[3 * li + c] = drawn[1 + c];
            four[li] = drawn[0];
            for (int c = 0; c < ld; ++c) four[li + 1 + c] = p[c];
            zk_info zi;
            rc = zkrelu_core(zu, 0, 2 * D, q, rb, ts, four, 0, &wb, &zi);
            free(four);
        }
        if (!rc) {
            *proof_len = wb.len;
            if (wb.len > wb.cap) rc = ZKO_ESMALL;
        }
    }
    free(zu);
    free(au);
    free(bp);
    return rc;
}

int zko_threads(void) { return max_threads(); }
