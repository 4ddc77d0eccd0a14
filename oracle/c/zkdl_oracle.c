/* zkdl_oracle.c - second tier of the CPU oracle: the product sumcheck and the
 * multilinear-extension partial evaluation in plain C, for inputs too large for the
 * Python-integer tier (the 2^24-entry kernel micro-benchmark).
 *
 * Test infrastructure: used by tests, the smoke check and the benchmark's CPU baseline only,
 * never by the product.  It shares no code with the HIP library: field elements are canonical
 * (no Montgomery form) in four 64-bit limbs, products are schoolbook 4 x 4 with unsigned
 * __int128 and reduced with Barrett's method exactly as in the Handbook of Applied
 * Cryptography, Alg. 14.42 (b = 2^64, k = 4), SHA-256 is written from FIPS 180-4.
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

static uint64_t mp_add(uint64_t* a, const uint64_t* b, int n) { /* a += b, returns carry */
    uint64_t carry = 0;
    for (int i = 0; i < n; ++i) {
        u128 s = (u128)a[i] + b[i] + carry;
        a[i] = (uint64_t)s;
        carry = (uint64_t)(s >> 64);
    }
    return carry;
}

static void mp_mul(const uint64_t* a, int na, const uint64_t* b, int nb, uint64_t* out) { /* out: na + nb limbs */
    memset(out, 0, sizeof(uint64_t) * (size_t)(na + nb));
    for (int i = 0; i < na; ++i) {
        uint64_t carry = 0;
        for (int j = 0; j < nb; ++j) {
            u128 t = (u128)a[i] * b[j] + out[i + j] + carry;
            out[i + j] = (uint64_t)t;
            carry = (uint64_t)(t >> 64);
        }
        out[i + nb] = carry;
    }
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

/* x (8 limbs, any value below 2^512) mod r: HAC Alg. 14.42 with b = 2^64, k = 4 */
static fe reduce512(const uint64_t x[8]) {
    uint64_t q2[10], r2[10], r1[5];
    mp_mul(x + 3, 5, MU, 5, q2);        /* q1 = floor(x / b^(k-1)); q2 = q1 mu */
    const uint64_t* q3 = q2 + 5;        /* q3 = floor(q2 / b^(k+1)) */
    uint64_t m5[5] = {MOD[0], MOD[1], MOD[2], MOD[3], 0};
    mp_mul(q3, 5, m5, 5, r2);           /* r2 = q3 m, low k+1 limbs used */
    for (int i = 0; i < 5; ++i) r1[i] = x[i];
    mp_sub(r1, r2, 5);                  /* r = r1 - r2 mod b^(k+1): the wrap-around is the "+ b^(k+1)" step */
    while (mp_cmp(r1, m5, 5) >= 0) mp_sub(r1, m5, 5);
    fe o = {{r1[0], r1[1], r1[2], r1[3]}};
    return o;
}

static fe fe_mul(fe a, fe b) {
    uint64_t p[8];
    mp_mul(a.l, 4, b.l, 4, p);
    return reduce512(p);
}

static fe fe_add(fe a, fe b) {
    uint64_t carry = mp_add(a.l, b.l, 4);
    if (carry || mp_cmp(a.l, MOD, 4) >= 0) mp_sub(a.l, MOD, 4);
    return a;
}

static fe fe_sub(fe a, fe b) {
    if (mp_sub(a.l, b.l, 4)) mp_add(a.l, MOD, 4);
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

int zko_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
