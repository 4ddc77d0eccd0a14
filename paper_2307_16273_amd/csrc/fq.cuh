// Arithmetic in F_q, the base field of BLS12-381 (q has 381 bits), and the group law of G1,
// y^2 = x^3 + 4, for the Pedersen commitments of Sec. 2.3 (Sec. 6 names the curve).
//
// An element is a fully reduced residue in Montgomery form with R = 2^406, held as 14 limbs of
// 29 bits: as for the scalar field, a 29 x 29-bit product is below 2^58, so a whole column of a product
// (at most 14 operand and 13 reduction products) accumulates in one 64-bit register with plain
// v_mad_u64_u32 and no carry handling.  q is not 1 modulo 2^29, so each column costs one extra
// multiplication for the Montgomery factor.  Sums and differences are reduced at once (one conditional
// subtraction or addition of q, selected without a branch): every value a kernel holds is the unique
// representative below q.
//
// Points are in homogeneous projective coordinates (X : Y : Z), the identity (0 : 1 : 0), with the
// complete addition and doubling formulas for curves of j-invariant 0 (Renes, Costello, Batina,
// "Complete addition formulas for prime order elliptic curves", Algorithms 7 and 9 with b3 = 3 b = 12):
// no case distinction for equal, opposite or neutral operands, so lanes never diverge inside a sum.
#pragma once
#include <stdint.h>
#include <hip/hip_runtime.h>

#define FQ_HD __host__ __device__ __forceinline__

namespace fqc {
constexpr int L = 14;
constexpr uint32_t M29 = 0x1fffffffu;
// q in 29-bit limbs
constexpr uint32_t Q[L] = {0x1fffaaabu, 0x0ff7ffffu, 0x14ffffeeu, 0x17fffd62u, 0x0f6241eau, 0x09507b58u, 0x0afd9cc3u,
                           0x109e70a2u, 0x1764774bu, 0x121a5d66u, 0x12c6e9edu, 0x12ffcd34u, 0x00111ea3u, 0x0000000du};
constexpr uint32_t NINV = 0x1ffcfffdu;   // -q^{-1} mod 2^29
// 2^406 mod q (Montgomery form of 1) and 2^812 mod q; re-derived by modular doubling in fq_selfcheck
constexpr uint32_t ONE[L] = {0x03a9fb84u, 0x0ba00690u, 0x071288f1u, 0x0f59bcc5u, 0x126cb614u, 0x0585bf36u, 0x1b85ac3du,
                             0x1cf856fau, 0x1891ecbdu, 0x1a7eec05u, 0x155a88f0u, 0x0741ac6du, 0x1317c30fu, 0x00000009u};
constexpr uint32_t R2[L] = {0x15bef7aeu, 0x1031cd0eu, 0x02dd93e8u, 0x09226323u, 0x0e6e2cd2u, 0x11684daau, 0x1170e5dbu,
                            0x088e25b1u, 0x1b366399u, 0x1c536f47u, 0x0d1f9cbcu, 0x0278b67fu, 0x1ea66a2bu, 0x0000000cu};
// exponents as 32-bit words, least significant first: (q + 1) / 4 (square roots: q = 3 mod 4) and q - 2
constexpr uint32_t EXP_SQRT[12] = {0xffffeaabu, 0xee7fbfffu, 0xac54ffffu, 0x07aaffffu, 0x3dac3d89u, 0xd9cc34a8u,
                                   0x3ce144afu, 0xd91dd2e1u, 0x90d2eb35u, 0x92c6e9edu, 0x8e5ff9a6u, 0x0680447au};
constexpr uint32_t EXP_INV[12] = {0xffffaaa9u, 0xb9feffffu, 0xb153ffffu, 0x1eabfffeu, 0xf6b0f624u, 0x6730d2a0u,
                                  0xf38512bfu, 0x64774b84u, 0x434bacd7u, 0x4b1ba7b6u, 0x397fe69au, 0x1a0111eau};
// the cofactor of G1 (the curve has COFACTOR * r points)
constexpr uint32_t COFACTOR[4] = {0x0000aaabu, 0x8c00aaabu, 0x5555e156u, 0x396c8c00u};
}  // namespace fqc

struct Fq {
    uint32_t v[fqc::L];
};

FQ_HD Fq fq_zero() {
    Fq z;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) z.v[i] = 0;
    return z;
}

FQ_HD Fq fq_const(const uint32_t (&c)[fqc::L]) {
    Fq z;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) z.v[i] = c[i];
    return z;
}

FQ_HD Fq fq_one() { return fq_const(fqc::ONE); }

FQ_HD bool fq_is_zero(const Fq& a) {
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) o |= a.v[i];
    return o == 0;
}

FQ_HD bool fq_eq(const Fq& a, const Fq& b) {
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) o |= a.v[i] ^ b.v[i];
    return o == 0;
}

// t - q if t >= q else t, for normal limbs and t < 2q
FQ_HD Fq fq_cond_sub(const Fq& t) {
    Fq d;
    int32_t c = 0;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        int32_t x = (int32_t)t.v[i] - (int32_t)fqc::Q[i] + c;
        d.v[i] = (uint32_t)x & fqc::M29;
        c = x >> 29;   // 0 or -1
    }
    Fq o;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) o.v[i] = c < 0 ? t.v[i] : d.v[i];
    return o;
}

FQ_HD Fq fq_add(const Fq& a, const Fq& b) {
    Fq t;
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        uint32_t x = a.v[i] + b.v[i] + c;
        t.v[i] = i < fqc::L - 1 ? (x & fqc::M29) : x;   // the sum is below 2q < 2^382: the top limb holds it
        c = i < fqc::L - 1 ? (x >> 29) : 0;
    }
    return fq_cond_sub(t);
}

FQ_HD Fq fq_sub(const Fq& a, const Fq& b) {
    Fq d;
    int32_t c = 0;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        int32_t x = (int32_t)a.v[i] - (int32_t)b.v[i] + c;
        d.v[i] = (uint32_t)x & fqc::M29;
        c = x >> 29;
    }
    // c < 0: the difference is negative (its limbs hold it modulo 2^406): add q back
    Fq e;
    uint32_t k = 0;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        uint32_t x = d.v[i] + fqc::Q[i] + k;
        e.v[i] = x & fqc::M29;
        k = x >> 29;
    }
    Fq o;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) o.v[i] = c < 0 ? e.v[i] : d.v[i];
    return o;
}

FQ_HD Fq fq_neg(const Fq& a) { return fq_sub(fq_zero(), a); }

// Montgomery product a b / 2^406 mod q for operands with normal limbs and a b < q 2^406 (any a, b below 2^12 q):
// the value before the last step is below a b / 2^406 + q < 2q; REDUCE takes q off it if it is not below q
template <bool REDUCE>
FQ_HD Fq fq_mul_t(const Fq& a, const Fq& b) {
    uint64_t acc = 0;
    uint32_t m[fqc::L];
    Fq t;
#pragma unroll
    for (int k = 0; k < 2 * fqc::L - 1; ++k) {
        const int lo_i = k < fqc::L ? 0 : k - (fqc::L - 1), hi_i = k < fqc::L ? k : fqc::L - 1;
#pragma unroll
        for (int i = lo_i; i <= hi_i; ++i) acc += (uint64_t)a.v[i] * b.v[k - i];
#pragma unroll
        for (int i = lo_i; i <= hi_i; ++i)
            if (k - i >= 1) acc += (uint64_t)m[i] * fqc::Q[k - i];
        if (k < fqc::L) {
            m[k] = ((uint32_t)acc * fqc::NINV) & fqc::M29;   // makes the low 29 bits of the column vanish
            acc += (uint64_t)m[k] * fqc::Q[0];
        } else {
            t.v[k - fqc::L] = (uint32_t)acc & fqc::M29;
        }
        acc >>= 29;
    }
    t.v[fqc::L - 1] = (uint32_t)acc;
    return REDUCE ? fq_cond_sub(t) : t;
}

// fully reduced; a, b below q (or as above)
FQ_HD Fq fq_mul(const Fq& a, const Fq& b) { return fq_mul_t<true>(a, b); }

FQ_HD Fq fq_sqr(const Fq& a) { return fq_mul(a, a); }

// a^e, e given as `words` 32-bit words, least significant first
template <int WORDS>
FQ_HD Fq fq_pow(const Fq& a, const uint32_t (&e)[WORDS]) {
    Fq acc = fq_one();
    for (int w = WORDS - 1; w >= 0; --w)
        for (int bit = 31; bit >= 0; --bit) {
            acc = fq_sqr(acc);
            if ((e[w] >> bit) & 1u) acc = fq_mul(acc, a);
        }
    return acc;
}

FQ_HD Fq fq_inv(const Fq& a) { return fq_pow(a, fqc::EXP_INV); }

// ---- inversion by the binary Euclidean algorithm ---------------------------------------------------------------
// u = a, v = q (odd throughout).  One trip: if u is odd, the smaller of u, v is taken from the larger (u becomes the
// difference, v the smaller one); then u is halved.  Instead of halving a cofactor modulo q the other one is doubled
// (Kaliski's almost-inverse): with S, R >= 0 and a sign, a (sign S) = u 2^k and a (sign R) = -v 2^k modulo q after k
// halvings, and S v + R u = q bounds both by q.  At u = 0, v = 1: 1/a = -sign R / 2^k, with 381 <= k <= 762.
// About 270 trips of a few 12-word operations instead of the ~570 field products of a^(q-2).  The running time
// depends on the value: for public data only (commitments, the verifier).
namespace fqe {
constexpr int W = 12;
struct U384 {
    uint32_t w[W];
};

FQ_HD U384 from_limbs(const Fq& a) {   // normal limbs, value below 2^384
    U384 o;
#pragma unroll
    for (int j = 0; j < W; ++j) {
        uint64_t x = 0;
#pragma unroll
        for (int i = 0; i < fqc::L; ++i) {
            const int sh = 29 * i - 32 * j;   // limb i covers bits [29 i, 29 i + 29)
            if (sh > -29 && sh < 32) x |= sh >= 0 ? ((uint64_t)a.v[i] << sh) : ((uint64_t)a.v[i] >> (-sh));
        }
        o.w[j] = (uint32_t)x;
    }
    return o;
}

FQ_HD Fq to_limbs(const U384& a) {
    Fq o;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        const int bit = 29 * i, j = bit >> 5, sh = bit & 31;
        uint64_t x = a.w[j];
        if (j + 1 < W) x |= (uint64_t)a.w[j + 1] << 32;
        o.v[i] = (uint32_t)(x >> sh) & fqc::M29;
    }
    return o;
}
}  // namespace fqe

// 1/a in Montgomery form for a in Montgomery form (0 for 0)
FQ_HD Fq fq_inv_euclid(const Fq& a) {
    using fqe::U384;
    using fqe::W;
    U384 u = fqe::from_limbs(a), v = fqe::from_limbs(fq_const(fqc::Q)), S, R;
#pragma unroll
    for (int i = 0; i < W; ++i) S.w[i] = R.w[i] = 0;
    S.w[0] = 1;
    uint32_t flip = 0;
    int k = 0;
    for (;;) {
        const uint32_t odd = 0u - (u.w[0] & 1u);
        U384 d;
        uint32_t bor = 0;
#pragma unroll
        for (int i = 0; i < W; ++i) d.w[i] = __builtin_subc(u.w[i], v.w[i], bor, &bor);   // d = u - v modulo 2^384
        const uint32_t sw = odd & (0u - bor);   // u odd and below v: the roles change
        uint32_t c = sw & 1u;
#pragma unroll
        for (int i = 0; i < W; ++i) d.w[i] = __builtin_addc(d.w[i] ^ sw, 0u, c, &c);   // |u - v|
        c = 0;
        uint32_t any = 0;
#pragma unroll
        for (int i = 0; i < W; ++i) {
            v.w[i] = sw ? u.w[i] : v.w[i];
            u.w[i] = odd ? d.w[i] : u.w[i];
            any |= u.w[i];
            const uint32_t s_old = S.w[i], r_old = R.w[i];
            const uint32_t s_new = sw ? r_old : s_old, r_new = sw ? s_old : r_old;
            S.w[i] = __builtin_addc(s_new, r_new & odd, c, &c);   // S += R when u was odd
            R.w[i] = r_new;
        }
        flip ^= sw & 1u;
        if (any == 0) break;   // v = 1 now; R is not doubled any more (R u <= q bounds it only while u > 0)
        // u is even here (it was, or it is a difference of two odd numbers): all its low zero bits at once, at most 31
        const int tz = __builtin_ctz(u.w[0] | 0x80000000u);
#pragma unroll
        for (int i = 0; i < W; ++i) u.w[i] = (u.w[i] >> tz) | (i + 1 < W ? u.w[i + 1] << (32 - tz) : 0u);
#pragma unroll
        for (int i = W - 1; i >= 0; --i) R.w[i] = (R.w[i] << tz) | (i ? R.w[i - 1] >> (32 - tz) : 0u);
        k += tz;
    }
    // the limbs of a hold a_true 2^406, so 1/limbs = (1/a_true) 2^-406 = -sign R 2^-k, and the Montgomery form of
    // 1/a_true is -sign R 2^(812 - k): two products by single bits 2^e1 2^e2 = 2^(812 - k) (each takes 2^406 away)
    // and two by 2^812 (each puts 2^406 back)
    int e = 812 - k;
    if (e < 0) e = 0;   // not reached: k <= 762
    if (e > 810) e = 810;   // not reached for a != 0: k >= 381
    const int e1 = e < 405 ? e : 405, e2 = e - e1;
    Fq b1 = fq_zero(), b2 = fq_zero();
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        b1.v[i] = (e1 / 29 == i) ? (1u << (e1 % 29)) : 0u;
        b2.v[i] = (e2 / 29 == i) ? (1u << (e2 % 29)) : 0u;
    }
    const Fq r2 = fq_const(fqc::R2);
    Fq y = fq_mul(fqe::to_limbs(R), b1);   // R <= q as the first operand
    y = fq_mul(y, b2);
    y = fq_mul(fq_mul(y, r2), r2);
    return flip ? y : fq_neg(y);
}

// 48 little-endian bytes (any value below 2^384) -> normal limbs of the plain value
FQ_HD Fq fq_limbs_from_bytes(const uint8_t* p) {
    Fq o;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        uint64_t w = 0;
        const int bit = 29 * i, byte = bit >> 3, sh = bit & 7;
#pragma unroll
        for (int b = 0; b < 5; ++b)
            if (byte + b < 48) w |= (uint64_t)p[byte + b] << (8 * b);
        o.v[i] = (uint32_t)(w >> sh) & fqc::M29;
    }
    return o;
}

// plain value below q as 48 little-endian bytes
FQ_HD void fq_limbs_to_bytes(const Fq& a, uint8_t* p) {
    for (int b = 0; b < 48; ++b) p[b] = 0;
    for (int i = 0; i < fqc::L; ++i) {
        const int bit = 29 * i, byte = bit >> 3, sh = bit & 7;
        uint64_t w = (uint64_t)a.v[i] << sh;
        for (int b = 0; b < 5; ++b)
            if (byte + b < 48) p[byte + b] |= (uint8_t)(w >> (8 * b));
    }
}

FQ_HD Fq fq_to_mont(const Fq& plain) { return fq_mul(plain, fq_const(fqc::R2)); }   // plain below q

FQ_HD Fq fq_from_mont(const Fq& a) {
    Fq one = fq_zero();
    one.v[0] = 1;
    return fq_mul(a, one);
}

// a value below 2^384 given as normal limbs, reduced modulo q into Montgomery form: the Montgomery product
// with 2^812 tolerates any first operand whose limbs are normal (a b / R + q < 2q still holds for a < 2^406)
FQ_HD Fq fq_reduce_to_mont(const Fq& any) { return fq_mul(any, fq_const(fqc::R2)); }

// ---- G1 -------------------------------------------------------------------------------------------
struct G1 {
    Fq X, Y, Z;
};

FQ_HD G1 g1_identity() {
    G1 p;
    p.X = fq_zero();
    p.Y = fq_one();
    p.Z = fq_zero();
    return p;
}

FQ_HD Fq fq_mul12(const Fq& a) {   // b3 = 3 b = 12
    Fq t = fq_add(a, a);
    t = fq_add(t, a);
    t = fq_add(t, t);
    return fq_add(t, t);
}

// complete addition (Algorithm 7 of the reference above, a = 0); `mul` is the field product to use (the
// kernels that add points in a loop pass an out-of-line one: twelve inlined products are 60 KB of code)
template <class Mul>
FQ_HD G1 g1_add_with(const G1& p, const G1& q, Mul mul) {
    Fq t0 = mul(p.X, q.X), t1 = mul(p.Y, q.Y), t2 = mul(p.Z, q.Z);
    Fq t3 = mul(fq_add(p.X, p.Y), fq_add(q.X, q.Y));
    t3 = fq_sub(t3, fq_add(t0, t1));
    Fq t4 = mul(fq_add(p.Y, p.Z), fq_add(q.Y, q.Z));
    t4 = fq_sub(t4, fq_add(t1, t2));
    Fq y3 = mul(fq_add(p.X, p.Z), fq_add(q.X, q.Z));
    y3 = fq_sub(y3, fq_add(t0, t2));
    Fq x3 = fq_add(t0, t0);
    t0 = fq_add(x3, t0);
    t2 = fq_mul12(t2);
    Fq z3 = fq_add(t1, t2);
    t1 = fq_sub(t1, t2);
    y3 = fq_mul12(y3);
    x3 = mul(t4, y3);
    t2 = mul(t3, t1);
    x3 = fq_sub(t2, x3);
    y3 = mul(y3, t0);
    t1 = mul(t1, z3);
    y3 = fq_add(t1, y3);
    t0 = mul(t0, t3);
    z3 = mul(z3, t4);
    z3 = fq_add(z3, t0);
    G1 r;
    r.X = x3;
    r.Y = y3;
    r.Z = z3;
    return r;
}

struct FqMulInline {
    FQ_HD Fq operator()(const Fq& a, const Fq& b) const { return fq_mul(a, b); }
};

FQ_HD G1 g1_add(const G1& p, const G1& q) { return g1_add_with(p, q, FqMulInline()); }

// ---- the same addition without reductions ----------------------------------------------------------------------
// For long sums of points: coordinates are kept below 6q with normal limbs instead of below q.  Sums are carried but
// not reduced, differences are shifted by a multiple of q that is spread over the limbs so that no limb borrows,
// small multiples go through one carry pass, and the product skips its conditional subtraction (its result is
// below 2q for every pair of operands that occurs here: the largest product of bounds is 120q x 10q, far below
// q 2^406 / q = 2^25 q).  About a quarter fewer instructions per addition than with every value reduced.
namespace fqc {
struct Limbs {
    uint32_t v[L];
};
constexpr Limbs times_q(uint32_t k) {   // normal limbs of k q
    Limbs o{};
    uint64_t c = 0;
    for (int i = 0; i < L; ++i) {
        const uint64_t x = (uint64_t)Q[i] * k + c;
        o.v[i] = i < L - 1 ? (uint32_t)(x & M29) : (uint32_t)x;
        c = x >> 29;
    }
    return o;
}
// k q with 2^30 lent to every limb below the top one and taken back, as 2, from the limb above: two normal limbs can
// be taken from each of these limbs without a borrow
constexpr Limbs spread_q(uint32_t k) {
    Limbs o = times_q(k);
    for (int i = 0; i < L - 1; ++i) {
        o.v[i] += 1u << 30;
        o.v[i + 1] -= 2;
    }
    return o;
}
}  // namespace fqc

FQ_HD Fq fq_add_lazy(const Fq& a, const Fq& b) {
    Fq o;
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        const uint32_t x = a.v[i] + b.v[i] + c;
        o.v[i] = i < fqc::L - 1 ? (x & fqc::M29) : x;
        c = i < fqc::L - 1 ? (x >> 29) : 0;
    }
    return o;
}

// a - b - c + K q for b + c below SUB q (c may be zero); the result is below a + K q
template <uint32_t K, uint32_t SUB>
FQ_HD Fq fq_sub2_lazy(const Fq& a, const Fq& b, const Fq& c) {
    constexpr fqc::Limbs C = fqc::spread_q(K);
    static_assert(K >= SUB && C.v[fqc::L - 1] < (1u << 29) && C.v[fqc::L - 1] >= fqc::times_q(SUB).v[fqc::L - 1] + 1,
                  "the top limb of K q covers the top limbs taken from it");
    Fq o;
    uint32_t carry = 0;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        const uint32_t x = a.v[i] + C.v[i] - b.v[i] - c.v[i] + carry;
        o.v[i] = i < fqc::L - 1 ? (x & fqc::M29) : x;
        carry = i < fqc::L - 1 ? (x >> 29) : 0;
    }
    return o;
}

template <uint32_t K>
FQ_HD Fq fq_times_lazy(const Fq& a) {   // K a, K small
    Fq o;
    uint64_t c = 0;
#pragma unroll
    for (int i = 0; i < fqc::L; ++i) {
        const uint64_t x = (uint64_t)a.v[i] * K + c;
        o.v[i] = i < fqc::L - 1 ? ((uint32_t)x & fqc::M29) : (uint32_t)x;
        c = x >> 29;
    }
    return o;
}

// p + q for coordinates below 6q (normal limbs); the result's are below 6q again.  `mul` is the product WITHOUT the
// conditional subtraction (results below 2q).
template <class Mul>
FQ_HD G1 g1_add_lazy_with(const G1& p, const G1& q, Mul mul) {
    const Fq zero = fq_zero();
    const Fq t0 = mul(p.X, q.X), t1 = mul(p.Y, q.Y), t2 = mul(p.Z, q.Z);                 // below 2q
    const Fq p3 = mul(fq_add_lazy(p.X, p.Y), fq_add_lazy(q.X, q.Y));                      // 12q x 12q
    const Fq p4 = mul(fq_add_lazy(p.Y, p.Z), fq_add_lazy(q.Y, q.Z));
    const Fq p5 = mul(fq_add_lazy(p.X, p.Z), fq_add_lazy(q.X, q.Z));
    const Fq t3 = fq_sub2_lazy<8, 4>(p3, t0, t1);                                         // X1Y2 + X2Y1, in (4q, 10q)
    const Fq t4 = fq_sub2_lazy<8, 4>(p4, t1, t2);                                         // Y1Z2 + Y2Z1
    const Fq y3 = fq_times_lazy<12>(fq_sub2_lazy<8, 4>(p5, t0, t2));                      // 12 (X1Z2 + X2Z1), below 120q
    const Fq x3 = fq_times_lazy<3>(t0);                                                   // below 6q
    const Fq t2b = fq_times_lazy<12>(t2);                                                 // below 24q
    const Fq z3 = fq_add_lazy(t1, t2b);                                                   // below 26q
    const Fq t1b = fq_sub2_lazy<32, 24>(t1, t2b, zero);                                   // in (8q, 34q)
    G1 r;
    r.X = fq_sub2_lazy<4, 2>(mul(t3, t1b), mul(t4, y3), zero);                            // below 6q
    r.Y = fq_add_lazy(mul(t1b, z3), mul(y3, x3));                                         // below 4q
    r.Z = fq_add_lazy(mul(z3, t4), mul(x3, t3));
    return r;
}

// The same with the second point affine (x2, y2; never the identity; x2 below q, y2 at most 2q): eleven products
// (Algorithm 8 of the same reference, a = 0).
template <class Mul>
FQ_HD G1 g1_add_mixed_lazy_with(const G1& p, const Fq& x2, const Fq& y2, Mul mul) {
    const Fq zero = fq_zero();
    const Fq t0 = mul(p.X, x2), t1 = mul(p.Y, y2);                                        // below 2q
    const Fq p3 = mul(fq_add_lazy(p.X, p.Y), fq_add_lazy(x2, y2));                        // 12q x 3q
    const Fq t3 = fq_sub2_lazy<8, 4>(p3, t0, t1);                                         // X1 y2 + x2 Y1, in (4q, 10q)
    const Fq t4 = fq_add_lazy(mul(y2, p.Z), p.Y);                                         // y2 Z1 + Y1, below 8q
    const Fq y3 = fq_times_lazy<12>(fq_add_lazy(mul(x2, p.Z), p.X));                      // 12 (x2 Z1 + X1), below 96q
    const Fq x3 = fq_times_lazy<3>(t0);                                                   // below 6q
    const Fq t2b = fq_times_lazy<12>(p.Z);                                                // below 72q
    const Fq z3 = fq_add_lazy(t1, t2b);                                                   // below 74q
    const Fq t1b = fq_sub2_lazy<80, 72>(t1, t2b, zero);                                   // in (8q, 82q)
    G1 r;
    r.X = fq_sub2_lazy<4, 2>(mul(t3, t1b), mul(t4, y3), zero);                            // below 6q
    r.Y = fq_add_lazy(mul(t1b, z3), mul(y3, x3));                                         // below 4q
    r.Z = fq_add_lazy(mul(z3, t4), mul(x3, t3));
    return r;
}

struct FqMulLazyInline {
    FQ_HD Fq operator()(const Fq& a, const Fq& b) const { return fq_mul_t<false>(a, b); }
};

// coordinates with normal limbs, any value below 2^12 q -> below q
FQ_HD G1 g1_reduce(const G1& p) {
    G1 r;
    r.X = fq_mul(p.X, fq_one());
    r.Y = fq_mul(p.Y, fq_one());
    r.Z = fq_mul(p.Z, fq_one());
    return r;
}

// doubling (Algorithm 9, a = 0)
template <class Mul>
FQ_HD G1 g1_dbl_with(const G1& p, Mul mul) {
    Fq t0 = mul(p.Y, p.Y);
    Fq z3 = fq_add(t0, t0);
    z3 = fq_add(z3, z3);
    z3 = fq_add(z3, z3);
    Fq t1 = mul(p.Y, p.Z);
    Fq t2 = fq_mul12(mul(p.Z, p.Z));
    Fq x3 = mul(t2, z3);
    Fq y3 = fq_add(t0, t2);
    z3 = mul(t1, z3);
    t1 = fq_add(t2, t2);
    t2 = fq_add(t1, t2);
    t0 = fq_sub(t0, t2);
    y3 = mul(t0, y3);
    y3 = fq_add(x3, y3);
    t1 = mul(p.X, p.Y);
    x3 = mul(t0, t1);
    x3 = fq_add(x3, x3);
    G1 r;
    r.X = x3;
    r.Y = y3;
    r.Z = z3;
    return r;
}

FQ_HD G1 g1_dbl(const G1& p) { return g1_dbl_with(p, FqMulInline()); }

FQ_HD G1 g1_neg(const G1& p) {
    G1 r = p;
    r.Y = fq_neg(p.Y);
    return r;
}

// k P for a scalar of `WORDS` 32-bit words (least significant first), double-and-add from the top bit
template <int WORDS>
FQ_HD G1 g1_mul_words(const G1& p, const uint32_t (&k)[WORDS]) {
    G1 acc = g1_identity();
    for (int w = WORDS - 1; w >= 0; --w)
        for (int bit = 31; bit >= 0; --bit) {
            acc = g1_dbl(acc);
            if ((k[w] >> bit) & 1u) acc = g1_add(acc, p);
        }
    return acc;
}

// affine (x, y) as 2 x 48 little-endian bytes of the plain values; the identity as 96 zero bytes
FQ_HD void g1_to_bytes(const G1& p, uint8_t* out) {
    if (fq_is_zero(p.Z)) {
        for (int b = 0; b < 96; ++b) out[b] = 0;
        return;
    }
    const Fq zi = fq_inv_euclid(p.Z);
    fq_limbs_to_bytes(fq_from_mont(fq_mul(p.X, zi)), out);
    fq_limbs_to_bytes(fq_from_mont(fq_mul(p.Y, zi)), out + 48);
}
