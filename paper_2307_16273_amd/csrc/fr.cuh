// Arithmetic in the BLS12-381 scalar field Fr (the field F of Sec. 2.4 / Sec. 6)
// for gfx950.
//
// Storage: 8 x 32-bit limbs, little-endian, fully reduced, Montgomery form with
// R = 2^261.  Multiplication unpacks both operands into 9 limbs of 29 bits: a
// 29 x 29-bit product is below 2^58, so a whole column of the product (up to 9
// operand products and 9 reduction products) accumulates in one 64-bit register
// with plain v_mad_u64_u32 and no carry handling.  On gfx950 every VALU
// instruction issues at the same rate, v_mad_u64_u32 included, and a carry chain
// through VCC costs an extra instruction plus wait states per product, so the
// count of instructions decides: 153 multiply-adds and about 60 shifts/masks
// per product here against about 470 instructions for 8 x 32-bit limbs with
// explicit carries.  Because r = 1 (mod 2^32), r = 1 (mod 2^29) too: the
// Montgomery factor -r^{-1} mod 2^29 is all ones, the per-column multiplier is a
// negation and its product with the lowest limb of r is the multiplier itself.
//
// Every function is __host__ __device__ so that the host side of the library
// (constants, transcript, self-checks) runs the same arithmetic.
#pragma once
#include <stdint.h>
#include <hip/hip_runtime.h>

#define FR_HD __host__ __device__ __forceinline__

struct Fr {
    uint32_t v[8];
};

namespace frc {
// the modulus r
constexpr uint32_t MOD[8] = {0x00000001u, 0xffffffffu, 0xfffe5bfeu, 0x53bda402u,
                             0x09a1d805u, 0x3339d808u, 0x299d7d48u, 0x73eda753u};
// 2^261 mod r (Montgomery form of 1), 2^522 mod r, 2^778 mod r; re-derived by
// repeated modular doubling when a context is created (zkdl_selfcheck_constants)
constexpr uint32_t ONE[8] = {0xffffffbau, 0x00000045u, 0x0072d846u, 0x1a25272eu,
                             0x5dbeee8bu, 0xfe2eedcdu, 0x9eefbe41u, 0x4d043f42u};
constexpr uint32_t R2[8] = {0xca71b3c0u, 0x67a6440fu, 0x49d98f66u, 0xc44e2d5eu,
                            0xe8703b58u, 0x7ddc57c6u, 0x009cf20au, 0x27fd91b3u};
constexpr uint32_t W3[8] = {0x6dceb833u, 0xb06020dbu, 0xc7e29ae5u, 0xb06c02ccu,
                            0x3bae542du, 0x9217b092u, 0x413a7a64u, 0x0b29f00eu};
// r in 9 limbs of 29 bits
constexpr uint32_t MOD9[9] = {0x00000001u, 0x1ffffff8u, 0x1f96ffbfu, 0x1b4805ffu, 0x1d80553bu,
                              0x0c0404d0u, 0x1520cce7u, 0x0a6533afu, 0x0073eda7u};
constexpr uint32_t M29 = 0x1fffffffu;
// 4r with limbs 0..7 raised by borrowing from the limb above (same value): every
// limb is >= 2^29 - 1, the top one is top(4r) - 1, so C4R - b is limbwise
// non-negative for any normal b below 2.6 r
constexpr uint32_t C4R[9] = {0x20000004u, 0x3fffffdfu, 0x3e5bfefeu, 0x2d2017feu, 0x360154eeu,
                             0x30101342u, 0x3483339cu, 0x2994cebdu, 0x01cfb69cu};
}  // namespace frc

// 9 limbs of 29 bits; "normal" means every limb < 2^29
struct F9 {
    uint32_t v[9];
};

FR_HD Fr fr_zero() {
    Fr z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z.v[i] = 0;
    return z;
}

FR_HD Fr fr_const(const uint32_t (&c)[8]) {
    Fr z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z.v[i] = c[i];
    return z;
}

FR_HD Fr fr_one() { return fr_const(frc::ONE); }

FR_HD bool fr_is_zero(const Fr& a) {
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) o |= a.v[i];
    return o == 0;
}

FR_HD bool fr_eq(const Fr& a, const Fr& b) {
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) o |= a.v[i] ^ b.v[i];
    return o == 0;
}

// t - r if t >= r else t, for t < 2^256 (one subtraction suffices when t < 2r)
FR_HD Fr fr_cond_sub(const Fr& t) {
    Fr d;
    uint64_t br = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint64_t x = (uint64_t)t.v[i] - frc::MOD[i] - br;
        d.v[i] = (uint32_t)x;
        br = (x >> 32) & 1u;
    }
    Fr o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o.v[i] = br ? t.v[i] : d.v[i];
    return o;
}

// a + b mod r, a, b in [0, r)
FR_HD Fr fr_add(const Fr& a, const Fr& b) {
    Fr s;
    uint64_t c = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        c += (uint64_t)a.v[i] + b.v[i];
        s.v[i] = (uint32_t)c;
        c >>= 32;
    }
    return fr_cond_sub(s);  // a + b < 2r < 2^256: no carry out of the top limb
}

// a - b mod r
FR_HD Fr fr_sub(const Fr& a, const Fr& b) {
    Fr d;
    uint64_t br = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint64_t x = (uint64_t)a.v[i] - b.v[i] - br;
        d.v[i] = (uint32_t)x;
        br = (x >> 32) & 1u;
    }
    uint32_t mask = br ? 0xffffffffu : 0u;
    uint64_t c = 0;
    Fr o;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        c += (uint64_t)d.v[i] + (frc::MOD[i] & mask);
        o.v[i] = (uint32_t)c;
        c >>= 32;
    }
    return o;
}

FR_HD Fr fr_neg(const Fr& a) { return fr_sub(fr_zero(), a); }

FR_HD Fr fr_dbl(const Fr& a) { return fr_add(a, a); }

// 8 x 32 -> 9 x 29 (any 256-bit value; the top limb gets bits 232..255)
FR_HD F9 fr_unpack(const Fr& a) {
    F9 o;
#pragma unroll
    for (int i = 0; i < 9; ++i) {
        const int bit = 29 * i, w = bit >> 5, sh = bit & 31;
        uint32_t x = a.v[w] >> sh;
        if (sh > 3 && w + 1 < 8) x |= a.v[w + 1] << (32 - sh);
        o.v[i] = x & frc::M29;
    }
    return o;
}

// normal 9 x 29 with value < 2^256 -> 8 x 32; word w starts at bit 3w of limb w
FR_HD Fr fr_pack(const F9& t) {
    Fr o;
#pragma unroll
    for (int w = 0; w < 8; ++w) o.v[w] = (t.v[w] >> (3 * w)) | (t.v[w + 1] << (29 - 3 * w));
    return o;
}

// Montgomery product of two values in 29-bit limbs: (a * b + m * r) / 2^261.
// Limb bounds: (max limb of a) * (max limb of b) < 2^60.6.  The result is normal and
// below a * b / 2^261 + r.
FR_HD F9 f9_mul(const F9& a, const F9& b) {
    uint64_t acc = 0;
    uint32_t m[9];
    F9 t;
#pragma unroll
    for (int k = 0; k < 17; ++k) {
        const int lo_i = k < 9 ? 0 : k - 8, hi_i = k < 9 ? k : 8;
#pragma unroll
        for (int i = lo_i; i <= hi_i; ++i) acc += (uint64_t)a.v[i] * b.v[k - i];
#pragma unroll
        for (int i = lo_i; i <= hi_i; ++i)
            if (k - i >= 1) acc += (uint64_t)m[i] * frc::MOD9[k - i];
        if (k < 9) {
            m[k] = (0u - (uint32_t)acc) & frc::M29;   // m = -t * r^{-1} mod 2^29, r^{-1} = 1
            acc += m[k];                              // m * r[0], r[0] = 1: the low 29 bits vanish
        } else {
            t.v[k - 9] = (uint32_t)acc & frc::M29;
        }
        acc >>= 29;
    }
    t.v[8] = (uint32_t)acc;
    return t;
}

// t - r if t >= r else t, for a normal t < 2r
FR_HD F9 f9_cond_sub(const F9& t) {
    F9 d;
    int32_t c = 0;
#pragma unroll
    for (int i = 0; i < 9; ++i) {
        int32_t x = (int32_t)t.v[i] - (int32_t)frc::MOD9[i] + c;
        d.v[i] = (uint32_t)x & frc::M29;
        c = x >> 29;   // 0 or -1
    }
    // the top limb holds the sign: after the loop c < 0 iff t < r
    F9 o;
#pragma unroll
    for (int i = 0; i < 9; ++i) o.v[i] = c < 0 ? t.v[i] : d.v[i];
    return o;
}

// Montgomery product a * b / 2^261 mod r, fully reduced.
// Requires a < r; b may be any 256-bit value (a * b / 2^261 + r < 2r), which is
// what the wide reduction of hash output relies on.
FR_HD Fr fr_mul(const Fr& a, const Fr& b) {
    return fr_pack(f9_cond_sub(f9_mul(fr_unpack(a), fr_unpack(b))));
}

FR_HD Fr fr_sqr(const Fr& a) { return fr_mul(a, a); }

#if defined(__HIPCC__)
// Not inlined: for the single-wave transcript kernels, whose instructions run once per
// launch from a cold instruction cache, one shared copy of the multiplier is fetched once.
static __device__ __noinline__ Fr fr_mul_ni(Fr a, Fr b) { return fr_mul(a, b); }
__device__ inline Fr fr_from_mont_ni(const Fr& x) {
    Fr one = fr_zero();
    one.v[0] = 1;
    return fr_mul_ni(x, one);
}
#endif

// ---- lazy arithmetic on 29-bit limbs ---------------------------------------------
// Inside a kernel, values may stay unpacked between operations: limbs are u32 and may
// exceed 29 bits, values may exceed r.  Each function states what it needs; the
// invariants used by the kernels are written where they are relied upon.

// limbwise sum: limb and value bounds add
FR_HD F9 f9_add(const F9& a, const F9& b) {
    F9 o;
#pragma unroll
    for (int i = 0; i < 9; ++i) o.v[i] = a.v[i] + b.v[i];
    return o;
}

// a - b + 4r, limbwise and without borrows.  Needs b normal with value < 2.6 r.
// Limbs of the result are below (limb of a) + 2^30; its value is value(a) - value(b) + 4r.
FR_HD F9 f9_sub(const F9& a, const F9& b) {
    F9 o;
#pragma unroll
    for (int i = 0; i < 9; ++i) o.v[i] = a.v[i] + (frc::C4R[i] - b.v[i]);
    return o;
}

// carry propagation: same value, limbs 0..7 below 2^29
FR_HD F9 f9_norm(const F9& a) {
    F9 o;
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t x = a.v[i] + c;
        o.v[i] = x & frc::M29;
        c = x >> 29;
    }
    o.v[8] = a.v[8] + c;
    return o;
}

// carry propagation that also removes q = (top limb >> 23) <= floor(value / 2^255)
// multiples of r.  Needs limbs below 2^32 and value below 2^263.  The result is
// normal, congruent to a, non-negative, and below 2.41 r (q misses at most one
// multiple because of carries still pending below the top limb).
FR_HD F9 f9_norm_reduce(const F9& a) {
    F9 o;
    const int64_t q = (int64_t)(a.v[8] >> 23);
    int64_t c = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int64_t y = (int64_t)a.v[i] - q * (int64_t)frc::MOD9[i] + c;
        o.v[i] = (uint32_t)y & frc::M29;
        c = y >> 29;
    }
    o.v[8] = (uint32_t)((int64_t)a.v[8] - q * (int64_t)frc::MOD9[8] + c);
    return o;
}

// any lazy value (limbs < 2^32, value < 2^261) -> fully reduced packed form
FR_HD Fr f9_to_fr(const F9& a) {
    // multiply by the Montgomery form of 1: the product is congruent to a and below 2r
    return fr_pack(f9_cond_sub(f9_mul(fr_unpack(fr_const(frc::ONE)), f9_norm(a))));
}

// ---- wide accumulation: sum of many products, one Montgomery reduction at the end ----
// cols[k] collects the weight-2^(29k) terms of sum_n a_n * b_n (64-bit unsigned columns).

// cols += a * b for normal a, b: 81 multiply-adds, no carries.  Each column gains at most
// 9 * 2^58; renormalise (f9_cols_norm) after every fourth product.
FR_HD void f9_cols_mac(uint64_t cols[17], const F9& a, const F9& b) {
#pragma unroll
    for (int i = 0; i < 9; ++i)
#pragma unroll
        for (int j = 0; j < 9; ++j) cols[i + j] += (uint64_t)a.v[i] * b.v[j];
}

// cols += a * x for a normal a and a 32-bit unsigned x: nine multiply-adds into columns
// 0..8, each gaining below 2^61; renormalise after every fourth product.
FR_HD void f9_cols_mac_small(uint64_t cols[17], const F9& a, uint32_t x) {
#pragma unroll
    for (int i = 0; i < 9; ++i) cols[i] += (uint64_t)a.v[i] * x;
}

// carry propagation over the first n columns: same value, columns 0..n-2 below 2^29
template <int N>
FR_HD void f9_cols_norm(uint64_t cols[17]) {
#pragma unroll
    for (int k = 0; k + 1 < N; ++k) {
        cols[k + 1] += cols[k] >> 29;
        cols[k] &= frc::M29;
    }
}

// Montgomery reduction of a column sum: (V + m r) / 2^261 for V = sum_k cols[k] 2^(29k),
// columns below 2^62.  Normal result below V / 2^261 + r.
FR_HD F9 f9_redc(const uint64_t cols[17]) {
    uint64_t acc = 0;
    uint32_t m[9];
    F9 t;
#pragma unroll
    for (int k = 0; k < 17; ++k) {
        const int lo_i = k < 9 ? 0 : k - 8, hi_i = k < 9 ? k : 8;
        acc += cols[k];
#pragma unroll
        for (int i = lo_i; i <= hi_i; ++i)
            if (k - i >= 1) acc += (uint64_t)m[i] * frc::MOD9[k - i];
        if (k < 9) {
            m[k] = (0u - (uint32_t)acc) & frc::M29;
            acc += m[k];
        } else {
            t.v[k - 9] = (uint32_t)acc & frc::M29;
        }
        acc >>= 29;
    }
    t.v[8] = (uint32_t)acc;
    return t;
}

FR_HD F9 f9_zero() {
    F9 z;
#pragma unroll
    for (int i = 0; i < 9; ++i) z.v[i] = 0;
    return z;
}

// plain 256-bit value (any) -> Montgomery form of its residue
FR_HD Fr fr_to_mont(const Fr& x) { return fr_mul(fr_const(frc::R2), x); }

// Montgomery form -> canonical representative in [0, r)
FR_HD Fr fr_from_mont(const Fr& x) {
    Fr one = fr_zero();
    one.v[0] = 1;
    return fr_mul(x, one);
}

// signed 64-bit integer -> Montgomery form of (x mod r)
FR_HD Fr fr_from_i64(int64_t x) {
    uint64_t mag = x < 0 ? (uint64_t)0 - (uint64_t)x : (uint64_t)x;
    Fr p = fr_zero();
    p.v[0] = (uint32_t)mag;
    p.v[1] = (uint32_t)(mag >> 32);
    Fr m = fr_to_mont(p);
    return x < 0 ? fr_neg(m) : m;
}

// small non-negative integer -> Montgomery form
FR_HD Fr fr_from_u32(uint32_t x) {
    Fr p = fr_zero();
    p.v[0] = x;
    return fr_to_mont(p);
}

// lo + 2^256 * hi mod r, both halves arbitrary 256-bit values, to Montgomery form
FR_HD Fr fr_from_wide(const Fr& lo, const Fr& hi) {
    return fr_add(fr_mul(fr_const(frc::R2), lo), fr_mul(fr_const(frc::W3), hi));
}

// a^e for a 256-bit exponent given as limbs (host-side constants only)
FR_HD Fr fr_pow(const Fr& a, const uint32_t e[8]) {
    Fr acc = fr_one();
    for (int i = 255; i >= 0; --i) {
        acc = fr_sqr(acc);
        if ((e[i >> 5] >> (i & 31)) & 1u) acc = fr_mul(acc, a);
    }
    return acc;
}

// ---- structure-of-arrays tables: limb l of element i lives at p[l * ps + i] ----
struct FrTab {
    uint32_t* p;
    uint64_t ps;  // plane stride in elements
};

FR_HD Fr tab_ld(const FrTab& t, uint64_t i) {
    Fr x;
#pragma unroll
    for (int l = 0; l < 8; ++l) x.v[l] = t.p[l * t.ps + i];
    return x;
}

FR_HD void tab_st(const FrTab& t, uint64_t i, const Fr& x) {
#pragma unroll
    for (int l = 0; l < 8; ++l) t.p[l * t.ps + i] = x.v[l];
}

// tables of lazy values: nine planes of u32, limb l of element i at p[l * ps + i]
struct F9Tab {
    uint32_t* p;
    uint64_t ps;
};

FR_HD F9 f9tab_ld(const F9Tab& t, uint64_t i) {
    F9 x;
#pragma unroll
    for (int l = 0; l < 9; ++l) x.v[l] = t.p[l * t.ps + i];
    return x;
}

FR_HD void f9tab_st(const F9Tab& t, uint64_t i, const F9& x) {
#pragma unroll
    for (int l = 0; l < 9; ++l) t.p[l * t.ps + i] = x.v[l];
}
