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

// lo + x * (hi - lo) evaluated along x = 0, 1, 2, 3 needs only additions:
// e(0) = lo, e(1) = hi, e(k+1) = e(k) + (hi - lo)
