// Arithmetic in the BLS12-381 scalar field Fr (the field F of Sec. 2.4 / Sec. 6)
// for gfx950: 8 x 32-bit limbs, little-endian, Montgomery form with R = 2^256.
//
// The 32x32+64 -> 64 multiply-adds below compile to v_mad_u64_u32.  Because
// r = 1 (mod 2^32), the Montgomery factor -r^{-1} mod 2^32 is 0xffffffff: the
// per-row multiplier is a negation and the product with the lowest limb of r is
// the multiplier itself.
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
// 2^256 mod r (Montgomery form of 1), 2^512 mod r, 2^768 mod r; re-derived by
// repeated modular doubling when a context is created (zkdl_selfcheck_constants)
constexpr uint32_t ONE[8] = {0xfffffffeu, 0x00000001u, 0x00034802u, 0x5884b7fau,
                             0xecbc4ff5u, 0x998c4fefu, 0xacc5056fu, 0x1824b159u};
constexpr uint32_t R2[8] = {0xf3f29c6du, 0xc999e990u, 0x87925c23u, 0x2b6cedcbu,
                            0x7254398fu, 0x05d31496u, 0x9f59ff11u, 0x0748d9d9u};
constexpr uint32_t R3[8] = {0x439b73afu, 0xc62c1807u, 0x8cf06990u, 0x1b3e0d18u,
                            0xc7b5f418u, 0x73d13c71u, 0xc8db33e9u, 0x6e2a5bb9u};
}  // namespace frc

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

// Montgomery product a * b / 2^256 mod r.
// Requires a < r; b may be any 256-bit value (the running value stays below
// a + r < 2r), which is what the wide reduction of hash output relies on.
FR_HD Fr fr_mul(const Fr& a, const Fr& b) {
    uint32_t t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = 0;
    uint32_t t8 = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // t += a * b[i]
        uint64_t c = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            c = (uint64_t)a.v[j] * b.v[i] + t[j] + c;
            t[j] = (uint32_t)c;
            c >>= 32;
        }
        uint64_t top = (uint64_t)t8 + c;  // < 2^33
        // t += m * r with m = -t[0] mod 2^32, then drop the (now zero) low limb
        uint32_t m = 0u - t[0];
        c = (t[0] != 0) ? 1u : 0u;        // carry of t[0] + m * r[0], r[0] = 1
#pragma unroll
        for (int j = 1; j < 8; ++j) {
            c = (uint64_t)m * frc::MOD[j] + t[j] + c;
            t[j - 1] = (uint32_t)c;
            c >>= 32;
        }
        top += c;
        t[7] = (uint32_t)top;
        t8 = (uint32_t)(top >> 32);
    }
    // t < 2r < 2^256, so t8 == 0 here
    Fr o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o.v[i] = t[i];
    return fr_cond_sub(o);
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
    return fr_add(fr_mul(fr_const(frc::R2), lo), fr_mul(fr_const(frc::R3), hi));
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
