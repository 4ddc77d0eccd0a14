// SHA-256 (FIPS 180-4) and the Fiat-Shamir transcript built on it, usable from
// host code and from a single GPU thread.
//
// The paper's verifier sends a uniform field element after each round
// polynomial (App. B); the transcript replaces that message by a hash.  The
// transcript is one byte stream:
//   stream_0         = "zkdl-mi355x/v3" zero-padded to 56 bytes || u64le(seed)
//   absorb(label, m) : stream <- stream || u8(|label|) || label || u64le(|m|) || m
//   challenges(n)    : for i < n: d0 = SHA256(stream || 0xF0 || u32le(i)),
//                      d1 = SHA256(stream || 0xF1 || u32le(i)), c_i = int_le(d0 || d1) mod r;
//                      then stream <- stream || 0xF2 || zero bytes up to the next multiple of 64.
//                      challenge() = challenges(1)[0].
//   digest()         = SHA256(stream)
// The state is the SHA-256 chaining value after the last whole block, the block count and the
// bytes of the unfinished block.  After a draw the stream is block-aligned, so a sumcheck round
// (a 106-byte frame, then one challenge) is one compression for the frame's first 64 bytes and
// then three independent ones from that chaining value: the two hashes of the draw (last block:
// the other 42 bytes, tag, index, padding, bit length) and the block that extends the stream.
// No message schedule depends on a chaining value, so they are all computed beforehand, in
// other lanes than the one that runs the rounds.
#pragma once
#include <stdint.h>
#include <hip/hip_runtime.h>
#include "fr.cuh"

#define SHA_HD __host__ __device__ inline

namespace sha {

SHA_HD uint32_t rotr(uint32_t x, int n) { return (x >> n) | (x << (32 - n)); }

SHA_HD uint32_t kconst(int i) {
    constexpr uint32_t K[64] = {
        0x428a2f98, 0x71374491, 0xb5c0fbcf, 0xe9b5dba5, 0x3956c25b, 0x59f111f1, 0x923f82a4, 0xab1c5ed5,
        0xd807aa98, 0x12835b01, 0x243185be, 0x550c7dc3, 0x72be5d74, 0x80deb1fe, 0x9bdc06a7, 0xc19bf174,
        0xe49b69c1, 0xefbe4786, 0x0fc19dc6, 0x240ca1cc, 0x2de92c6f, 0x4a7484aa, 0x5cb0a9dc, 0x76f988da,
        0x983e5152, 0xa831c66d, 0xb00327c8, 0xbf597fc7, 0xc6e00bf3, 0xd5a79147, 0x06ca6351, 0x14292967,
        0x27b70a85, 0x2e1b2138, 0x4d2c6dfc, 0x53380d13, 0x650a7354, 0x766a0abb, 0x81c2c92e, 0x92722c85,
        0xa2bfe8a1, 0xa81a664b, 0xc24b8b70, 0xc76c51a3, 0xd192e819, 0xd6990624, 0xf40e3585, 0x106aa070,
        0x19a4c116, 0x1e376c08, 0x2748774c, 0x34b0bcb5, 0x391c0cb3, 0x4ed8aa4a, 0x5b9cca4f, 0x682e6ff3,
        0x748f82ee, 0x78a5636f, 0x84c87814, 0x8cc70208, 0x90befffa, 0xa4506ceb, 0xbef9a3f7, 0xc67178f2};
    return K[i];
}

// Message schedule with the round constants folded in: wk[t] = W[t] + K[t].  It does not
// depend on the chaining value, so on the GPU it runs in other lanes than the rounds.
SHA_HD void schedule_wk(const uint32_t w_in[16], uint32_t wk[64]) {
    uint32_t w[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) w[i] = w_in[i];
#pragma unroll
    for (int i = 0; i < 64; ++i) {
        if (i >= 16) {
            uint32_t w15 = w[(i + 1) & 15], w2 = w[(i + 14) & 15];
            uint32_t s0 = rotr(w15, 7) ^ rotr(w15, 18) ^ (w15 >> 3);
            uint32_t s1 = rotr(w2, 17) ^ rotr(w2, 19) ^ (w2 >> 10);
            w[i & 15] = w[i & 15] + s0 + w[(i + 9) & 15] + s1;
        }
        wk[i] = w[i & 15] + kconst(i);
    }
}

// the 64 rounds on a prepared schedule
SHA_HD void rounds(uint32_t h[8], const uint32_t wk[64]) {
    uint32_t a = h[0], b = h[1], c = h[2], d = h[3], e = h[4], f = h[5], g = h[6], hh = h[7];
#pragma unroll
    for (int i = 0; i < 64; ++i) {
        uint32_t S1 = rotr(e, 6) ^ rotr(e, 11) ^ rotr(e, 25);
        uint32_t ch = (e & f) | (~e & g);              // bit select: v_bfi_b32
        uint32_t t1 = hh + S1 + ch + wk[i];
        uint32_t S0 = rotr(a, 2) ^ rotr(a, 13) ^ rotr(a, 22);
        uint32_t ab = a ^ b;
        uint32_t mj = (ab & c) | (~ab & b);            // majority as a bit select
        hh = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + S0 + mj;
    }
    h[0] += a; h[1] += b; h[2] += c; h[3] += d; h[4] += e; h[5] += f; h[6] += g; h[7] += hh;
}

// one compression of a 64-byte block given as 16 big-endian words
SHA_HD void compress(uint32_t h[8], uint32_t w[16]) {
    uint32_t wk[64];
    schedule_wk(w, wk);
    rounds(h, wk);
}

#if defined(__HIPCC__)
// Compact device versions for the single-wave transcript steps.  Those steps execute
// every instruction once per launch, from a cold instruction cache, so code bytes cost as
// much as instructions: the bodies below are loops of 16 rounds and are not inlined.
struct Words8 {
    uint32_t v[8];
};
struct Words16 {
    uint32_t v[16];
};

static __device__ const uint32_t K_TABLE[64] = {
    0x428a2f98, 0x71374491, 0xb5c0fbcf, 0xe9b5dba5, 0x3956c25b, 0x59f111f1, 0x923f82a4, 0xab1c5ed5,
    0xd807aa98, 0x12835b01, 0x243185be, 0x550c7dc3, 0x72be5d74, 0x80deb1fe, 0x9bdc06a7, 0xc19bf174,
    0xe49b69c1, 0xefbe4786, 0x0fc19dc6, 0x240ca1cc, 0x2de92c6f, 0x4a7484aa, 0x5cb0a9dc, 0x76f988da,
    0x983e5152, 0xa831c66d, 0xb00327c8, 0xbf597fc7, 0xc6e00bf3, 0xd5a79147, 0x06ca6351, 0x14292967,
    0x27b70a85, 0x2e1b2138, 0x4d2c6dfc, 0x53380d13, 0x650a7354, 0x766a0abb, 0x81c2c92e, 0x92722c85,
    0xa2bfe8a1, 0xa81a664b, 0xc24b8b70, 0xc76c51a3, 0xd192e819, 0xd6990624, 0xf40e3585, 0x106aa070,
    0x19a4c116, 0x1e376c08, 0x2748774c, 0x34b0bcb5, 0x391c0cb3, 0x4ed8aa4a, 0x5b9cca4f, 0x682e6ff3,
    0x748f82ee, 0x78a5636f, 0x84c87814, 0x8cc70208, 0x90befffa, 0xa4506ceb, 0xbef9a3f7, 0xc67178f2};

// three-input bit operations in one instruction (truth table in the immediate)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}
__device__ __forceinline__ uint32_t choose(uint32_t e, uint32_t f, uint32_t g) {   // e ? f : g
    return __builtin_amdgcn_bitop3_b32(e, f, g, 0xCA);
}
__device__ __forceinline__ uint32_t majority(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0xE8);
}
__device__ __forceinline__ uint32_t big_sigma1(uint32_t e) { return xor3(rotr(e, 6), rotr(e, 11), rotr(e, 25)); }
__device__ __forceinline__ uint32_t big_sigma0(uint32_t a) { return xor3(rotr(a, 2), rotr(a, 13), rotr(a, 22)); }
__device__ __forceinline__ uint32_t small_sigma0(uint32_t w) { return xor3(rotr(w, 7), rotr(w, 18), w >> 3); }
__device__ __forceinline__ uint32_t small_sigma1(uint32_t w) { return xor3(rotr(w, 17), rotr(w, 19), w >> 10); }

typedef __attribute__((address_space(3))) uint32_t* lds_u32_ptr;
typedef const __attribute__((address_space(3))) uint32_t* lds_u32_cptr;

static __device__ __noinline__ Words8 compress_ni(Words8 hin, Words16 win) {
    uint32_t w[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) w[i] = win.v[i];
    uint32_t a = hin.v[0], b = hin.v[1], c = hin.v[2], d = hin.v[3], e = hin.v[4], f = hin.v[5],
             g = hin.v[6], hh = hin.v[7];
#pragma unroll 1
    for (int r = 0; r < 4; ++r) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (r > 0) w[i] = w[i] + small_sigma0(w[(i + 1) & 15]) + w[(i + 9) & 15] + small_sigma1(w[(i + 14) & 15]);
            uint32_t t1 = hh + big_sigma1(e) + choose(e, f, g) + K_TABLE[16 * r + i] + w[i];
            uint32_t t2 = big_sigma0(a) + majority(a, b, c);
            hh = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + t2;
        }
    }
    Words8 o;
    o.v[0] = hin.v[0] + a; o.v[1] = hin.v[1] + b; o.v[2] = hin.v[2] + c; o.v[3] = hin.v[3] + d;
    o.v[4] = hin.v[4] + e; o.v[5] = hin.v[5] + f; o.v[6] = hin.v[6] + g; o.v[7] = hin.v[7] + hh;
    return o;
}

__device__ inline Words8 iv_words() {
    Words8 h = {{0x6a09e667, 0xbb67ae85, 0x3c6ef372, 0xa54ff53a, 0x510e527f, 0x9b05688c, 0x1f83d9ab,
                 0x5be0cd19}};
    return h;
}

// wk[0..64) = W[t] + K[t] of one block, written to LDS; compact (one 16-step loop body)
static __device__ __noinline__ void schedule_wk_lds(Words16 win, lds_u32_ptr wk) {
    uint32_t w[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        w[i] = win.v[i];
        wk[i] = w[i] + K_TABLE[i];
    }
#pragma unroll 1
    for (int r = 1; r < 4; ++r) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            w[i] = w[i] + small_sigma0(w[(i + 1) & 15]) + w[(i + 9) & 15] + small_sigma1(w[(i + 14) & 15]);
            wk[16 * r + i] = w[i] + K_TABLE[16 * r + i];
        }
    }
}

// the 64 rounds on a schedule prepared in LDS; compact (one 8-round loop body); the
// next eight schedule words are fetched while the current eight rounds run
static __device__ __noinline__ Words8 rounds_lds(Words8 hin, lds_u32_cptr wk) {
    uint32_t a = hin.v[0], b = hin.v[1], c = hin.v[2], d = hin.v[3], e = hin.v[4], f = hin.v[5],
             g = hin.v[6], hh = hin.v[7];
    uint32_t x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = wk[i];
#pragma unroll 1
    for (int r = 0; r < 8; ++r) {
        uint32_t nx[8];
        const int nr = (r + 1) & 7;   // the last fetch wraps to the first words and is dropped
#pragma unroll
        for (int i = 0; i < 8; ++i) nx[i] = wk[8 * nr + i];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t t1 = hh + big_sigma1(e) + choose(e, f, g) + x[i];
            uint32_t t2 = big_sigma0(a) + majority(a, b, c);
            hh = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + t2;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = nx[i];
    }
    Words8 o;
    o.v[0] = hin.v[0] + a; o.v[1] = hin.v[1] + b; o.v[2] = hin.v[2] + c; o.v[3] = hin.v[3] + d;
    o.v[4] = hin.v[4] + e; o.v[5] = hin.v[5] + f; o.v[6] = hin.v[6] + g; o.v[7] = hin.v[7] + hh;
    return o;
}

#endif

SHA_HD uint32_t bswap32(uint32_t x) {
    return (x >> 24) | ((x >> 8) & 0xff00u) | ((x << 8) & 0xff0000u) | (x << 24);
}

SHA_HD void bytes_to_words(const uint8_t b[32], uint32_t w[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
        w[i] = ((uint32_t)b[4 * i] << 24) | ((uint32_t)b[4 * i + 1] << 16) | ((uint32_t)b[4 * i + 2] << 8) | b[4 * i + 3];
}

SHA_HD void words_to_bytes(const uint32_t w[8], uint8_t b[32]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        b[4 * i] = (uint8_t)(w[i] >> 24);
        b[4 * i + 1] = (uint8_t)(w[i] >> 16);
        b[4 * i + 2] = (uint8_t)(w[i] >> 8);
        b[4 * i + 3] = (uint8_t)w[i];
    }
}

}  // namespace sha

namespace ts {

constexpr uint32_t MAX_LABEL = 32;

// chaining value after the last whole block of the stream, the number of whole blocks, and
// the bytes of the unfinished block
struct State {
    uint32_t h[8];
    uint64_t nblk;
    uint8_t buf[64];
    uint32_t fill;
};

SHA_HD void compress_bytes(uint32_t h[8], const uint8_t blk[64]) {
    uint32_t w[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint8_t* p = blk + 4 * i;
        w[i] = ((uint32_t)p[0] << 24) | ((uint32_t)p[1] << 16) | ((uint32_t)p[2] << 8) | p[3];
    }
    sha::compress(h, w);
}

SHA_HD void push_byte(State& s, uint8_t b) {
    s.buf[s.fill++] = b;
    if (s.fill == 64) {
        compress_bytes(s.h, s.buf);
        s.nblk += 1;
        s.fill = 0;
    }
}

SHA_HD void init(State& s, uint64_t seed) {
    const uint32_t iv[8] = {0x6a09e667, 0xbb67ae85, 0x3c6ef372, 0xa54ff53a,
                            0x510e527f, 0x9b05688c, 0x1f83d9ab, 0x5be0cd19};
    for (int i = 0; i < 8; ++i) s.h[i] = iv[i];
    s.nblk = 0;
    s.fill = 0;
    const char dom[] = "zkdl-mi355x/v3";
    for (int i = 0; i < 56; ++i) push_byte(s, i < (int)sizeof(dom) - 1 ? (uint8_t)dom[i] : 0);
    for (int i = 0; i < 8; ++i) push_byte(s, (uint8_t)(seed >> (8 * i)));
}

// stream <- stream || u8(label_len) || label || u64le(n) || data
SHA_HD void absorb(State& s, const char* label, uint32_t label_len, const uint8_t* data, uint64_t n) {
    push_byte(s, (uint8_t)label_len);
    for (uint32_t i = 0; i < label_len; ++i) push_byte(s, (uint8_t)label[i]);
    for (int i = 0; i < 8; ++i) push_byte(s, (uint8_t)(n >> (8 * i)));
    for (uint64_t i = 0; i < n; ++i) push_byte(s, data[i]);
}

// SHA256(stream || tail), tail of at most 8 bytes, as big-endian words
SHA_HD void tail_digest_w(const State& s, const uint8_t* tail, uint32_t tail_len, uint32_t out[8]) {
    State f = s;
    const uint64_t bits = (s.nblk * 64 + s.fill + tail_len) * 8;
    for (uint32_t i = 0; i < tail_len; ++i) push_byte(f, tail[i]);
    push_byte(f, 0x80);
    while (f.fill != 56) push_byte(f, 0);
    for (int i = 7; i >= 0; --i) push_byte(f, (uint8_t)(bits >> (8 * i)));
    for (int i = 0; i < 8; ++i) out[i] = f.h[i];
}

// element idx of a draw (Montgomery form)
SHA_HD Fr challenge_elem(const State& s, uint32_t idx) {
    uint32_t d[2][8];
    for (uint32_t j = 0; j < 2; ++j) {
        const uint8_t tail[5] = {(uint8_t)(0xF0 + j), (uint8_t)idx, (uint8_t)(idx >> 8), (uint8_t)(idx >> 16),
                                 (uint8_t)(idx >> 24)};
        tail_digest_w(s, tail, 5, d[j]);
    }
    Fr lo, hi;
#pragma unroll
    for (int l = 0; l < 8; ++l) {
        lo.v[l] = sha::bswap32(d[0][l]);   // little-endian limbs of the digest bytes
        hi.v[l] = sha::bswap32(d[1][l]);
    }
    return fr_from_wide(lo, hi);
}

// the stream extension that follows a draw: 0xF2, then zeros up to the block boundary
SHA_HD void ratchet(State& s) {
    push_byte(s, 0xF2);
    while (s.fill != 0) push_byte(s, 0);
}

// canonical little-endian bytes of a Montgomery-form element
SHA_HD void fr_to_le(const Fr& mont, uint8_t out[32]) {
    Fr plain = fr_from_mont(mont);
#pragma unroll
    for (int l = 0; l < 8; ++l) {
        out[4 * l] = (uint8_t)plain.v[l];
        out[4 * l + 1] = (uint8_t)(plain.v[l] >> 8);
        out[4 * l + 2] = (uint8_t)(plain.v[l] >> 16);
        out[4 * l + 3] = (uint8_t)(plain.v[l] >> 24);
    }
}

// draw one challenge; returns it in Montgomery form and, if le_out != nullptr,
// as 32 canonical little-endian bytes
SHA_HD Fr challenge(State& s, uint8_t* le_out) {
    Fr c = challenge_elem(s, 0);
    ratchet(s);
    if (le_out) fr_to_le(c, le_out);
    return c;
}

SHA_HD void digest(const State& s, uint8_t out[32]) {
    uint32_t w[8];
    tail_digest_w(s, nullptr, 0, w);
    sha::words_to_bytes(w, out);
}

}  // namespace ts
