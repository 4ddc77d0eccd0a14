// Device helpers shared by the sumcheck kernels: block reduction of field
// elements, the block-cooperative transcript steps, Lagrange evaluation.
//
// Transcript steps are latency-bound (SHA-256 compressions are sequential), so
// whatever is independent is spread over lanes: the canonical forms of the
// elements to absorb, the message assembly, the three hashes of a challenge
// draw, the terms of the Lagrange sum.  All block_* functions must be called by
// every thread of the block (they contain barriers); blockDim.x >= 64.
#pragma once
#include "zkdl_internal.h"

// Sum of one Fr per thread over the block; result valid in thread 0.
// red: 64 words of LDS.
__device__ __forceinline__ Fr block_sum(Fr x, uint32_t* red) {
    const int tid = threadIdx.x;
    // first inside each wave with cross-lane shuffles, then across the waves via LDS
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        Fr y;
#pragma unroll
        for (int l = 0; l < 8; ++l) y.v[l] = __shfl_down(x.v[l], off, 64);
        x = fr_add(x, y);
    }
    const int wave = tid >> 6, lane = tid & 63;
    const int n_waves = (blockDim.x + 63) >> 6;
    __syncthreads();   // red may still be read from a previous call
    if (lane == 0) {
#pragma unroll
        for (int l = 0; l < 8; ++l) red[l * 8 + wave] = x.v[l];
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < n_waves; ++w) {
            Fr y;
#pragma unroll
            for (int l = 0; l < 8; ++l) y.v[l] = red[l * 8 + w];
            x = fr_add(x, y);
        }
    }
    return x;
}

// Sums N lazy values per thread (normal limbs, each below 2.41 r) over a block of at most
// 8 waves; thread j < N returns the fully reduced sum of value j, other threads zero.
// Limbs are added without carries: three shuffle levels take them from below 2^29 to below
// 2^32, a carry pass follows, three more levels, then a reducing pass (the wave's sum is
// below 64 * 2.41 r < 2^263); at most 8 such wave sums are added before the final reduction.
// red: BLOCK_SUM_LAZY_WORDS words of LDS.
constexpr int BLOCK_SUM_LAZY_WORDS = 8 * ZK_MAX_EVALS * 9;

// Sum over the 64 lanes of a wave of a lazy value (normal limbs, below 2.41 r); every lane
// must call; lane 0 returns the total, normal and below 2.41 r.
__device__ __forceinline__ F9 wave_sum_lazy(F9 s) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
#pragma unroll
        for (int l = 0; l < 9; ++l) s.v[l] += __shfl_down(s.v[l], off, 64);
        if (off == 8) s = f9_norm(s);
    }
    return f9_norm_reduce(s);
}

template <int N>
__device__ __forceinline__ Fr block_sum_lazy(const F9 (&x)[N], uint32_t* red) {
    static_assert(N <= ZK_MAX_EVALS, "red is sized for ZK_MAX_EVALS values");
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n_waves = (blockDim.x + 63) >> 6;
    F9 s[N];
#pragma unroll
    for (int j = 0; j < N; ++j) s[j] = wave_sum_lazy(x[j]);
    __syncthreads();   // red may still be read from a previous call
    if (lane == 0) {
#pragma unroll
        for (int j = 0; j < N; ++j)
#pragma unroll
            for (int l = 0; l < 9; ++l) red[(wave * N + j) * 9 + l] = s[j].v[l];
    }
    __syncthreads();
    Fr out = fr_zero();
    if (tid < N) {
        F9 t = f9_zero();
        for (int w = 0; w < n_waves; ++w)
#pragma unroll
            for (int l = 0; l < 9; ++l) t.v[l] += red[(w * N + tid) * 9 + l];
        out = f9_to_fr(t);
    }
    return out;
}

constexpr int TS_MAX_ABSORB = 8;     // field elements per device-side absorb
constexpr int TS_MAX_DRAW = 64;      // challenges per block_challenges chunk
constexpr int TS_MAX_BLOCKS = 8;     // whole blocks one append may complete (ZK_PEND_CAP + 63 bytes)

// LDS working set of the transcript steps
struct TsShared {
    uint32_t state[8];                       // chaining value after the last whole block of the stream
    uint64_t nblk;                           // whole blocks in the stream
    uint32_t fill;                           // bytes of the unfinished block
    uint32_t bufsel;                         // which of buf[] holds them
    uint32_t buf[2][16];                     // unfinished block, big-endian words, zero beyond fill
    uint32_t msg[16 * (TS_MAX_BLOCKS + 3)];  // blocks being absorbed, then a draw's three blocks
    uint32_t wk[TS_MAX_BLOCKS + 3][64];      // their schedules
    uint32_t canon[TS_MAX_ABSORB][8];        // canonical little-endian limbs being absorbed
    uint32_t dig[2 * TS_MAX_DRAW + 1][8];    // digests of a challenge draw
    Fr tmp[TS_MAX_ABSORB];
    Fr v;
};

__device__ __forceinline__ void block_ts_load(TsShared& S, const DevState* st) {
    if (threadIdx.x < 8) S.state[threadIdx.x] = st->ts_state[threadIdx.x];
    if (threadIdx.x >= 16 && threadIdx.x < 32) S.buf[0][threadIdx.x - 16] = st->ts_buf[threadIdx.x - 16];
    if (threadIdx.x == 8) {
        S.nblk = ((uint64_t)st->ts_nblk[1] << 32) | st->ts_nblk[0];
        S.fill = st->ts_fill;
        S.bufsel = 0;
    }
    __syncthreads();
}

__device__ __forceinline__ void block_ts_store(const TsShared& S, DevState* st) {
    __syncthreads();
    if (threadIdx.x < 8) st->ts_state[threadIdx.x] = S.state[threadIdx.x];
    if (threadIdx.x >= 16 && threadIdx.x < 32) st->ts_buf[threadIdx.x - 16] = S.buf[S.bufsel][threadIdx.x - 16];
    if (threadIdx.x == 8) {
        st->ts_nblk[0] = (uint32_t)S.nblk;
        st->ts_nblk[1] = (uint32_t)(S.nblk >> 32);
        st->ts_fill = S.fill;
    }
}

// byte q of the block that closes a draw hash (tag 0xF0 / 0xF1: tag, u32le(idx), 0x80, zeros,
// 64-bit big-endian bit length at the end of block `last`) or that extends the stream after a
// draw (tag 0xF2: tag, zeros), for an unfinished block of `rem` bytes given by `rest`;
// blk = 0 or 1 is the block the byte belongs to
template <class RestByte>
__device__ __forceinline__ uint32_t ts_draw_byte(uint32_t blk, uint32_t q, uint32_t rem, RestByte rest, uint32_t tag,
                                                 uint32_t idx, uint32_t last, uint64_t bits) {
    const uint32_t p = 64 * blk + q;
    if (p < rem) return rest(p);
    if (p == rem) return tag;
    if (tag == 0xF2u) return 0;
    if (p <= rem + 4) return (idx >> (8 * (p - rem - 1))) & 0xffu;
    if (p == rem + 5) return 0x80u;
    if (blk == last && q >= 56) return (uint32_t)(bits >> (8 * (63 - q))) & 0xffu;
    return 0;
}

// Appends `len` bytes, given by frame(q), to the stream.  Lane j of wave 0 prepares the
// schedule of whole block j, then lane 0 runs the rounds block after block.  With draw1, and
// if the unfinished block that remains leaves room (at most 50 bytes), the three blocks of a
// single-challenge draw that follows (the closing blocks of the two hashes at index 0, and the
// block that extends the stream) get their schedules in the same step, in wk[nb .. nb + 3),
// where nb, the number of whole blocks completed, is returned; -1 - nb if they were not
// prepared.  frame(q) may read S.canon; a barrier is taken first.
template <class FrameByte>
__device__ __forceinline__ int block_append(TsShared& S, uint32_t len, FrameByte frame, bool draw1) {
    __syncthreads();
    const uint32_t fill = S.fill, sel = S.bufsel;
    const uint32_t total = fill + len;
    const uint32_t nb = total / 64, rem = total % 64;
    const bool fused = draw1 && rem <= 50;
    const uint64_t nblk_after = S.nblk + nb;
    const uint64_t bits = (nblk_after * 64u + rem + 5u) * 8u;
    auto stream_byte = [&](uint32_t p) -> uint32_t {   // byte p counted from the start of the unfinished block
        if (p < fill) return (S.buf[sel][p >> 2] >> (24 - 8 * (p & 3))) & 0xffu;
        return frame(p - fill) & 0xffu;
    };
    auto rest_byte = [&](uint32_t p) -> uint32_t { return stream_byte(64 * nb + p); };
    // every thread builds whole words, byte by byte: the whole blocks, the new unfinished block,
    // the draw's blocks
    const uint32_t nwords = 16 * nb + 16 + (fused ? 48u : 0u);
    for (uint32_t j = threadIdx.x; j < nwords; j += blockDim.x) {
        uint32_t word = 0;
        if (j < 16 * nb) {
#pragma unroll
            for (int b = 0; b < 4; ++b) word = (word << 8) | stream_byte(4 * j + b);
            S.msg[j] = word;
        } else if (j < 16 * nb + 16) {
            const uint32_t q0 = 4 * (j - 16 * nb);
#pragma unroll
            for (int b = 0; b < 4; ++b) word = (word << 8) | (q0 + b < rem ? rest_byte(q0 + b) : 0u);
            S.buf[sel ^ 1][j - 16 * nb] = word;
        } else {
            const uint32_t k = j - 16 * nb - 16, t = k >> 4, q0 = 4 * (k & 15);
#pragma unroll
            for (int b = 0; b < 4; ++b)
                word = (word << 8) | ts_draw_byte(0, q0 + b, rem, rest_byte, 0xF0u + t, 0u, 0u, bits);
            S.msg[16 * nb + k] = word;
        }
    }
    __syncthreads();
    if (threadIdx.x < nb + (fused ? 3u : 0u)) {
        sha::Words16 w;
#pragma unroll
        for (int i = 0; i < 16; ++i) w.v[i] = S.msg[16 * threadIdx.x + i];
        sha::schedule_wk_lds(w, (sha::lds_u32_ptr)S.wk[threadIdx.x]);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (nb > 0) {
            sha::Words8 h;
#pragma unroll
            for (int i = 0; i < 8; ++i) h.v[i] = S.state[i];
            for (uint32_t blk = 0; blk < nb; ++blk) h = sha::rounds_lds(h, (sha::lds_u32_cptr)S.wk[blk]);
#pragma unroll
            for (int i = 0; i < 8; ++i) S.state[i] = h.v[i];
        }
        S.nblk = nblk_after;
        S.fill = rem;
        S.bufsel = sel ^ 1;
    }
    __syncthreads();
    return fused ? (int)nb : -1 - (int)nb;
}

// stream <- stream || 0x01 || label || u64le(32 count) || canon[0..count) for a one-character
// label; canon must be complete (a barrier is taken first).  Return value as block_append.
// On a block-aligned stream - every round after a draw - the words are put together from
// whole limbs: the data start at byte 10, so a message word is the upper half of one limb and
// the lower half of the next, bytes swapped.
__device__ inline int block_absorb1(TsShared& S, char label, int count, bool draw1) {
    const uint32_t data_len = 32u * (uint32_t)count;
    __syncthreads();
    if (S.fill != 0) {
        auto frame = [&](uint32_t q) -> uint32_t {
            if (q == 0) return 1u;
            if (q == 1) return (uint32_t)(uint8_t)label;
            if (q < 10) return q - 2 < 4 ? (data_len >> (8 * (q - 2))) & 0xffu : 0u;
            const uint32_t d = q - 10;
            return (S.canon[d >> 5][(d & 31) >> 2] >> (8 * (d & 3))) & 0xffu;
        };
        return block_append(S, 10u + data_len, frame, draw1);
    }
    const uint32_t sel = S.bufsel;
    const uint32_t total = 10u + data_len, nb = total / 64, rem = total % 64;   // rem % 4 == 2
    const bool fused = draw1 && rem <= 50;
    const uint64_t nblk_after = S.nblk + nb;
    const uint64_t bits = (nblk_after * 64u + rem + 5u) * 8u;
    const uint32_t nlimb = 8u * (uint32_t)count;
    auto frame_word = [&](uint32_t k) -> uint32_t {   // bytes 4k .. 4k+3 of the frame, first byte on top
        if (k == 0) return (1u << 24) | ((uint32_t)(uint8_t)label << 16) | ((data_len & 0xffu) << 8) | ((data_len >> 8) & 0xffu);
        if (k == 1) return 0u;                        // length bytes 2..5: data_len < 2^16
        const uint32_t ip = k - 3, in = k - 2;        // limbs that end / begin in this word
        const uint32_t lp = (k >= 3 && ip < nlimb) ? S.canon[ip >> 3][ip & 7] : 0u;
        const uint32_t ln = in < nlimb ? S.canon[in >> 3][in & 7] : 0u;
        return (((lp >> 16) & 0xffu) << 24) | ((lp >> 24) << 16) | ((ln & 0xffu) << 8) | ((ln >> 8) & 0xffu);
    };
    const uint32_t wr = rem >> 2;                     // word of the unfinished block that takes the tag
    const uint32_t nwords = 16 * nb + 16 + (fused ? 48u : 0u);
    for (uint32_t j = threadIdx.x; j < nwords; j += blockDim.x) {
        if (j < 16 * nb) {
            S.msg[j] = frame_word(j);
        } else if (j < 16 * nb + 16) {
            S.buf[sel ^ 1][j - 16 * nb] = frame_word(j);
        } else {
            const uint32_t k = j - 16 * nb - 16, t = k >> 4, i = k & 15;
            uint32_t word = frame_word(16 * nb + i);
            if (i == wr) word |= (0xF0u + t) << 8;                    // tag; the index bytes are zero
            if (t < 2) {
                if (i == wr + 1) word |= 0x80u;
                if (i == 14) word = (uint32_t)(bits >> 32);
                if (i == 15) word = (uint32_t)bits;
            }
            S.msg[16 * nb + k] = word;
        }
    }
    __syncthreads();
    if (threadIdx.x < nb + (fused ? 3u : 0u)) {
        sha::Words16 w;
#pragma unroll
        for (int i = 0; i < 16; ++i) w.v[i] = S.msg[16 * threadIdx.x + i];
        sha::schedule_wk_lds(w, (sha::lds_u32_ptr)S.wk[threadIdx.x]);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (nb > 0) {
            sha::Words8 h;
#pragma unroll
            for (int i = 0; i < 8; ++i) h.v[i] = S.state[i];
            for (uint32_t blk = 0; blk < nb; ++blk) h = sha::rounds_lds(h, (sha::lds_u32_cptr)S.wk[blk]);
#pragma unroll
            for (int i = 0; i < 8; ++i) S.state[i] = h.v[i];
        }
        S.nblk = nblk_after;
        S.fill = rem;
        S.bufsel = sel ^ 1;
    }
    __syncthreads();
    return fused ? (int)nb : -1 - (int)nb;
}

// canonical forms of vals[0..count) (Montgomery, LDS or global) -> proof words (if
// proof_dst) and into the transcript under a one-character label
__device__ inline void block_absorb_frs(TsShared& S, char label, const Fr* vals, int count,
                                        uint32_t* proof_dst) {
    if (threadIdx.x < (unsigned)count) {
        Fr plain = fr_from_mont_ni(vals[threadIdx.x]);
#pragma unroll
        for (int l = 0; l < 8; ++l) {
            S.canon[threadIdx.x][l] = plain.v[l];
            if (proof_dst) proof_dst[8 * threadIdx.x + l] = plain.v[l];
        }
    }
    block_absorb1(S, label, count, false);
}

// draws `count` challenges into st->chal[base..), st->chal_le; one stream extension.
// The first one is also left in S.v.  Works for any unfinished block (the closing blocks of
// a hash are two when it holds more than 50 bytes).
__device__ inline void block_challenges(TsShared& S, DevState* st, int base, int count) {
    if (count <= 0) return;
    __syncthreads();
    const uint32_t rem = S.fill, sel = S.bufsel;
    const uint32_t last = rem + 14 > 64 ? 1u : 0u;
    const uint64_t bits = (S.nblk * 64u + rem + 5u) * 8u;
    auto rest_byte = [&](uint32_t p) -> uint32_t { return (S.buf[sel][p >> 2] >> (24 - 8 * (p & 3))) & 0xffu; };
    for (int c0 = 0; c0 < count; c0 += TS_MAX_DRAW) {
        const int n = count - c0 < TS_MAX_DRAW ? count - c0 : TS_MAX_DRAW;
        const bool lastchunk = c0 + n >= count;
        const int jobs = 2 * n + (lastchunk ? 1 : 0);
        for (int t = threadIdx.x; t < jobs; t += blockDim.x) {
            sha::Words8 h;
#pragma unroll
            for (int i = 0; i < 8; ++i) h.v[i] = S.state[i];
            const bool elem = t < 2 * n;
            const uint32_t tag = elem ? 0xF0u + (uint32_t)(t & 1) : 0xF2u;
            const uint32_t idx = elem ? (uint32_t)(c0 + (t >> 1)) : 0u;
            const uint32_t nbk = elem ? last + 1 : 1u;
            for (uint32_t blk = 0; blk < nbk; ++blk) {
                sha::Words16 w;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    uint32_t word = 0;
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        word = (word << 8) | ts_draw_byte(blk, 4 * i + b, rem, rest_byte, tag, idx, last, bits);
                    w.v[i] = word;
                }
                h = sha::compress_ni(h, w);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) S.dig[t][i] = h.v[i];
        }
        __syncthreads();
        // wide reduction: one lane per half, then one lane per element
        for (int t = threadIdx.x; t < 2 * n; t += blockDim.x) {
            Fr x;
#pragma unroll
            for (int l = 0; l < 8; ++l) x.v[l] = sha::bswap32(S.dig[t][l]);
            Fr m = fr_mul_ni(fr_const((t & 1) ? frc::W3 : frc::R2), x);
#pragma unroll
            for (int l = 0; l < 8; ++l) S.dig[t][l] = m.v[l];
        }
        __syncthreads();
        for (int t = threadIdx.x; t < n; t += blockDim.x) {
            Fr lo, hi;
#pragma unroll
            for (int l = 0; l < 8; ++l) {
                lo.v[l] = S.dig[2 * t][l];
                hi.v[l] = S.dig[2 * t + 1][l];
            }
            Fr c = fr_add(lo, hi);
            st->chal[base + c0 + t] = c;
            if (c0 + t == 0) S.v = c;
            Fr plain = fr_from_mont_ni(c);
            uint32_t* le = (uint32_t*)(st->chal_le + 32 * (size_t)(base + c0 + t));
#pragma unroll
            for (int l = 0; l < 8; ++l) le[l] = plain.v[l];
        }
        __syncthreads();
        if (lastchunk) {
            if (threadIdx.x < 8) S.state[threadIdx.x] = S.dig[2 * n][threadIdx.x];
            if (threadIdx.x == 8) {
                S.nblk += 1;
                S.fill = 0;
            }
        }
        __syncthreads();
    }
}

// g(v) from the prepared Lagrange coefficients c[k] = g(k) / prod_{j != k} (k - j), npts = 2..4,
// by one wave (all 64 lanes call, no barrier inside); lane 0 returns the value.
//   npts = 4: g(v) = (v-2)(v-3) [c0 (v-1) + c1 v] + v (v-1) [c2 (v-3) + c3 (v-2)]
//   npts = 3: g(v) = (v-2) [c0 (v-1) + c1 v] + c2 v (v-1)
//   npts = 2: g(v) = c0 (v-1) + c1 v
// The operands of each level are selected per lane and multiplied by one call: lanes that
// branch to separate calls would run them one after the other.
__device__ inline Fr wave_lagrange(const Fr* c, int npts, const Fr& v) {
    const int lane = threadIdx.x & 63;
    const Fr one = fr_one();
    const Fr v1 = fr_sub(v, one), v2 = fr_sub(v1, one), v3 = fr_sub(v2, one);
    // level 1, lanes 0..5: c0 (v-1), c1 v, c2 (v-3) | c2 v, c3 (v-2), (v-2)(v-3), v (v-1)
    Fr A = lane == 4 ? v2 : v;
    if (lane < npts) A = c[lane];
    Fr B = lane == 1 ? v : v1;
    if (npts == 4) {
        if (lane == 2 || lane == 4) B = v3;
        else if (lane == 3) B = v2;
    } else if (lane == 2) {
        B = v;
    }
    const Fr p = fr_mul_ni(A, B);
    // level 2, lanes 0, 1
    Fr qa, qb, qc;   // products of lanes 2 lane, 2 lane + 1, 4 + lane
#pragma unroll
    for (int l = 0; l < 8; ++l) {
        qa.v[l] = __shfl(p.v[l], (2 * lane) & 63, 64);
        qb.v[l] = __shfl(p.v[l], (2 * lane + 1) & 63, 64);
        qc.v[l] = __shfl(p.v[l], (4 + lane) & 63, 64);
    }
    Fr r;
    if (npts == 2) {
        r = fr_add(qa, qb);   // lane 0: q0 + q1
    } else {
        Fr A2, B2;
        if (npts == 4) {
            A2 = qc;                   // lane 0: (v-2)(v-3), lane 1: v (v-1)
            B2 = fr_add(qa, qb);       // lane 0: q0 + q1, lane 1: q2 + q3
        } else {
            A2 = lane == 0 ? v2 : qa;  // lane 1: q2 = c2 v
            B2 = lane == 0 ? fr_add(qa, qb) : v1;
        }
        r = fr_mul_ni(A2, B2);
        Fr r1;
#pragma unroll
        for (int l = 0; l < 8; ++l) r1.v[l] = __shfl(r.v[l], 1, 64);
        r = fr_add(r, r1);
    }
    return r;
}

// The claim of the last finished round may still be owed: a round kernel needs only the
// challenge, so the evaluation g_t(v_t) is left to whoever needs the claim next, who does it
// in a spare wave next to other work.  One wave calls this; afterwards st->claim is current.
__device__ inline void wave_resolve_claim(DevState* st) {
    const uint32_t npts = st->lag_npts;   // wave-uniform
    if (npts) {
        const Fr c = wave_lagrange(st->lag, (int)npts, st->chal[st->lag_chal]);
        if ((threadIdx.x & 63) == 0) {
            st->claim = c;
            st->lag_npts = 0;
        }
    }
}

// S.canon[0..count) go into the transcript under a one-character label, then one challenge is drawn: it is
// returned to every thread and stored in st->chal[chal_idx] (Montgomery form) and st->chal_le (canonical).
// When the unfinished block leaves room, the closing blocks of the draw's hashes are scheduled during the
// absorb and hashed by lanes 0..2 side by side.  Needs blockDim.x >= 192 (lane 128 writes the canonical form).
__device__ inline Fr block_absorb_draw1(TsShared& S, DevState* st, char label, int count, int chal_idx) {
    const int tid = threadIdx.x;
    const int prep = block_absorb1(S, label, count, true);
    Fr v;
    if (prep >= 0) {
        // challenge hashes on the schedules prepared during the absorb: lanes 0, 1 (the two
        // halves of the element), 2 (the block that extends the stream)
        if (tid < 3) {
            sha::Words8 h;
#pragma unroll
            for (int i = 0; i < 8; ++i) h.v[i] = S.state[i];
            const sha::Words8 ow = sha::rounds_lds(h, (sha::lds_u32_cptr)S.wk[prep + tid]);
            if (tid < 2) {
                Fr x;
#pragma unroll
                for (int l = 0; l < 8; ++l) x.v[l] = sha::bswap32(ow.v[l]);
                Fr m = fr_mul_ni(fr_const(tid ? frc::W3 : frc::R2), x);
#pragma unroll
                for (int l = 0; l < 8; ++l) S.dig[tid][l] = m.v[l];
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) S.dig[2][i] = ow.v[i];
            }
        }
        __syncthreads();
        Fr lo, hi;
#pragma unroll
        for (int l = 0; l < 8; ++l) {
            lo.v[l] = S.dig[0][l];
            hi.v[l] = S.dig[1][l];
        }
        v = fr_add(lo, hi);   // every thread
        if (tid < 8) S.state[tid] = S.dig[2][tid];
        if (tid == 8) {
            S.nblk += 1;
            S.fill = 0;
        }
        if (tid == 128) {
            Fr plain = fr_from_mont_ni(v);
            uint32_t* le = (uint32_t*)(st->chal_le + 32 * (size_t)chal_idx);
#pragma unroll
            for (int l = 0; l < 8; ++l) le[l] = plain.v[l];
        }
    } else {
        // the unfinished block is too full for single closing blocks (a round that follows
        // other frames without a draw in between): the general draw
        block_challenges(S, st, chal_idx, 1);
        v = S.v;
    }
    if (tid == 0) st->chal[chal_idx] = v;
    return v;
}

// First part of closing a round: g_t(0..npts-1) (LDS, Montgomery, npts = 2..4) go to the proof
// and into the transcript, the round's challenge v_t is drawn and returned to every thread.
// The Lagrange coefficients of g_t are left in S.tmp[0..npts) for the claim g_t(v_t).
// Needs blockDim.x >= 192: while wave 0 hashes, wave 1 prepares the coefficients and wave 2
// later writes the canonical form of the challenge.
__device__ inline Fr block_round_challenge(TsShared& S, DevState* st, const Fr* g, int npts,
                                           uint32_t proof_off, int chal_idx, char label = 'g',
                                           bool skip1 = true) {
    const int tid = threadIdx.x;
    uint32_t* proof_dst = (uint32_t*)(st->proof + proof_off);
    __syncthreads();
    // canonical forms (wave 0) | Lagrange coefficients (wave 1).  The transcript takes
    // g(0), g(2), .., g(npts-1): g(1) is fixed by the claim the transcript already determines.
    // (skip1 = false, the f_t of the optimized matrix-product protocol: all evaluations.)
    if (tid < npts) {
        Fr plain = fr_from_mont_ni(g[tid]);
        const int slot = (!skip1 || tid == 0) ? tid : tid - 1;
#pragma unroll
        for (int l = 0; l < 8; ++l) {
            if (!skip1 || tid != 1) S.canon[slot][l] = plain.v[l];
            proof_dst[8 * tid + l] = plain.v[l];
        }
    } else if (tid >= 64 && tid < 64 + npts) {
        const int k = tid - 64;
        Fr c = g[k];
        if (npts == 3) {            // 1/2, -1, 1/2
            c = (k == 1) ? fr_neg(c) : fr_mul_ni(c, st->inv2);
        } else if (npts == 4) {     // -1/6, 1/2, -1/2, 1/6
            c = fr_mul_ni(c, (k == 0 || k == 3) ? st->inv6 : st->inv2);
            if (k == 0 || k == 2) c = fr_neg(c);
        } else if (k == 0) {        // -1, 1
            c = fr_neg(c);
        }
        S.tmp[k] = c;
    }
    return block_absorb_draw1(S, st, label, skip1 ? npts - 1 : npts, chal_idx);
}

// Closes a round completely: challenge, then the next claim g_t(v_t) in st->claim.
__device__ inline Fr block_finalise_round(TsShared& S, DevState* st, const Fr* g, int npts,
                                          uint32_t proof_off, int chal_idx) {
    const Fr v = block_round_challenge(S, st, g, npts, proof_off, chal_idx);
    if ((threadIdx.x >> 6) == 1) {
        const Fr c = wave_lagrange(S.tmp, npts, v);
        if ((threadIdx.x & 63) == 0) st->claim = c;
    }
    __syncthreads();
    return v;
}

// Sums per-block partial sums part[b * npts + x], b < nblk, into g[x] (LDS): wave x
// handles evaluation x on its own (skip1: evaluation 1 is not summed, wave 1 is free for
// other work before the closing barrier).  Needs blockDim.x >= 64 * npts.
__device__ inline void block_reduce_partials(const Fr* part, int nblk, int npts, Fr* g, bool skip1 = false) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (wave < npts && !(skip1 && wave == 1)) {
        Fr s = fr_zero();
        // up to eight rows of 64 partials at a time, their loads issued together: the loop is
        // bound by memory latency
        for (int base = 0; base < nblk; base += 512) {
            const int rows = (nblk - base + 63) / 64 < 8 ? (nblk - base + 63) / 64 : 8;   // wave-uniform
            Fr p[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if (q < rows) {
                    const int b = base + 64 * q + lane;
                    p[q] = b < nblk ? part[(uint64_t)b * npts + wave] : fr_zero();
                }
            }
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (q < rows) s = fr_add(s, p[q]);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            Fr y;
#pragma unroll
            for (int l = 0; l < 8; ++l) y.v[l] = __shfl_down(s.v[l], off, 64);
            s = fr_add(s, y);
        }
        if (lane == 0) g[wave] = s;
    }
    __syncthreads();
}

// ---- Montgomery form times plain integer --------------------------------------------------------
// A value in Montgomery form times a plain integer is the Montgomery form of the product: such
// products are accumulated as 64-bit columns of 29-bit limb products with no reduction, and reduced
// once per thread or per output.
// cols += c * mag for a normal or negated-normal c (limbs below 2^30.6) and mag < 2^58
__device__ __forceinline__ void cols11_mac(uint64_t* cols, const F9& c, uint64_t mag) {
    const uint32_t m0 = (uint32_t)mag & frc::M29, m1 = (uint32_t)(mag >> 29);
#pragma unroll
    for (int i = 0; i < 9; ++i) {
        cols[i] += (uint64_t)c.v[i] * m0;
        cols[i + 1] += (uint64_t)c.v[i] * m1;
    }
}

// cols += p * c for a signed c, |c| < 2^58, and a normal p below 2.6 r: a negative c turns p
// into 4r - p
__device__ __forceinline__ void cols11_mac_signed(uint64_t* cols, const F9& p, int64_t c) {
    const bool neg = c < 0;
    const uint64_t mag = neg ? (uint64_t)0 - (uint64_t)c : (uint64_t)c;
    F9 q;
#pragma unroll
    for (int i = 0; i < 9; ++i) q.v[i] = neg ? frc::C4R[i] - p.v[i] : p.v[i];
    cols11_mac(cols, q, mag);
}

// carries of an 11-column accumulator: columns 0..9 below 2^29 afterwards
__device__ __forceinline__ void cols11_carry(uint64_t* cols) {
#pragma unroll
    for (int k = 0; k + 1 < 11; ++k) {
        cols[k + 1] += cols[k] >> 29;
        cols[k] &= frc::M29;
    }
}

// carried 11-column sum V -> lazy value congruent to it, normal and below 2.41 r:
// V = low nine limbs + 2^261 * high part, and 2^261 is the Montgomery radix, so the high part
// times R^2 as a Montgomery product is congruent to 2^261 * high part
__device__ __forceinline__ F9 cols11_value(const uint64_t* cols) {
    F9 vlo, vhi = f9_zero();
#pragma unroll
    for (int i = 0; i < 9; ++i) vlo.v[i] = (uint32_t)cols[i];
    vhi.v[0] = (uint32_t)cols[9];
    vhi.v[1] = (uint32_t)cols[10] & frc::M29;
    vhi.v[2] = (uint32_t)(cols[10] >> 29) & frc::M29;
    vhi.v[3] = (uint32_t)(cols[10] >> 58);
    return f9_norm_reduce(f9_add(vlo, f9_mul(vhi, fr_unpack(fr_const(frc::R2)))));
}

// a0 + v0 (a2 - a0) in Montgomery form from the integers; k = (R^2, -R^2, v0 R^2, -v0 R^2),
// canonical.  Four products below 2^58 per column; the result is normal and below 2 r.
__device__ __forceinline__ F9 fold_ints(const F9* k, int64_t a0, int64_t a2) {
    const int64_t d = a2 - a0;
    const bool n0 = a0 < 0, nd = d < 0;
    uint64_t cols[17];
#pragma unroll
    for (int c = 0; c < 17; ++c) cols[c] = 0;
    F9 c0, cd;
#pragma unroll
    for (int i = 0; i < 9; ++i) {
        c0.v[i] = n0 ? k[1].v[i] : k[0].v[i];
        cd.v[i] = nd ? k[3].v[i] : k[2].v[i];
    }
    cols11_mac(cols, c0, n0 ? (uint64_t)0 - (uint64_t)a0 : (uint64_t)a0);
    cols11_mac(cols, cd, nd ? (uint64_t)0 - (uint64_t)d : (uint64_t)d);
    return f9_redc(cols);
}

// ---- launchers defined in k_sumcheck.hip ----
void zk_launch_finalise(zkdl_ctx* ctx, int nblk, int npts, int chal_idx, uint32_t proof_off, int first,
                        uint32_t claim_off, int derive1);
