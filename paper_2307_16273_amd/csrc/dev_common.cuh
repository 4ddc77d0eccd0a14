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
constexpr int TS_MAX_FRAME_BLOCKS = (10 + 32 * TS_MAX_ABSORB + 63) / 64;

// LDS working set of the transcript steps
struct TsShared {
    uint32_t state[8];                       // chaining value after the last block of the stream
    uint64_t nblk;                           // blocks in the stream
    uint32_t msg[16 * TS_MAX_FRAME_BLOCKS];  // frame being absorbed, big-endian words
    uint32_t wk[TS_MAX_FRAME_BLOCKS + 3][64];// schedules: frame blocks, then a draw's three blocks
    uint32_t canon[TS_MAX_ABSORB][8];        // canonical little-endian limbs being absorbed
    uint32_t dig[2 * TS_MAX_DRAW + 1][8];    // digests of a challenge draw
    Fr tmp[TS_MAX_ABSORB];
    Fr v;
};

__device__ __forceinline__ void block_ts_load(TsShared& S, const DevState* st) {
    if (threadIdx.x < 8) S.state[threadIdx.x] = st->ts_state[threadIdx.x];
    if (threadIdx.x == 8) S.nblk = ((uint64_t)st->ts_nblk[1] << 32) | st->ts_nblk[0];
    __syncthreads();
}

__device__ __forceinline__ void block_ts_store(const TsShared& S, DevState* st) {
    __syncthreads();
    if (threadIdx.x < 8) st->ts_state[threadIdx.x] = S.state[threadIdx.x];
    if (threadIdx.x == 8) {
        st->ts_nblk[0] = (uint32_t)S.nblk;
        st->ts_nblk[1] = (uint32_t)(S.nblk >> 32);
    }
}

// blocks of the frame of `count` field elements under a one-character label
__device__ __forceinline__ uint32_t ts_frame_blocks(int count) { return (10u + 32u * (uint32_t)count + 63u) / 64u; }

// stream <- stream || pad64(0x01 || label || u64le(32 count) || canon[0..count)) for a
// one-character label; canon must be complete (a barrier is taken first).  Lane j of
// wave 0 prepares the schedule of frame block j, then lane 0 runs the rounds block after
// block.  With draw1 the three blocks of a single-challenge draw that follows this absorb
// (halves 0xF0, 0xF1 at index 0, and the 0xF2 block) get their schedules in the same step,
// in wk[nb .. nb + 3), nb = ts_frame_blocks(count): they depend on the block count only.
__device__ inline void block_absorb1(TsShared& S, char label, int count, bool draw1) {
    __syncthreads();
    const uint32_t total = 10u + 32u * (uint32_t)count;
    const uint32_t nb = ts_frame_blocks(count);
    const uint32_t data_len = 32u * (uint32_t)count;
    // every thread builds whole message words, byte by byte
    for (uint32_t j = threadIdx.x; j < 16 * nb; j += blockDim.x) {
        uint32_t word = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t p = 4 * j + b;
            uint32_t byte;
            if (p == 0) byte = 1;
            else if (p == 1) byte = (uint8_t)label;
            else if (p < 10) byte = (p - 2 < 4) ? ((data_len >> (8 * (p - 2))) & 0xffu) : 0u;
            else if (p < total) {
                const uint32_t q = p - 10;
                byte = (S.canon[q >> 5][(q & 31) >> 2] >> (8 * (q & 3))) & 0xffu;
            } else byte = 0;
            word = (word << 8) | byte;
        }
        S.msg[j] = word;
    }
    __syncthreads();
    const uint64_t nblk_after = S.nblk + nb;
    if (threadIdx.x < nb + (draw1 ? 3u : 0u)) {
        sha::Words16 w;
        if (threadIdx.x < nb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) w.v[i] = S.msg[16 * threadIdx.x + i];
        } else {
            w = sha::draw_block_words(0xF0u + (threadIdx.x - nb), 0u, nblk_after);
        }
        sha::schedule_wk_lds(w, (sha::lds_u32_ptr)S.wk[threadIdx.x]);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        sha::Words8 h;
#pragma unroll
        for (int i = 0; i < 8; ++i) h.v[i] = S.state[i];
        for (uint32_t blk = 0; blk < nb; ++blk) h = sha::rounds_lds(h, (sha::lds_u32_cptr)S.wk[blk]);
#pragma unroll
        for (int i = 0; i < 8; ++i) S.state[i] = h.v[i];
        S.nblk = nblk_after;
    }
    __syncthreads();
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
// The first one is also left in S.v.
__device__ inline void block_challenges(TsShared& S, DevState* st, int base, int count) {
    if (count <= 0) return;
    __syncthreads();
    for (int c0 = 0; c0 < count; c0 += TS_MAX_DRAW) {
        const int n = count - c0 < TS_MAX_DRAW ? count - c0 : TS_MAX_DRAW;
        const bool last = c0 + n >= count;
        const int jobs = 2 * n + (last ? 1 : 0);
        for (int t = threadIdx.x; t < jobs; t += blockDim.x) {
            sha::Words8 h;
#pragma unroll
            for (int i = 0; i < 8; ++i) h.v[i] = S.state[i];
            const bool elem = t < 2 * n;
            const sha::Words16 w = sha::draw_block_words(elem ? 0xF0u + (uint32_t)(t & 1) : 0xF2u,
                                                         elem ? (uint32_t)(c0 + (t >> 1)) : 0u, S.nblk);
            const sha::Words8 out = sha::compress_ni(h, w);
#pragma unroll
            for (int i = 0; i < 8; ++i) S.dig[t][i] = out.v[i];
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
        if (last) {
            if (threadIdx.x < 8) S.state[threadIdx.x] = S.dig[2 * n][threadIdx.x];
            if (threadIdx.x == 8) S.nblk += 1;
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

// First part of closing a round: g_t(0..npts-1) (LDS, Montgomery, npts = 2..4) go to the proof
// and into the transcript, the round's challenge v_t is drawn and returned to every thread.
// The Lagrange coefficients of g_t are left in S.tmp[0..npts) for the claim g_t(v_t).
// Needs blockDim.x >= 192: while wave 0 hashes, wave 1 prepares the coefficients and wave 2
// later writes the canonical form of the challenge.
__device__ inline Fr block_round_challenge(TsShared& S, DevState* st, const Fr* g, int npts,
                                           uint32_t proof_off, int chal_idx) {
    const int tid = threadIdx.x;
    uint32_t* proof_dst = (uint32_t*)(st->proof + proof_off);
    __syncthreads();
    // canonical forms (wave 0) | Lagrange coefficients (wave 1).  The transcript takes
    // g(0), g(2), .., g(npts-1): g(1) is fixed by the claim the transcript already determines.
    if (tid < npts) {
        Fr plain = fr_from_mont_ni(g[tid]);
        const int slot = tid == 0 ? 0 : tid - 1;
#pragma unroll
        for (int l = 0; l < 8; ++l) {
            if (tid != 1) S.canon[slot][l] = plain.v[l];
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
    block_absorb1(S, 'g', npts - 1, true);
    // challenge hashes on the schedules prepared during the absorb: lanes 0, 1 (the two
    // halves of the element), 2 (the block that extends the stream)
    if (tid < 3) {
        sha::Words8 h;
#pragma unroll
        for (int i = 0; i < 8; ++i) h.v[i] = S.state[i];
        const sha::Words8 ow = sha::rounds_lds(h, (sha::lds_u32_cptr)S.wk[ts_frame_blocks(npts - 1) + tid]);
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
    const Fr v = fr_add(lo, hi);   // every thread
    if (tid < 8) S.state[tid] = S.dig[2][tid];
    if (tid == 8) S.nblk += 1;
    if (tid == 0) st->chal[chal_idx] = v;
    if (tid == 128) {
        Fr plain = fr_from_mont_ni(v);
        uint32_t* le = (uint32_t*)(st->chal_le + 32 * (size_t)chal_idx);
#pragma unroll
        for (int l = 0; l < 8; ++l) le[l] = plain.v[l];
    }
    return v;
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

// ---- launchers defined in k_sumcheck.hip ----
void zk_launch_finalise(zkdl_ctx* ctx, int nblk, int npts, int chal_idx, uint32_t proof_off, int first,
                        uint32_t claim_off, int derive1);
