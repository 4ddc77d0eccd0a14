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

constexpr int TS_MAX_ABSORB = 8;     // field elements per device-side absorb
constexpr int TS_MAX_DRAW = 64;      // challenges per block_challenges chunk

// LDS working set of the transcript steps
struct TsShared {
    uint32_t state[8];                       // transcript state, big-endian words
    uint32_t msg[96];                        // padded message, big-endian words (<= 6 blocks)
    uint32_t canon[TS_MAX_ABSORB][8];        // canonical little-endian limbs being absorbed
    uint32_t dig[2 * TS_MAX_DRAW + 1][8];    // digests of a challenge draw
    Fr tmp[TS_MAX_ABSORB];
    Fr v;
};

__device__ __forceinline__ void block_ts_load(TsShared& S, const DevState* st) {
    if (threadIdx.x < 8) S.state[threadIdx.x] = st->ts_state[threadIdx.x];
    __syncthreads();
}

__device__ __forceinline__ void block_ts_store(const TsShared& S, DevState* st) {
    __syncthreads();
    if (threadIdx.x < 8) st->ts_state[threadIdx.x] = S.state[threadIdx.x];
}

// state <- SHA256(state || 0x01 || label || u64le(32 count) || canon[0..count))
// for a one-character label; canon must be complete (a barrier is taken first).
__device__ inline void block_absorb1(TsShared& S, char label, int count) {
    __syncthreads();
    const uint32_t total = 42u + 32u * (uint32_t)count;
    const uint32_t padded = ((total + 9 + 63) / 64) * 64;
    const uint32_t data_len = 32u * (uint32_t)count;
    // every thread builds whole message words, byte by byte
    for (uint32_t j = threadIdx.x; j < padded / 4; j += blockDim.x) {
        uint32_t word = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t p = 4 * j + b;
            uint32_t byte;
            if (p < 32) byte = (S.state[p >> 2] >> (24 - 8 * (p & 3))) & 0xffu;
            else if (p == 32) byte = 1;
            else if (p == 33) byte = (uint8_t)label;
            else if (p < 42) byte = (p - 34 < 4) ? ((data_len >> (8 * (p - 34))) & 0xffu) : 0u;
            else if (p < total) {
                const uint32_t q = p - 42;
                byte = (S.canon[q >> 5][(q & 31) >> 2] >> (8 * (q & 3))) & 0xffu;
            } else if (p == total) byte = 0x80u;
            else if (p >= padded - 4) byte = ((total * 8) >> (8 * (padded - 1 - p))) & 0xffu;
            else byte = 0;
            word = (word << 8) | byte;
        }
        S.msg[j] = word;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t h[8] = {0x6a09e667, 0xbb67ae85, 0x3c6ef372, 0xa54ff53a,
                         0x510e527f, 0x9b05688c, 0x1f83d9ab, 0x5be0cd19};
        for (uint32_t off = 0; off < padded / 4; off += 16) {
            uint32_t w[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) w[i] = S.msg[off + i];
            sha::compress(h, w);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) S.state[i] = h[i];
    }
    __syncthreads();
}

// canonical forms of vals[0..count) (Montgomery, LDS or global) -> proof words (if
// proof_dst) and into the transcript under a one-character label
__device__ inline void block_absorb_frs(TsShared& S, char label, const Fr* vals, int count,
                                        uint32_t* proof_dst) {
    if (threadIdx.x < (unsigned)count) {
        Fr plain = fr_from_mont(vals[threadIdx.x]);
#pragma unroll
        for (int l = 0; l < 8; ++l) {
            S.canon[threadIdx.x][l] = plain.v[l];
            if (proof_dst) proof_dst[8 * threadIdx.x + l] = plain.v[l];
        }
    }
    block_absorb1(S, label, count);
}

// draws `count` challenges into st->chal[base..), st->chal_le; one state update.
// The first one is also left in S.v.
__device__ inline void block_challenges(TsShared& S, DevState* st, int base, int count) {
    if (count <= 0) return;
    __syncthreads();
    for (int c0 = 0; c0 < count; c0 += TS_MAX_DRAW) {
        const int n = count - c0 < TS_MAX_DRAW ? count - c0 : TS_MAX_DRAW;
        const bool last = c0 + n >= count;
        const int jobs = 2 * n + (last ? 1 : 0);
        for (int t = threadIdx.x; t < jobs; t += blockDim.x) {
            uint32_t stw[8], out[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) stw[i] = S.state[i];
            if (t < 2 * n) sha::digest_state_suffix_w(stw, (uint32_t)(t & 1), true, (uint32_t)(c0 + (t >> 1)), out);
            else sha::digest_state_suffix_w(stw, 2u, false, 0u, out);
#pragma unroll
            for (int i = 0; i < 8; ++i) S.dig[t][i] = out[i];
        }
        __syncthreads();
        // wide reduction: one lane per half, then one lane per element
        for (int t = threadIdx.x; t < 2 * n; t += blockDim.x) {
            Fr x;
#pragma unroll
            for (int l = 0; l < 8; ++l) x.v[l] = sha::bswap32(S.dig[t][l]);
            Fr m = fr_mul(fr_const((t & 1) ? frc::W3 : frc::R2), x);
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
            Fr plain = fr_from_mont(c);
            uint32_t* le = (uint32_t*)(st->chal_le + 32 * (size_t)(base + c0 + t));
#pragma unroll
            for (int l = 0; l < 8; ++l) le[l] = plain.v[l];
        }
        __syncthreads();
        if (last && threadIdx.x < 8) S.state[threadIdx.x] = S.dig[2 * n][threadIdx.x];
        __syncthreads();
    }
}

// g (LDS, Montgomery, npts = 2..4 values at 0..npts-1) -> value at v, spread over
// npts lanes: lane k computes g[k] * prod_{j != k} (v - j) / prod_{j != k} (k - j)
__device__ inline Fr block_lagrange(TsShared& S, const Fr* g, int npts, const Fr& v, const Fr& inv2,
                                    const Fr& inv6) {
    __syncthreads();
    const int k = threadIdx.x;
    if (k < npts) {
        const Fr one = fr_one();
        Fr vj[4];
        vj[0] = v;
        for (int j = 1; j < npts; ++j) vj[j] = fr_sub(vj[j - 1], one);
        Fr num = g[k];
        for (int j = 0; j < npts; ++j)
            if (j != k) num = fr_mul(num, vj[j]);
        // 1 / prod_{j != k} (k - j)
        Fr coef;
        bool negate;
        if (npts == 2) { coef = one; negate = (k == 0); }            // -1, 1
        else if (npts == 3) { coef = (k == 1) ? one : inv2; negate = (k == 1); }   // 1/2, -1, 1/2
        else { coef = (k == 0 || k == 3) ? inv6 : inv2; negate = (k == 0 || k == 2); }  // -1/6, 1/2, -1/2, 1/6
        num = fr_mul(num, coef);
        S.tmp[k] = negate ? fr_neg(num) : num;
    }
    __syncthreads();
    Fr acc = S.tmp[0];
    for (int j = 1; j < npts; ++j) acc = fr_add(acc, S.tmp[j]);
    return acc;   // every thread holds the value
}

// Closes a round: g_t(0..npts-1) go to the proof and into the transcript, the round's
// challenge is drawn, the next claim is g_t(v_t).  g in LDS.  Returns v_t.
__device__ inline Fr block_finalise_round(TsShared& S, DevState* st, const Fr* g, int npts,
                                          uint32_t proof_off, int chal_idx) {
    block_absorb_frs(S, 'g', g, npts, (uint32_t*)(st->proof + proof_off));
    block_challenges(S, st, chal_idx, 1);
    Fr v = S.v;
    Fr claim = block_lagrange(S, g, npts, v, st->inv2, st->inv6);
    if (threadIdx.x == 0) st->claim = claim;
    return v;
}

// ---- launchers defined in k_sumcheck.hip ----
void zk_launch_finalise(zkdl_ctx* ctx, int nblk, int npts, int chal_idx, uint32_t proof_off, int first,
                        uint32_t claim_off);
