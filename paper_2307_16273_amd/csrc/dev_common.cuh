// Device helpers shared by the sumcheck kernels: block reduction of field
// elements, the per-round transcript step, Lagrange evaluation.
#pragma once
#include "zkdl_internal.h"

// Sum of one Fr per thread over a 256-thread block; result valid in thread 0.
// red: 8 * ZK_BLOCK words of LDS, limb-major so that lanes hit distinct banks.
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

// value at v of the polynomial through (k, g[k]), k = 0..npts-1 (npts = 2, 3, 4)
__device__ inline Fr lagrange_at(const Fr* g, int npts, const Fr& v, const Fr& inv2, const Fr& inv6) {
    const Fr one = fr_one();
    if (npts == 2) return fr_add(g[0], fr_mul(v, fr_sub(g[1], g[0])));
    Fr v1 = fr_sub(v, one);
    Fr v2 = fr_sub(v1, one);
    if (npts == 3) {
        // L0 = (v-1)(v-2)/2, L1 = -v(v-2), L2 = v(v-1)/2
        Fr l0 = fr_mul(fr_mul(v1, v2), inv2);
        Fr l1 = fr_neg(fr_mul(v, v2));
        Fr l2 = fr_mul(fr_mul(v, v1), inv2);
        return fr_add(fr_add(fr_mul(g[0], l0), fr_mul(g[1], l1)), fr_mul(g[2], l2));
    }
    Fr v3 = fr_sub(v2, one);
    // L0 = -(v-1)(v-2)(v-3)/6, L1 = v(v-2)(v-3)/2, L2 = -v(v-1)(v-3)/2, L3 = v(v-1)(v-2)/6
    Fr v23 = fr_mul(v2, v3);
    Fr v01 = fr_mul(v, v1);
    Fr l0 = fr_neg(fr_mul(fr_mul(v1, v23), inv6));
    Fr l1 = fr_mul(fr_mul(v, v23), inv2);
    Fr l2 = fr_neg(fr_mul(fr_mul(v01, v3), inv2));
    Fr l3 = fr_mul(fr_mul(v01, v2), inv6);
    return fr_add(fr_add(fr_mul(g[0], l0), fr_mul(g[1], l1)),
                  fr_add(fr_mul(g[2], l2), fr_mul(g[3], l3)));
}

constexpr int TS_LDS_BYTES = 512;   // hashing scratch: absorbs of at most 8 field elements

// thread-0 step: canonical bytes of `count` elements -> proof (if dst != nullptr) and absorb
__device__ inline void dev_absorb_frs(DevState* st, const char* label, uint32_t label_len,
                                      const Fr* vals, int count, uint8_t* proof_dst, uint8_t* lds) {
    uint8_t* data = lds + 256;   // absorb() assembles the message in lds[0..), data kept apart
    for (int k = 0; k < count; ++k) ts::fr_to_le(vals[k], data + 32 * k);
    if (proof_dst)
        for (int i = 0; i < 32 * count; ++i) proof_dst[i] = data[i];
    uint8_t state[32];
    for (int i = 0; i < 32; ++i) state[i] = st->ts_state[i];
    // message: 32 + 1 + label + 8 + 32*count (+ padding) must fit before `data` is overwritten:
    // absorb() copies data into the message front to back, and the message start is below data.
    ts::absorb(state, label, label_len, data, 32 * count, lds + 0);
    for (int i = 0; i < 32; ++i) st->ts_state[i] = state[i];
}

__device__ inline Fr dev_challenge(DevState* st, int idx) {
    uint8_t state[32];
    for (int i = 0; i < 32; ++i) state[i] = st->ts_state[i];
    uint8_t le[32];
    Fr c = ts::challenge(state, le);
    for (int i = 0; i < 32; ++i) st->ts_state[i] = state[i];
    st->chal[idx] = c;
    for (int i = 0; i < 32; ++i) st->chal_le[32 * idx + i] = le[i];
    return c;
}

// thread-0 step that closes a round: g_t(0..npts-1) go to the proof and into the
// transcript, the round's challenge is drawn, the next claim is g_t(v_t).
__device__ inline Fr dev_finalise_round(DevState* st, const Fr* g, int npts, uint32_t proof_off,
                                        int chal_idx, uint8_t* lds) {
    dev_absorb_frs(st, "g", 1, g, npts, st->proof + proof_off, lds);
    Fr v = dev_challenge(st, chal_idx);
    st->claim = lagrange_at(g, npts, v, st->inv2, st->inv6);
    return v;
}

// ---- launchers defined in k_sumcheck.hip ----
void zk_launch_finalise(zkdl_ctx* ctx, int nblk, int npts, int chal_idx, uint32_t proof_off, int first,
                        uint32_t claim_off);
