// Product sumcheck rounds (Sec. 2.2; round structure of the protocols in App. B):
// fused fold-and-evaluate kernel, per-round finaliser with the device-side
// transcript, final fold.
#include "dev_common.cuh"

struct RoundArgs {
    FrTab src[3];
    FrTab dst[3];
    uint64_t m;        // half length of the tables this round sums over
    const Fr* chal;    // challenge of the previous round (FOLD only)
    Fr* part;          // partial sums: block b, evaluation x at part[b * (K+1) + x]
};

// Round t of a product of K multilinear tables.
// FOLD = false: the tables have length 2m; g(x) = sum_b prod_k (lo + x (hi - lo)),
//               lo = T[b], hi = T[b + m].
// FOLD = true : the tables still have length 4m; the previous challenge v is bound
//               first, T'[b] = T[b] + v (T[b + 2m] - T[b]) for b < 2m, the folded
//               halves are written to dst and the round polynomial is evaluated on
//               them in the same pass.
template <int K, bool FOLD>
__global__ __launch_bounds__(ZK_BLOCK) void k_sc_round(RoundArgs a) {
    __shared__ uint32_t red[64];
    Fr acc[K + 1];
#pragma unroll
    for (int x = 0; x <= K; ++x) acc[x] = fr_zero();
    Fr v;
    if (FOLD) v = *a.chal;
    const uint64_t m = a.m;
    for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; b < m;
         b += (uint64_t)gridDim.x * blockDim.x) {
        Fr e[K + 1];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            Fr lo, hi;
            if (FOLD) {
                Fr t0 = tab_ld(a.src[k], b), t1 = tab_ld(a.src[k], b + m);
                Fr t2 = tab_ld(a.src[k], b + 2 * m), t3 = tab_ld(a.src[k], b + 3 * m);
                lo = fr_add(t0, fr_mul(v, fr_sub(t2, t0)));
                hi = fr_add(t1, fr_mul(v, fr_sub(t3, t1)));
                tab_st(a.dst[k], b, lo);
                tab_st(a.dst[k], b + m, hi);
            } else {
                lo = tab_ld(a.src[k], b);
                hi = tab_ld(a.src[k], b + m);
            }
            Fr d = fr_sub(hi, lo);
            Fr cur = lo;
#pragma unroll
            for (int x = 0; x <= K; ++x) {
                if (x == 1) cur = hi;
                if (x >= 2) cur = fr_add(cur, d);
                e[x] = (k == 0) ? cur : fr_mul(e[x], cur);
            }
        }
#pragma unroll
        for (int x = 0; x <= K; ++x) acc[x] = fr_add(acc[x], e[x]);
    }
#pragma unroll
    for (int x = 0; x <= K; ++x) {
        Fr s = block_sum(acc[x], red);
        if (threadIdx.x == 0) a.part[(uint64_t)blockIdx.x * (K + 1) + x] = s;
    }
}

struct FinArgs {
    const Fr* part;
    int nblk;
    int npts;
    DevState* st;
    int chal_idx;
    uint32_t proof_off;    // where g_t(0..npts-1) go
    int first;             // round 0: claim_0 = g(0) + g(1) is written and absorbed first
    uint32_t claim_off;
};

// Sums the per-block partials of one round, appends g_t to the proof, absorbs it,
// draws the round's challenge and sets the next claim g_t(v_t).
__global__ __launch_bounds__(ZK_BLOCK) void k_sc_finalise(FinArgs a) {
    __shared__ uint32_t red[64];
    __shared__ TsShared S;
    __shared__ Fr g[ZK_MAX_EVALS + 1];
    DevState* st = a.st;
    block_ts_load(S, st);
    for (int x = 0; x < a.npts; ++x) {
        Fr s = fr_zero();
        for (int b = threadIdx.x; b < a.nblk; b += blockDim.x)
            s = fr_add(s, a.part[(uint64_t)b * a.npts + x]);
        s = block_sum(s, red);
        if (threadIdx.x == 0) g[x] = s;
    }
    __syncthreads();
    if (a.first) {
        if (threadIdx.x == 0) g[ZK_MAX_EVALS] = fr_add(g[0], g[1]);
        __syncthreads();
        block_absorb_frs(S, 'c', &g[ZK_MAX_EVALS], 1, (uint32_t*)(st->proof + a.claim_off));
    }
    block_finalise_round(S, st, g, a.npts, a.proof_off, a.chal_idx);
    block_ts_store(S, st);
}

void zk_launch_finalise(zkdl_ctx* ctx, int nblk, int npts, int chal_idx, uint32_t proof_off, int first,
                        uint32_t claim_off) {
    FinArgs fa;
    fa.part = ctx->partials;
    fa.nblk = nblk;
    fa.npts = npts;
    fa.st = ctx->dev;
    fa.chal_idx = chal_idx;
    fa.proof_off = proof_off;
    fa.first = first;
    fa.claim_off = claim_off;
    zk_prof_begin(ctx, ZKDL_PROF_FINALISE, 32.0 * npts);
    hipLaunchKernelGGL(k_sc_finalise, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, fa);
    zk_prof_end(ctx);
}

struct FinishArgs {
    FrTab src[3];
    int K;
    int fold;            // 1: tables have length 2 and are folded with chal; 0: length 1
    const Fr* chal;
    DevState* st;
    int scal_base;       // finals are left in st->scal[scal_base + k]
    uint32_t finals_off;
    int absorb_claim;    // d == 0: claim_0 = product of the single entries
    uint32_t claim_off;
};

__global__ __launch_bounds__(64) void k_sc_finish(FinishArgs a) {
    __shared__ TsShared S;
    __shared__ Fr f[4];
    DevState* st = a.st;
    block_ts_load(S, st);
    if (threadIdx.x < (unsigned)a.K) {
        const int k = threadIdx.x;
        Fr lo = tab_ld(a.src[k], 0);
        if (a.fold) {
            Fr hi = tab_ld(a.src[k], 1);
            lo = fr_add(lo, fr_mul(*a.chal, fr_sub(hi, lo)));
        }
        f[k] = lo;
        st->scal[a.scal_base + k] = lo;
    }
    __syncthreads();
    if (a.absorb_claim) {
        if (threadIdx.x == 0) {
            Fr c0 = f[0];
            for (int k = 1; k < a.K; ++k) c0 = fr_mul(c0, f[k]);
            st->claim = c0;
            f[3] = c0;
        }
        __syncthreads();
        block_absorb_frs(S, 'c', &f[3], 1, (uint32_t*)(st->proof + a.claim_off));
    }
    block_absorb_frs(S, 'f', f, a.K, (uint32_t*)(st->proof + a.finals_off));
    block_ts_store(S, st);
}

template <int K>
static void launch_round(zkdl_ctx* ctx, bool fold, const RoundArgs& ra, unsigned grid) {
    if (fold)
        hipLaunchKernelGGL((k_sc_round<K, true>), dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, ra);
    else
        hipLaunchKernelGGL((k_sc_round<K, false>), dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, ra);
}

static const uint32_t SC_MAGIC = 0x43534B5Au;

int zk_sumcheck_product(zkdl_ctx* ctx, int K, const FrTab* src, const FrTab* work, int d,
                        int finals_scal_base) {
    if (K < 1 || K > 3) return ZKDL_EINVAL;
    if (ctx->n_chal + d > ZK_MAX_CHAL) return ZKDL_EINVAL;
    const int npts = K + 1;
    uint32_t hdr[4] = {SC_MAGIC, (uint32_t)K, (uint32_t)K, (uint32_t)d};
    zk_write_proof_words(ctx, hdr, 4);
    uint32_t claim_off = (uint32_t)ctx->proof_len;
    uint32_t rounds_off = claim_off + 32;
    uint32_t finals_off = rounds_off + (uint32_t)d * npts * 32;
    if (finals_off + K * 32 > (uint32_t)ZK_PROOF_CAP) return ZKDL_ESMALL;
    ctx->proof_len = finals_off + K * 32;

    int first_chal = ctx->n_chal;
    for (int t = 0; t < d; ++t) {
        RoundArgs ra;
        const bool fold = t > 0;
        const FrTab* from = (t <= 1) ? src : work;
        for (int k = 0; k < K; ++k) {
            ra.src[k] = from[k];
            ra.dst[k] = work[k];
        }
        ra.m = (uint64_t)1 << (d - t - 1);
        ra.chal = fold ? &ctx->dev->chal[first_chal + t - 1] : nullptr;
        ra.part = ctx->partials;
        uint64_t want = (ra.m + ZK_BLOCK - 1) / ZK_BLOCK;
        unsigned grid = (unsigned)(want > ZK_MAX_PART_BLOCKS ? ZK_MAX_PART_BLOCKS : want);
        // algorithmic bytes: per pair index and table, 2 reads (first round) or 4 reads + 2 writes
        zk_prof_begin(ctx, fold ? ZKDL_PROF_SC_ROUND_FUSED : ZKDL_PROF_SC_ROUND_FIRST,
                      (double)K * (fold ? 192.0 : 64.0) * (double)ra.m);
        if (K == 1) launch_round<1>(ctx, fold, ra, grid);
        else if (K == 2) launch_round<2>(ctx, fold, ra, grid);
        else launch_round<3>(ctx, fold, ra, grid);
        zk_prof_end(ctx);
        zk_launch_finalise(ctx, (int)grid, npts, ctx->n_chal++, rounds_off + (uint32_t)t * npts * 32,
                           t == 0, claim_off);
    }
    FinishArgs fi;
    const FrTab* from = (d <= 1) ? src : work;
    for (int k = 0; k < K; ++k) fi.src[k] = from[k];
    fi.K = K;
    fi.fold = d >= 1;
    fi.chal = d >= 1 ? &ctx->dev->chal[first_chal + d - 1] : nullptr;
    fi.st = ctx->dev;
    fi.scal_base = finals_scal_base;
    fi.finals_off = finals_off;
    fi.absorb_claim = (d == 0);
    fi.claim_off = claim_off;
    hipLaunchKernelGGL(k_sc_finish, dim3(1), dim3(64), 0, ctx->stream, fi);
    return ZKDL_OK;
}

// ---- transcript-only kernels -----------------------------------------------------
__global__ __launch_bounds__(ZK_BLOCK) void k_draw(DevState* st, int base, int count) {
    __shared__ TsShared S;
    block_ts_load(S, st);
    block_challenges(S, st, base, count);
    block_ts_store(S, st);
}

void zk_launch_draw(zkdl_ctx* ctx, int chal_base, int count) {
    if (count <= 0) return;
    hipLaunchKernelGGL(k_draw, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev, chal_base, count);
}
