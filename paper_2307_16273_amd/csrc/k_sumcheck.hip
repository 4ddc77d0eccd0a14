// Product sumcheck rounds (Sec. 2.2; round structure of the protocols in App. B):
// fused fold-and-evaluate kernel, per-round finaliser with the device-side
// transcript, the last rounds in one block, final fold; the stack rounds of the
// optimized aggregated matrix-product protocol (f_t without its beta factor).
#include <string.h>
#include "dev_common.cuh"

struct RoundArgs {
    FrTab src8[3];     // packed source tables (first round, first fused round)
    F9Tab work[3];     // lazy 29-bit-limb work tables (written by every fused round)
    uint64_t m;        // half length of the tables this round sums over
    const Fr* chal;    // challenge of the previous round (fused rounds)
    Fr* part;          // partial sums: block b, evaluation x at part[b * (K+1) + x]
};

// Round t of a product of K multilinear tables (Sec. 2.2).
// MODE 0 (first round): the tables have length 2m; g(x) = sum_b prod_k (lo + x (hi - lo)),
//         lo = T[b], hi = T[b + m], for x = 0..K.
// MODE 1, 2 (fused): the tables still have length 4m; the previous challenge v is bound
//         first, T'[b] = T[b] + v (T[b + 2m] - T[b]) for b < 2m, the folded halves are
//         written to the work tables and the round polynomial is evaluated on them in the
//         same pass.  MODE 1 reads the packed sources, MODE 2 the work tables (in place).
//         g(1) is not computed: the finaliser takes it from the running claim,
//         g(1) = claim - g(0).
//
// Arithmetic stays in 29-bit limbs from load to the per-thread sums.  Invariants:
//   stored work values: normal, value < 2.41 r (f9_norm_reduce at the store);
//   d = hi - lo + 4r has limbs < 2^29 + 2^30; the challenge is normal: product bound holds;
//   evaluation points: e(2) = hi + dn, e(3) = e(2) + dn with dn = norm(hi - lo + 4r):
//   limbs < 2^30.6, and every product has one normal factor;
//   sums are renormalised and reduced after every second addition.
// one pair index: fold (fused modes), evaluate, add the products to acc
template <int K, int MODE>
__device__ __forceinline__ void sc_pair(const RoundArgs& a, uint64_t b, uint64_t m, const F9& v, F9 acc[K + 1]) {
    constexpr bool FOLD = MODE != 0;
    F9 prod[K + 1];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        F9 lo, hi;
        if (MODE == 0) {
            lo = fr_unpack(tab_ld(a.src8[k], b));
            hi = fr_unpack(tab_ld(a.src8[k], b + m));
        } else {
            F9 t0, t1, t2, t3;
            if (MODE == 1) {
                t0 = fr_unpack(tab_ld(a.src8[k], b));
                t1 = fr_unpack(tab_ld(a.src8[k], b + m));
                t2 = fr_unpack(tab_ld(a.src8[k], b + 2 * m));
                t3 = fr_unpack(tab_ld(a.src8[k], b + 3 * m));
            } else {
                t0 = f9tab_ld(a.work[k], b);
                t1 = f9tab_ld(a.work[k], b + m);
                t2 = f9tab_ld(a.work[k], b + 2 * m);
                t3 = f9tab_ld(a.work[k], b + 3 * m);
            }
            lo = f9_norm_reduce(f9_add(t0, f9_mul(f9_sub(t2, t0), v)));
            hi = f9_norm_reduce(f9_add(t1, f9_mul(f9_sub(t3, t1), v)));
            f9tab_st(a.work[k], b, lo);
            f9tab_st(a.work[k], b + m, hi);
        }
        // e(x) = lo + x (hi - lo) at the points needed
        F9 e[K + 1];
        e[0] = lo;
        e[1] = hi;
        if (K >= 2) {
            F9 dn = f9_norm(f9_sub(hi, lo));
            e[2] = f9_add(hi, dn);
            if (K >= 3) e[K] = f9_add(e[2], dn);
            if (k == 0) {   // the running product needs one normal factor
                e[2] = f9_norm(e[2]);
                if (K >= 3) e[K] = f9_norm(e[K]);
            }
        }
#pragma unroll
        for (int x = 0; x <= K; ++x) {
            if (FOLD && x == 1) continue;
            prod[x] = (k == 0) ? e[x] : f9_mul(prod[x], e[x]);
        }
    }
#pragma unroll
    for (int x = 0; x <= K; ++x) {
        if (FOLD && x == 1) continue;
        acc[x] = f9_add(acc[x], prod[x]);
    }
}

template <int K, int MODE>
__global__ __launch_bounds__(ZK_BLOCK) void k_sc_round(RoundArgs a) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    F9 acc[K + 1];
#pragma unroll
    for (int x = 0; x <= K; ++x) acc[x] = f9_zero();
    F9 v = f9_zero();
    if (MODE != 0) v = fr_unpack(*a.chal);
    const uint64_t m = a.m;
    int pending = 0;
    for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; b < m;
         b += (uint64_t)gridDim.x * blockDim.x) {
        sc_pair<K, MODE>(a, b, m, v, acc);
        if (++pending == 2) {
            pending = 0;
#pragma unroll
            for (int x = 0; x <= K; ++x) acc[x] = f9_norm_reduce(acc[x]);
        }
    }
    // fused rounds leave g(1) out: K sums instead of K + 1
    constexpr int NS = MODE != 0 ? K : K + 1;
    F9 need[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) need[j] = f9_norm_reduce(acc[(MODE != 0 && j >= 1) ? j + 1 : j]);
    const Fr s = block_sum_lazy<NS>(need, red);
    if (threadIdx.x < NS) {
        const int x = (MODE != 0 && threadIdx.x >= 1) ? threadIdx.x + 1 : threadIdx.x;
        a.part[(uint64_t)blockIdx.x * (K + 1) + x] = s;
    }
}

struct FinArgs {
    const Fr* part;
    int nblk;
    int npts;
    DevState* st;
    int chal_idx;
    uint32_t proof_off;    // where g_t(0..npts-1) go
    int first;             // 1: claim_0 = g(0) + g(1) is written and absorbed first; 2: written only
                           // (the transcript already fixes it)
    uint32_t claim_off;
    uint32_t claim_copy_off;   // != 0: a second place in the proof for claim_0
    int derive1;           // g(1) = running claim - g(0) (the round kernel left it out)
};

// Sums the per-block partials of one round, appends g_t to the proof, absorbs it,
// draws the round's challenge and sets the next claim g_t(v_t).
__global__ __launch_bounds__(ZK_BLOCK) void k_sc_finalise(FinArgs a) {
    __shared__ TsShared S;
    __shared__ Fr g[ZK_MAX_EVALS + 1];
    __shared__ Fr claim_s;
    DevState* st = a.st;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    block_ts_load(S, st);
    // g(1) comes from the running claim, which the previous round may still owe: wave 1 has no
    // partial sums to add in that case and evaluates it meanwhile
    if (a.derive1 && wave == 1) {
        wave_resolve_claim(st);
        if (lane == 0) claim_s = st->claim;
    }
    block_reduce_partials(a.part, a.nblk, a.npts, g, a.derive1 != 0);
    if (a.derive1 && threadIdx.x == 0) g[1] = fr_sub(claim_s, g[0]);
    __syncthreads();
    if (a.first == 1) {
        if (threadIdx.x == 0) g[ZK_MAX_EVALS] = fr_add(g[0], g[1]);
        __syncthreads();
        block_absorb_frs(S, 'c', &g[ZK_MAX_EVALS], 1, (uint32_t*)(st->proof + a.claim_off));
    }
    if (a.first && (a.first == 2 || a.claim_copy_off) && threadIdx.x == 64) {
        const Fr plain = fr_from_mont_ni(fr_add(g[0], g[1]));
        uint32_t* dst = (uint32_t*)(st->proof + (a.first == 2 ? a.claim_off : a.claim_copy_off));
#pragma unroll
        for (int l = 0; l < 8; ++l) dst[l] = plain.v[l];
    }
    block_round_challenge(S, st, g, a.npts, a.proof_off, a.chal_idx);
    // the next claim g_t(v_t) is owed: whoever needs it evaluates it from these coefficients
    if (wave == 1) {
        if (lane < a.npts) st->lag[lane] = S.tmp[lane];
        if (lane == 0) {
            st->lag_npts = (uint32_t)a.npts;
            st->lag_chal = (uint32_t)a.chal_idx;
        }
    }
    block_ts_store(S, st);
}

static FinArgs zk_fin_args(zkdl_ctx* ctx, int nblk, int npts, int chal_idx, uint32_t proof_off, int first,
                           uint32_t claim_off, int derive1) {
    FinArgs fa;
    fa.part = ctx->partials;
    fa.nblk = nblk;
    fa.npts = npts;
    fa.st = ctx->dev;
    fa.chal_idx = chal_idx;
    fa.proof_off = proof_off;
    fa.first = first;
    fa.claim_off = claim_off;
    fa.claim_copy_off = 0;
    fa.derive1 = derive1;
    return fa;
}

void zk_launch_finalise(zkdl_ctx* ctx, int nblk, int npts, int chal_idx, uint32_t proof_off, int first,
                        uint32_t claim_off, int derive1) {
    FinArgs fa = zk_fin_args(ctx, nblk, npts, chal_idx, proof_off, first, claim_off, derive1);
    zk_prof_begin(ctx, ZKDL_PROF_FINALISE, 32.0 * npts);
    hipLaunchKernelGGL(k_sc_finalise, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, fa);
    zk_prof_end(ctx);
}

struct FinishArgs {
    FrTab src[3];
    F9Tab work[3];
    int from_work;       // the length-2 tables are the lazy work tables
    int K;
    int fold;            // 1: tables have length 2 and are folded with chal; 0: length 1
    const Fr* chal;
    DevState* st;
    int scal_base;       // finals are left in st->scal[scal_base + k]
    uint32_t finals_off;
    int absorb_claim;    // d == 0: claim_0 = product of the single entries
    uint32_t claim_off;
    uint32_t claim_copy_off;         // != 0 (with absorb_claim): a second place in the proof for claim_0
    uint32_t write_owed_claim_off;   // != 0: the running claim (possibly still owed) is written there
};

__global__ __launch_bounds__(64) void k_sc_finish(FinishArgs a) {
    __shared__ TsShared S;
    __shared__ Fr f[4];
    DevState* st = a.st;
    block_ts_load(S, st);
    if (a.write_owed_claim_off) {      // one wave: blockDim.x = 64
        wave_resolve_claim(st);
        if (threadIdx.x == 0) {
            const Fr plain = fr_from_mont_ni(st->claim);
            uint32_t* dst = (uint32_t*)(st->proof + a.write_owed_claim_off);
#pragma unroll
            for (int l = 0; l < 8; ++l) dst[l] = plain.v[l];
        }
    }
    if (threadIdx.x < (unsigned)a.K) {
        const int k = threadIdx.x;
        Fr lo, hi = fr_zero();
        if (a.from_work) {
            lo = f9_to_fr(f9tab_ld(a.work[k], 0));
            hi = f9_to_fr(f9tab_ld(a.work[k], 1));
        } else {
            lo = tab_ld(a.src[k], 0);
            if (a.fold) hi = tab_ld(a.src[k], 1);
        }
        if (a.fold) lo = fr_add(lo, fr_mul_ni(*a.chal, fr_sub(hi, lo)));
        f[k] = lo;
        st->scal[a.scal_base + k] = lo;
    }
    __syncthreads();
    if (a.absorb_claim) {
        if (threadIdx.x == 0) {
            Fr c0 = f[0];
            for (int k = 1; k < a.K; ++k) c0 = fr_mul_ni(c0, f[k]);
            st->claim = c0;
            st->lag_npts = 0;
            f[3] = c0;
        }
        __syncthreads();
        block_absorb_frs(S, 'c', &f[3], 1, (uint32_t*)(st->proof + a.claim_off));
        if (a.claim_copy_off && threadIdx.x < 8)
            ((uint32_t*)(st->proof + a.claim_copy_off))[threadIdx.x] = S.canon[0][threadIdx.x];
    }
    block_absorb_frs(S, 'f', f, a.K, (uint32_t*)(st->proof + a.finals_off));
    block_ts_store(S, st);
}

struct ScTailArgs {
    RoundArgs ra;          // work tables; ra.m = pairs of the first round handled here
    int rounds;            // rounds handled here (the last ones of the sumcheck)
    int first_chal;        // challenge index of the round before the first one handled here
    DevState* st;
    uint32_t rounds_off;   // proof offset of g of the first round handled here
    uint32_t finals_off;
    int scal_base;
};

// The last rounds of a product sumcheck in one block: once a round has at most a few
// pairs per thread, a kernel launch per round costs more than the round.  Same arithmetic
// as k_sc_round<K, 2>, round after round with barriers in between, then the final fold.
template <int K>
__global__ __launch_bounds__(ZK_BLOCK) void k_sc_tail(ScTailArgs a) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    __shared__ uint32_t el[2][K][2][9][64];   // small rounds: [buffer][table][lo/hi][limb][pair]
    __shared__ TsShared S;
    __shared__ Fr g[ZK_MAX_EVALS + 1];
    DevState* st = a.st;
    block_ts_load(S, st);
    uint64_t m = a.ra.m;
    F9 v = fr_unpack(st->chal[a.first_chal]);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // the claim of the round before may still be owed; it is first read after a barrier
    if (wave == 3) wave_resolve_claim(st);
    int el_cur = -1;   // buffer of `el` that holds the current tables; -1: they are in memory
    bool owe = false;  // the claim g(v_owe) of the round before is still to be evaluated
    Fr v_owe = fr_zero();
    for (int t = 0; t < a.rounds; ++t) {
        if (m > 64) {
            if (owe && wave == 3) {
                const Fr c = wave_lagrange(S.tmp, K + 1, v_owe);
                if (lane == 0) st->claim = c;
            }
            owe = false;
            F9 acc[K + 1];
#pragma unroll
            for (int x = 0; x <= K; ++x) acc[x] = f9_zero();
            int pending = 0;
            for (uint64_t b = threadIdx.x; b < m; b += blockDim.x) {
                sc_pair<K, 2>(a.ra, b, m, v, acc);
                if (++pending == 2) {
                    pending = 0;
#pragma unroll
                    for (int x = 0; x <= K; ++x) acc[x] = f9_norm_reduce(acc[x]);
                }
            }
            F9 need[K];
#pragma unroll
            for (int j = 0; j < K; ++j) need[j] = f9_norm_reduce(acc[j >= 1 ? j + 1 : j]);
            const Fr s = block_sum_lazy<K>(need, red);
            if (threadIdx.x < K) g[threadIdx.x >= 1 ? threadIdx.x + 1 : 0] = s;
            if (threadIdx.x == 0) g[1] = fr_sub(st->claim, s);
        } else {
            // At most 64 pairs: a thread per (table, pair) folds, then a thread per
            // (evaluation point, pair) multiplies, so a round is two products deep instead of
            // 4 K; wave w sums the point x = 0, 2, 3 [w] by itself.  The folded pairs stay in
            // LDS from here on (stores of a few words per plane to memory are slow).
            const int mi = (int)m;
            const int nxt = el_cur < 0 ? 0 : el_cur ^ 1;
            if (wave < K && lane < mi) {
                F9 t4[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int i = lane + q * mi;   // index in the table of length 4 m
                    if (el_cur < 0) {
                        t4[q] = f9tab_ld(a.ra.work[wave], (uint64_t)i);
                    } else {
                        const int h = i >= 2 * mi, b = i - h * 2 * mi;
#pragma unroll
                        for (int l = 0; l < 9; ++l) t4[q].v[l] = el[el_cur][wave][h][l][b];
                    }
                }
                const F9 lo = f9_norm_reduce(f9_add(t4[0], f9_mul(f9_sub(t4[2], t4[0]), v)));
                const F9 hi = f9_norm_reduce(f9_add(t4[1], f9_mul(f9_sub(t4[3], t4[1]), v)));
#pragma unroll
                for (int l = 0; l < 9; ++l) {
                    el[nxt][wave][0][l][lane] = lo.v[l];
                    el[nxt][wave][1][l][lane] = hi.v[l];
                }
            }
            __syncthreads();
            if (owe && wave == 3) {   // between the two barriers the other waves multiply
                const Fr c = wave_lagrange(S.tmp, K + 1, v_owe);
                if (lane == 0) st->claim = c;
            }
            owe = false;
            F9 prod = f9_zero();
            if (wave < K && lane < mi) {
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    F9 lo, hi;
#pragma unroll
                    for (int l = 0; l < 9; ++l) {
                        lo.v[l] = el[nxt][k][0][l][lane];
                        hi.v[l] = el[nxt][k][1][l][lane];
                    }
                    F9 e = lo;
                    if (wave >= 1) {   // x = 2, 3: hi + (x - 1)(hi - lo); limbs below 2^30.6
                        const F9 dn = f9_norm(f9_sub(hi, lo));
                        e = f9_add(hi, dn);
                        if (wave == 2) e = f9_add(e, dn);
                        if (k == 0) e = f9_norm(e);   // the running product needs one normal factor
                    }
                    prod = k == 0 ? e : f9_mul(prod, e);
                }
                prod = f9_norm_reduce(prod);
            }
            const F9 s = wave_sum_lazy(prod);
            if (wave < K && lane == 0) g[wave == 0 ? 0 : wave + 1] = f9_to_fr(s);
            __syncthreads();
            if (threadIdx.x == 0) g[1] = fr_sub(st->claim, g[0]);
            el_cur = nxt;
        }
        __syncthreads();
        Fr vr = block_round_challenge(S, st, g, K + 1, a.rounds_off + (uint32_t)t * (K + 1) * 32,
                                      a.first_chal + 1 + t);
        // the next claim is evaluated by wave 3 next to the following round's work; it is
        // read after the barriers of that round's sums
        owe = true;
        v_owe = vr;
        v = fr_unpack(vr);
        m >>= 1;
    }
    // final fold of the length-2 tables, finals into the proof and the transcript
    __shared__ Fr f[4];
    if (threadIdx.x < K) {
        const int k = threadIdx.x;
        F9 lo9, hi9;
        if (el_cur < 0) {
            lo9 = f9tab_ld(a.ra.work[k], 0);
            hi9 = f9tab_ld(a.ra.work[k], 1);
        } else {
#pragma unroll
            for (int l = 0; l < 9; ++l) {
                lo9.v[l] = el[el_cur][k][0][l][0];
                hi9.v[l] = el[el_cur][k][1][l][0];
            }
        }
        Fr lo = f9_to_fr(lo9);
        const Fr hi = f9_to_fr(hi9);
        lo = fr_add(lo, fr_mul_ni(fr_pack(f9_cond_sub(f9_norm_reduce(v))), fr_sub(hi, lo)));
        f[k] = lo;
        st->scal[a.scal_base + k] = lo;
    }
    __syncthreads();
    block_absorb_frs(S, 'f', f, K, (uint32_t*)(st->proof + a.finals_off));
    block_ts_store(S, st);
}

template <int K>
static void launch_tail(zkdl_ctx* ctx, const ScTailArgs& ta) {
    hipLaunchKernelGGL((k_sc_tail<K>), dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ta);
}

template <int K>
static void launch_round(zkdl_ctx* ctx, int mode, const RoundArgs& ra, unsigned grid) {
    if (mode == 0)
        hipLaunchKernelGGL((k_sc_round<K, 0>), dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, ra);
    else if (mode == 1)
        hipLaunchKernelGGL((k_sc_round<K, 1>), dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, ra);
    else
        hipLaunchKernelGGL((k_sc_round<K, 2>), dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, ra);
}

static const uint32_t SC_MAGIC = 0x43534B5Au;

size_t zk_sumcheck_work_bytes(int K, int d) {
    const uint64_t half = d >= 1 ? ((uint64_t)1 << (d - 1)) : 1;
    return (size_t)K * half * 36;
}

int zk_sumcheck_product(zkdl_ctx* ctx, int K, const FrTab* src, void* work_mem, int d,
                        int finals_scal_base) {
    if (K < 1 || K > 3) return ZKDL_EINVAL;
    if (ctx->n_chal + d > ZK_MAX_CHAL) return ZKDL_EINVAL;
    zk_flush_frames(ctx);
    const int npts = K + 1;
    uint32_t hdr[4] = {SC_MAGIC, (uint32_t)K, (uint32_t)K, (uint32_t)d};
    zk_write_proof_words(ctx, hdr, 4);
    uint32_t claim_off = (uint32_t)ctx->proof_len;
    uint32_t rounds_off = claim_off + 32;
    uint32_t finals_off = rounds_off + (uint32_t)d * npts * 32;
    if (finals_off + K * 32 > (uint32_t)ZK_PROOF_CAP) return ZKDL_ESMALL;
    ctx->proof_len = finals_off + K * 32;

    const uint64_t half = d >= 1 ? ((uint64_t)1 << (d - 1)) : 1;
    F9Tab work[3];
    for (int k = 0; k < K; ++k) {
        work[k].p = (uint32_t*)work_mem + (size_t)k * half * 9;
        work[k].ps = half;
    }
    int first_chal = ctx->n_chal;
    // the last rounds (at most SC_TAIL_LOG of them, never the first two) run in one block
    constexpr int SC_TAIL_LOG = 10;
    const int t_tail = d >= 3 ? (d - SC_TAIL_LOG > 2 ? d - SC_TAIL_LOG : 2) : d;
    for (int t = 0; t < t_tail; ++t) {
        RoundArgs ra;
        const int mode = t == 0 ? 0 : t == 1 ? 1 : 2;
        for (int k = 0; k < K; ++k) {
            ra.src8[k] = src[k];
            ra.work[k] = work[k];
        }
        ra.m = (uint64_t)1 << (d - t - 1);
        ra.chal = mode ? &ctx->dev->chal[first_chal + t - 1] : nullptr;
        ra.part = ctx->partials;
        uint64_t want = (ra.m + ZK_BLOCK - 1) / ZK_BLOCK;
        unsigned grid = (unsigned)(want > ZK_MAX_PART_BLOCKS ? ZK_MAX_PART_BLOCKS : want);
        // algorithmic bytes: per pair index and table, 2 reads (first round) or 4 reads + 2 writes
        zk_prof_begin(ctx, mode ? ZKDL_PROF_SC_ROUND_FUSED : ZKDL_PROF_SC_ROUND_FIRST,
                      (double)K * (mode ? 192.0 : 64.0) * (double)ra.m);
        if (K == 1) launch_round<1>(ctx, mode, ra, grid);
        else if (K == 2) launch_round<2>(ctx, mode, ra, grid);
        else launch_round<3>(ctx, mode, ra, grid);
        zk_prof_end(ctx);
        zk_launch_finalise(ctx, (int)grid, npts, ctx->n_chal++, rounds_off + (uint32_t)t * npts * 32,
                           t == 0, claim_off, mode != 0);
    }
    if (t_tail < d) {
        ScTailArgs ta;
        for (int k = 0; k < K; ++k) {
            ta.ra.src8[k] = src[k];
            ta.ra.work[k] = work[k];
        }
        ta.ra.m = (uint64_t)1 << (d - t_tail - 1);
        ta.ra.chal = nullptr;
        ta.ra.part = nullptr;
        ta.rounds = d - t_tail;
        ta.first_chal = first_chal + t_tail - 1;
        ta.st = ctx->dev;
        ta.rounds_off = rounds_off + (uint32_t)t_tail * npts * 32;
        ta.finals_off = finals_off;
        ta.scal_base = finals_scal_base;
        ctx->n_chal += d - t_tail;
        if (K == 1) launch_tail<1>(ctx, ta);
        else if (K == 2) launch_tail<2>(ctx, ta);
        else launch_tail<3>(ctx, ta);
        return ZKDL_OK;
    }
    FinishArgs fi;
    for (int k = 0; k < K; ++k) {
        fi.src[k] = src[k];
        fi.work[k] = work[k];
    }
    fi.from_work = d >= 2;
    fi.K = K;
    fi.fold = d >= 1;
    fi.chal = d >= 1 ? &ctx->dev->chal[first_chal + d - 1] : nullptr;
    fi.st = ctx->dev;
    fi.scal_base = finals_scal_base;
    fi.finals_off = finals_off;
    fi.absorb_claim = (d == 0);
    fi.claim_off = claim_off;
    fi.claim_copy_off = 0;
    fi.write_owed_claim_off = 0;
    hipLaunchKernelGGL(k_sc_finish, dim3(1), dim3(64), 0, ctx->stream, fi);
    return ZKDL_OK;
}

// ---------------------------------------------------------------------------
// Optimized aggregated protocol for the batched matrix product (App. B, Protocol
// tensor-op-aggr-optimized): stack rounds send f_t, the round polynomial without its factor
// beta~(w_t, .); beta~(w, .) is never a table that gets folded.
//   f_t(x) = sum_{n'} beta~(w_[t+1:], n') sum_i X0'(x, n', i) X1'(x, n', i),  x = 0, 1, 2,
// X0', X1' the two tables with the earlier stack variables bound.  Pair index b = (n', i),
// partner b + m.  MODE as in k_sc_round: 0 first round (packed sources), 1 fold the previous
// challenge while reading the packed sources, 2 the same in place on the work tables.
// The weight multiplies the first factor's line once (w lo, w hi, and 2 w hi - w lo at x = 2),
// so a pair costs five products and, after the first round, four folds.
// ---------------------------------------------------------------------------
struct FtRoundArgs {
    FrTab src8[2];
    F9Tab work[2];
    uint64_t m;        // pair indices this round: (rows / 2) * inner
    int log_inner;     // row n' of pair index b is b >> log_inner
    FrTab wsuf;        // beta~(w_[t+1:], n'), rows / 2 entries
    const Fr* chal;    // challenge of the previous round (MODE != 0)
    Fr* part;          // block b: f(0), f(1), f(2) at part[3 b + x]
};

template <int MODE>
__global__ __launch_bounds__(ZK_BLOCK) void k_ft_round(FtRoundArgs a) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    F9 acc[3];
#pragma unroll
    for (int x = 0; x < 3; ++x) acc[x] = f9_zero();
    F9 v = f9_zero();
    if (MODE != 0) v = fr_unpack(*a.chal);
    const uint64_t m = a.m;
    for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; b < m;
         b += (uint64_t)gridDim.x * blockDim.x) {
        F9 lo[2], hi[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            if (MODE == 0) {
                lo[k] = fr_unpack(tab_ld(a.src8[k], b));
                hi[k] = fr_unpack(tab_ld(a.src8[k], b + m));
            } else {
                F9 t0, t1, t2, t3;
                if (MODE == 1) {
                    t0 = fr_unpack(tab_ld(a.src8[k], b));
                    t1 = fr_unpack(tab_ld(a.src8[k], b + m));
                    t2 = fr_unpack(tab_ld(a.src8[k], b + 2 * m));
                    t3 = fr_unpack(tab_ld(a.src8[k], b + 3 * m));
                } else {
                    t0 = f9tab_ld(a.work[k], b);
                    t1 = f9tab_ld(a.work[k], b + m);
                    t2 = f9tab_ld(a.work[k], b + 2 * m);
                    t3 = f9tab_ld(a.work[k], b + 3 * m);
                }
                lo[k] = f9_norm_reduce(f9_add(t0, f9_mul(f9_sub(t2, t0), v)));
                hi[k] = f9_norm_reduce(f9_add(t1, f9_mul(f9_sub(t3, t1), v)));
                f9tab_st(a.work[k], b, lo[k]);
                f9tab_st(a.work[k], b + m, hi[k]);
            }
        }
        const F9 w = fr_unpack(tab_ld(a.wsuf, b >> a.log_inner));
        // first factor times the weight: normal values below 2 r
        const F9 wl = f9_mul(lo[0], w), wh = f9_mul(hi[0], w);
        const F9 w2 = f9_norm(f9_add(wh, f9_norm(f9_sub(wh, wl))));          // at x = 2
        const F9 e2 = f9_add(hi[1], f9_norm(f9_sub(hi[1], lo[1])));           // second factor at x = 2
        acc[0] = f9_add(acc[0], f9_mul(wl, lo[1]));
        acc[1] = f9_add(acc[1], f9_mul(wh, hi[1]));
        acc[2] = f9_add(acc[2], f9_mul(w2, e2));
#pragma unroll
        for (int x = 0; x < 3; ++x) acc[x] = f9_norm_reduce(acc[x]);
    }
    const Fr s = block_sum_lazy<3>(acc, red);
    if (threadIdx.x < 3) a.part[(uint64_t)blockIdx.x * 3 + threadIdx.x] = s;
}

struct FtFinArgs {
    const Fr* part;
    int nblk;
    DevState* st;
    int chal_idx;
    uint32_t proof_off;    // where f_t(0..2) go
    int first;             // round 0: claim_0 = (1 - w_0) f_0(0) + w_0 f_0(1) is written and absorbed first
    uint32_t claim_off;
    int w_idx;             // challenge index of w_0
};

// Closes a stack round: sums the partials, [claim_0], f_t into the proof and the transcript,
// the round's challenge; the next claim f_t(v_t) is left owed.
__global__ __launch_bounds__(ZK_BLOCK) void k_ft_finalise(FtFinArgs a) {
    __shared__ TsShared S;
    __shared__ Fr g[ZK_MAX_EVALS + 1];
    DevState* st = a.st;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    block_ts_load(S, st);
    block_reduce_partials(a.part, a.nblk, 3, g);
    if (a.first) {
        if (threadIdx.x == 0) {
            g[ZK_MAX_EVALS] = fr_add(g[0], fr_mul_ni(st->chal[a.w_idx], fr_sub(g[1], g[0])));
            st->lag_npts = 0;
        }
        __syncthreads();
        block_absorb_frs(S, 'c', &g[ZK_MAX_EVALS], 1, (uint32_t*)(st->proof + a.claim_off));
    }
    block_round_challenge(S, st, g, 3, a.proof_off, a.chal_idx, 'f', false);
    if (wave == 1) {
        if (lane < 3) st->lag[lane] = S.tmp[lane];
        if (lane == 0) {
            st->lag_npts = 3;
            st->lag_chal = (uint32_t)a.chal_idx;
        }
    }
    block_ts_store(S, st);
}

// Stack rounds with f_t, then the single-product sumcheck (K = 2) on the bound tables.
// src: X0'[n, i], X1'[n, i] (packed, 2^(ln + l2) entries each); wsuf[t]: beta~(w_[t+1:], .);
// w_idx: challenge index of w_0.  Proof: "ZKSF" block, then the SC block of the second part.
int zk_matmul_ft(zkdl_ctx* ctx, const FrTab* src, void* work_mem, int ln, int l2, const FrTab* wsuf, int w_idx,
                 int finals_scal_base) {
    const int d = ln + l2;
    if (ctx->n_chal + d > ZK_MAX_CHAL) return ZKDL_EINVAL;
    zk_flush_frames(ctx);
    uint32_t hdr[4] = {0x46534B5Au, (uint32_t)ln, (uint32_t)l2, 0};
    zk_write_proof_words(ctx, hdr, 4);
    const uint32_t outer_claim_off = (uint32_t)ctx->proof_len;
    const uint32_t stack_off = outer_claim_off + 32;
    ctx->proof_len = stack_off + 96 * (size_t)ln;
    uint32_t ihdr[4] = {SC_MAGIC, 2, 2, (uint32_t)l2};
    zk_write_proof_words(ctx, ihdr, 4);
    const uint32_t inner_claim_off = (uint32_t)ctx->proof_len;
    const uint32_t inner_rounds_off = inner_claim_off + 32;
    const uint32_t finals_off = inner_rounds_off + 96 * (uint32_t)l2;
    if (finals_off + 64 > (uint32_t)ZK_PROOF_CAP) return ZKDL_ESMALL;
    ctx->proof_len = finals_off + 64;

    const uint64_t half = d >= 1 ? ((uint64_t)1 << (d - 1)) : 1;
    F9Tab work[2];
    for (int k = 0; k < 2; ++k) {
        work[k].p = (uint32_t*)work_mem + (size_t)k * half * 9;
        work[k].ps = half;
    }
    const int first_chal = ctx->n_chal;
    constexpr int SC_TAIL_LOG = 10;
    // the tail kernel takes single-product rounds only, and never the first of them
    int t_tail = d >= 3 ? (d - SC_TAIL_LOG > 2 ? d - SC_TAIL_LOG : 2) : d;
    if (t_tail < ln + 1) t_tail = ln + 1;
    if (t_tail > d) t_tail = d;
    for (int t = 0; t < t_tail; ++t) {
        const int mode = t == 0 ? 0 : t == 1 ? 1 : 2;
        const uint64_t m = (uint64_t)1 << (d - t - 1);
        const uint64_t want = (m + ZK_BLOCK - 1) / ZK_BLOCK;
        const unsigned grid = (unsigned)(want > ZK_MAX_PART_BLOCKS ? ZK_MAX_PART_BLOCKS : want);
        const Fr* prev = mode ? &ctx->dev->chal[first_chal + t - 1] : nullptr;
        if (t < ln) {
            FtRoundArgs fa;
            for (int k = 0; k < 2; ++k) {
                fa.src8[k] = src[k];
                fa.work[k] = work[k];
            }
            fa.m = m;
            fa.log_inner = l2;
            fa.wsuf = wsuf[t];
            fa.chal = prev;
            fa.part = ctx->partials;
            zk_prof_begin(ctx, mode ? ZKDL_PROF_SC_ROUND_FUSED : ZKDL_PROF_SC_ROUND_FIRST,
                          2.0 * (mode ? 192.0 : 64.0) * (double)m);
            if (mode == 0) hipLaunchKernelGGL(k_ft_round<0>, dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, fa);
            else if (mode == 1) hipLaunchKernelGGL(k_ft_round<1>, dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, fa);
            else hipLaunchKernelGGL(k_ft_round<2>, dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, fa);
            zk_prof_end(ctx);
            FtFinArgs ff;
            ff.part = ctx->partials;
            ff.nblk = (int)grid;
            ff.st = ctx->dev;
            ff.chal_idx = ctx->n_chal++;
            ff.proof_off = stack_off + 96 * (uint32_t)t;
            ff.first = t == 0;
            ff.claim_off = outer_claim_off;
            ff.w_idx = w_idx;
            zk_prof_begin(ctx, ZKDL_PROF_FINALISE, 96.0);
            hipLaunchKernelGGL(k_ft_finalise, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ff);
            zk_prof_end(ctx);
            continue;
        }
        RoundArgs ra;
        for (int k = 0; k < 2; ++k) {
            ra.src8[k] = src[k];
            ra.work[k] = work[k];
        }
        ra.src8[2] = src[0];
        ra.work[2] = work[0];
        ra.m = m;
        ra.chal = prev;
        ra.part = ctx->partials;
        zk_prof_begin(ctx, mode ? ZKDL_PROF_SC_ROUND_FUSED : ZKDL_PROF_SC_ROUND_FIRST,
                      2.0 * (mode ? 192.0 : 64.0) * (double)m);
        launch_round<2>(ctx, mode, ra, grid);
        zk_prof_end(ctx);
        // first single-product round: its claim_0 is f_{n-1}(v_{n-1}), which the transcript already
        // fixes (written, not absorbed); without stack rounds it is Y~(u0, u1) itself (absorbed, and
        // copied into the outer block)
        FinArgs fin = zk_fin_args(ctx, (int)grid, 3, ctx->n_chal++, inner_rounds_off + 96 * (uint32_t)(t - ln),
                                  t == ln ? (ln == 0 ? 1 : 2) : 0, inner_claim_off, mode != 0);
        fin.claim_copy_off = (t == ln && ln == 0) ? outer_claim_off : 0;
        zk_prof_begin(ctx, ZKDL_PROF_FINALISE, 96.0);
        hipLaunchKernelGGL(k_sc_finalise, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, fin);
        zk_prof_end(ctx);
    }
    if (t_tail < d) {
        ScTailArgs ta;
        for (int k = 0; k < 2; ++k) {
            ta.ra.src8[k] = src[k];
            ta.ra.work[k] = work[k];
        }
        ta.ra.src8[2] = src[0];
        ta.ra.work[2] = work[0];
        ta.ra.m = (uint64_t)1 << (d - t_tail - 1);
        ta.ra.chal = nullptr;
        ta.ra.part = nullptr;
        ta.rounds = d - t_tail;
        ta.first_chal = first_chal + t_tail - 1;
        ta.st = ctx->dev;
        ta.rounds_off = inner_rounds_off + 96 * (uint32_t)(t_tail - ln);
        ta.finals_off = finals_off;
        ta.scal_base = finals_scal_base;
        ctx->n_chal += d - t_tail;
        launch_tail<2>(ctx, ta);
        return ZKDL_OK;
    }
    FinishArgs fi;
    for (int k = 0; k < 2; ++k) {
        fi.src[k] = src[k];
        fi.work[k] = work[k];
    }
    fi.src[2] = src[0];
    fi.work[2] = work[0];
    fi.from_work = d >= 2;
    fi.K = 2;
    fi.fold = d >= 1;
    fi.chal = d >= 1 ? &ctx->dev->chal[first_chal + d - 1] : nullptr;
    fi.st = ctx->dev;
    fi.scal_base = finals_scal_base;
    fi.finals_off = finals_off;
    fi.absorb_claim = (d == 0);
    fi.claim_off = inner_claim_off;
    fi.claim_copy_off = d == 0 ? outer_claim_off : 0;
    fi.write_owed_claim_off = (l2 == 0 && ln >= 1) ? inner_claim_off : 0;
    hipLaunchKernelGGL(k_sc_finish, dim3(1), dim3(64), 0, ctx->stream, fi);
    return ZKDL_OK;
}



// ---- transcript-only kernels -----------------------------------------------------
struct FramesArg {
    uint32_t words[ZK_PEND_CAP / 4];   // the frames' bytes, four per word, first byte in the top bits
    uint32_t len;                      // bytes
};

// absorbs host-known frames (protocol headers), then draws `count` challenges
__global__ __launch_bounds__(ZK_BLOCK) void k_frames_draw(DevState* st, FramesArg f, int base, int count) {
    __shared__ TsShared S;
    block_ts_load(S, st);
    if (f.len > 0) {
        auto frame = [&](uint32_t q) -> uint32_t { return (f.words[q >> 2] >> (24 - 8 * (q & 3))) & 0xffu; };
        block_append(S, f.len, frame, false);
    }
    block_challenges(S, st, base, count);
    block_ts_store(S, st);
}

void zk_absorb_words(zkdl_ctx* ctx, const char* label, const uint32_t* words, int n) {
    uint32_t ll = 0;
    while (label[ll] && ll < ts::MAX_LABEL) ++ll;
    const uint32_t len = 1 + ll + 8 + 4 * (uint32_t)n;
    if (ctx->pend_len + len > (uint32_t)ZK_PEND_CAP) zk_flush_frames(ctx);
    uint8_t* p = ctx->pend + ctx->pend_len;
    *p++ = (uint8_t)ll;
    for (uint32_t i = 0; i < ll; ++i) *p++ = (uint8_t)label[i];
    const uint64_t dl = 4 * (uint64_t)n;
    for (int i = 0; i < 8; ++i) *p++ = (uint8_t)(dl >> (8 * i));
    for (int i = 0; i < n; ++i)
        for (int b = 0; b < 4; ++b) *p++ = (uint8_t)(words[i] >> (8 * b));
    ctx->pend_len += len;
}

void zk_launch_draw(zkdl_ctx* ctx, int chal_base, int count) {
    if (count <= 0 && ctx->pend_len == 0) return;
    static_assert((ZK_PEND_CAP + 63) / 64 <= TS_MAX_BLOCKS, "one schedule row per block an append completes");
    FramesArg f;
    f.len = ctx->pend_len;
    for (uint32_t i = 0; i < (uint32_t)ZK_PEND_CAP / 4; ++i) f.words[i] = 0;
    for (uint32_t i = 0; i < ctx->pend_len; ++i) f.words[i >> 2] |= (uint32_t)ctx->pend[i] << (24 - 8 * (i & 3));
    ctx->pend_len = 0;
    hipLaunchKernelGGL(k_frames_draw, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev, f, chal_base,
                       count > 0 ? count : 0);
}

// ---------------------------------------------------------------------------
// Hadamard product (Eq. exm-hadamard-batched) without a table for beta~(p, .) in the large rounds.
// With the variables before t bound at v,
//   g_t(x) = c_t l_t(x) f_t(x),   c_t = prod_{s<t} l_s(v_s),   l_t(x) = (1 - p_t)(1 - x) + p_t x,
//   f_t(x) = sum_b beta~(p_[t+1:], b) X0'(x, b) X1'(x, b)      (degree 2),
// so the rounds of k_ft_round (weight beta~(p_[t+1:], .) per pair index, inner size 1) give f_t at
// 0, 1, 2, the finaliser extends it to 3 and multiplies the scalar factors back: the prover's
// messages g_t(0..3) and the whole proof are those of the product sumcheck on (beta~(p, .), X0, X1),
// while two tables are folded instead of three.  The last rounds run in the single-block kernel on
// three tables; its table of the equality factor, c beta~(p_[t:], .), is written out for it.
// ---------------------------------------------------------------------------
struct HdFinArgs {
    const Fr* part;        // block b: f(0), f(1), f(2) at part[3 b + x]
    int nblk;
    DevState* st;
    int chal_idx;          // where the round's challenge goes
    int p_idx;             // challenge index of p_t
    int c_slot;            // scal[c_slot] = c_{t-1} on entry (t > 0), c_t on exit
    uint32_t proof_off;    // where g_t(0..3) go
    int first;             // round 0: c_0 = 1; claim_0 = g(0) + g(1) is written and absorbed first
    uint32_t claim_off;
};

__global__ __launch_bounds__(ZK_BLOCK) void k_hd_finalise(HdFinArgs a) {
    __shared__ TsShared S;
    __shared__ Fr g[ZK_MAX_EVALS + 1];
    __shared__ Fr fs[4];
    __shared__ Fr cl[4];
    DevState* st = a.st;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    block_ts_load(S, st);
    // wave 3 has no partial sums to add: meanwhile it brings the scalar factor up to date,
    // c_t = c_{t-1} l_{t-1}(v_{t-1}), l(v) = (1 - p) + v (2 p - 1), and forms c_t l_t(x), x = 0..3:
    // l(0) = 1 - p, l(1) = p, l(2) = 3 p - 1, l(3) = 5 p - 2
    if (wave == 3 && lane < 4) {
        const Fr one = fr_const(frc::ONE);
        Fr c = one;
        if (!a.first) {
            const Fr pp = st->chal[a.p_idx - 1], vp = st->chal[a.chal_idx - 1];
            const Fr lv = fr_add(fr_sub(one, pp), fr_mul_ni(vp, fr_sub(fr_add(pp, pp), one)));
            c = fr_mul_ni(st->scal[a.c_slot], lv);
        }
        const Fr p = st->chal[a.p_idx];
        const Fr p2 = fr_add(p, p);
        Fr l;
        if (lane == 0) l = fr_sub(one, p);
        else if (lane == 1) l = p;
        else if (lane == 2) l = fr_sub(fr_add(p2, p), one);
        else l = fr_sub(fr_add(fr_add(p2, p2), p), fr_add(one, one));
        cl[lane] = fr_mul_ni(c, l);
        if (lane == 0) st->scal[a.c_slot] = c;
    }
    block_reduce_partials(a.part, a.nblk, 3, fs);
    if (threadIdx.x < 4) {
        // f(3) = f(0) - 3 f(1) + 3 f(2)
        const int x = threadIdx.x;
        Fr f = fs[x < 3 ? x : 0];
        if (x == 3) {
            const Fr d21 = fr_sub(fs[2], fs[1]);
            f = fr_add(fs[0], fr_add(d21, fr_add(d21, d21)));
        }
        g[x] = fr_mul_ni(cl[x], f);
    }
    __syncthreads();
    if (a.first) {
        if (threadIdx.x == 0) {
            g[ZK_MAX_EVALS] = fr_add(g[0], g[1]);
            st->lag_npts = 0;
        }
        __syncthreads();
        block_absorb_frs(S, 'c', &g[ZK_MAX_EVALS], 1, (uint32_t*)(st->proof + a.claim_off));
    }
    block_round_challenge(S, st, g, 4, a.proof_off, a.chal_idx);
    if (wave == 1) {
        if (lane < 4) st->lag[lane] = S.tmp[lane];
        if (lane == 0) {
            st->lag_npts = 4;
            st->lag_chal = (uint32_t)a.chal_idx;
        }
    }
    block_ts_store(S, st);
}

// One more leading variable for a table of beta~: dst[b] = (1 - p) src[b], dst[b + n] = p src[b], b < n
__global__ __launch_bounds__(ZK_BLOCK) void k_hd_suffix_expand(FrTab src, FrTab dst, uint64_t n, const Fr* p) {
    const Fr pv = *p;
    for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; b < n; b += (uint64_t)gridDim.x * blockDim.x) {
        const Fr s0 = tab_ld(src, b);
        const Fr hi = fr_mul(pv, s0);
        tab_st(dst, b + n, hi);
        tab_st(dst, b, fr_sub(s0, hi));
    }
}

// wsuf[t] = beta~(p_[t+1:], .) for t = t_last - 1 .. t_first from wsuf[t_last] (each has one variable more)
void zk_hadamard_suffix_tables(zkdl_ctx* ctx, const FrTab* wsuf, int t_last, int t_first, int d, int p_idx) {
    for (int t = t_last - 1; t >= t_first; --t) {
        const uint64_t n = (uint64_t)1 << (d - t - 2);   // entries of wsuf[t + 1]
        const uint64_t want = (n + ZK_BLOCK - 1) / ZK_BLOCK;
        hipLaunchKernelGGL(k_hd_suffix_expand, dim3((unsigned)(want < 8192 ? want : 8192)), dim3(ZK_BLOCK), 0, ctx->stream,
                           wsuf[t + 1], wsuf[t], n, &ctx->dev->chal[p_idx + t + 1]);
    }
}

// out[b] = scal[c_slot] * beta~((p_idx .. p_idx + nvars), b), b < 2^nvars, as a work table
__global__ void k_hd_eq_tail(const DevState* st, int c_slot, int p_idx, int nvars, F9Tab out) {
    const uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= (1u << nvars)) return;
    const Fr one = fr_const(frc::ONE);
    Fr acc = st->scal[c_slot];
    for (int k = 0; k < nvars; ++k) {
        const Fr pk = st->chal[p_idx + k];
        acc = fr_mul_ni(acc, ((b >> (nvars - 1 - k)) & 1u) ? pk : fr_sub(one, pk));
    }
    f9tab_st(out, b, fr_unpack(acc));
}

// The first two rounds on int32 sources (no conversion pass).  Round 0: the lines of X0 and X1
// through x = 0, 1, 2 are integers below 2^34 in magnitude, their products below 2^68, and a weight
// in Montgomery form times such an integer is the Montgomery form of the product: 27 limb products
// into 12 columns, no reduction until the thread's sum is complete.  Round 1 binds v_0 on the way,
// a + v_0 (a' - a) = redc(R^2 |a| +- v_0 R^2 |a' - a|), and writes the folded work tables.
struct HdIntArgs {
    const int32_t* x[2];
    F9Tab work[2];
    uint64_t m;        // pair indices this round
    FrTab wsuf;        // MODE 1: beta~(p_[2:], .), m entries
    FrTab wH, wL;      // MODE 0: beta~(p_[1:], b) = wH[b >> lb] wL[b & (2^lb - 1)]
    int lb;
    const Fr* chal;    // MODE 1: v_0
    Fr* part;          // block b: f(0), f(1), f(2) at part[3 b + x]
};

// cols += w * (a * c) for a normal w below 2.6 r and |a|, |c| < 2^34; a negative product turns w into 4r - w
__device__ __forceinline__ void cols12_mac_prod(uint64_t* cols, const F9& w, int64_t a, int64_t c) {
    const bool neg = (a < 0) != (c < 0);
    const uint64_t ua = a < 0 ? (uint64_t)0 - (uint64_t)a : (uint64_t)a;
    const uint64_t uc = c < 0 ? (uint64_t)0 - (uint64_t)c : (uint64_t)c;
    const uint64_t lo = ua * uc, hi = __umul64hi(ua, uc);   // the product is below 2^68
    const uint32_t m0 = (uint32_t)lo & frc::M29, m1 = (uint32_t)(lo >> 29) & frc::M29;
    const uint32_t m2 = (uint32_t)(lo >> 58) | ((uint32_t)hi << 6);
#pragma unroll
    for (int i = 0; i < 9; ++i) {
        const uint32_t wi = neg ? frc::C4R[i] - w.v[i] : w.v[i];
        cols[i] += (uint64_t)wi * m0;
        cols[i + 1] += (uint64_t)wi * m1;
        cols[i + 2] += (uint64_t)wi * m2;
    }
#pragma unroll
    for (int k = 0; k + 1 < 12; ++k) {   // columns 0..10 below 2^29 again
        cols[k + 1] += cols[k] >> 29;
        cols[k] &= frc::M29;
    }
}

// carried 12-column sum -> lazy value congruent to it, normal and below 2.41 r (as cols11_value)
__device__ __forceinline__ F9 cols12_value(const uint64_t* cols) {
    F9 vlo, vhi = f9_zero();
#pragma unroll
    for (int i = 0; i < 9; ++i) vlo.v[i] = (uint32_t)cols[i];
    vhi.v[0] = (uint32_t)cols[9];
    vhi.v[1] = (uint32_t)cols[10];
    vhi.v[2] = (uint32_t)cols[11] & frc::M29;
    vhi.v[3] = (uint32_t)(cols[11] >> 29) & frc::M29;
    vhi.v[4] = (uint32_t)(cols[11] >> 58);
    return f9_norm_reduce(f9_add(vlo, f9_mul(vhi, fr_unpack(fr_const(frc::R2)))));
}

template <int MODE>
__global__ __launch_bounds__(ZK_BLOCK) void k_hd_round_i32(HdIntArgs a) {
    __shared__ uint32_t red[BLOCK_SUM_LAZY_WORDS];
    __shared__ F9 kf[4];     // R^2, -R^2, v0 R^2, -v0 R^2
    const uint64_t m = a.m;
    F9 acc[3];
    if (MODE == 0) {
        uint64_t cols[3][12];
#pragma unroll
        for (int x = 0; x < 3; ++x)
#pragma unroll
            for (int c = 0; c < 12; ++c) cols[x][c] = 0;
        // sum_b wH[bh] wL[bl] q(b) = sum_bh wH[bh] (sum_bl wL[bl] q(b)): a block takes a contiguous range
        // of pair indices, a thread keeps the inner sums as columns while its bh stays the same
        // (wL is small and stays in the caches; no table of 2^(d-1) weights is read or built)
#pragma unroll
        for (int x = 0; x < 3; ++x) acc[x] = f9_zero();
        const uint64_t per = ((m + gridDim.x - 1) / gridDim.x + ZK_BLOCK - 1) / ZK_BLOCK * ZK_BLOCK;
        const uint64_t b0 = blockIdx.x * per, b1 = b0 + per < m ? b0 + per : m;
        const uint64_t mask = ((uint64_t)1 << a.lb) - 1, none = ~(uint64_t)0;
        uint64_t cur = none;
        auto flush = [&](uint64_t bh) {
            const F9 hv = fr_unpack(tab_ld(a.wH, bh));
#pragma unroll
            for (int x = 0; x < 3; ++x) {
                acc[x] = f9_norm_reduce(f9_add(acc[x], f9_mul(hv, cols12_value(cols[x]))));
#pragma unroll
                for (int c = 0; c < 12; ++c) cols[x][c] = 0;
            }
        };
        for (uint64_t b = b0 + threadIdx.x; b < b1; b += ZK_BLOCK) {
            const uint64_t bh = b >> a.lb;
            if (bh != cur) {
                if (cur != none) flush(cur);
                cur = bh;
            }
            const int64_t a0 = a.x[0][b], a1 = a.x[0][b + m], c0 = a.x[1][b], c1 = a.x[1][b + m];
            const F9 w = fr_unpack(tab_ld(a.wL, b & mask));
            cols12_mac_prod(cols[0], w, a0, c0);
            cols12_mac_prod(cols[1], w, a1, c1);
            cols12_mac_prod(cols[2], w, 2 * a1 - a0, 2 * c1 - c0);
        }
        if (cur != none) flush(cur);
    } else {
        if (threadIdx.x < 4) {
            const Fr v0 = *a.chal, r2 = fr_const(frc::R2);
            const Fr c = threadIdx.x < 2 ? r2 : fr_mul(v0, r2);
            kf[threadIdx.x] = fr_unpack((threadIdx.x & 1) ? fr_neg(c) : c);
        }
        __syncthreads();
#pragma unroll
        for (int x = 0; x < 3; ++x) acc[x] = f9_zero();
        for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; b < m; b += (uint64_t)gridDim.x * blockDim.x) {
            F9 lo[2], hi[2];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int64_t t0 = a.x[k][b], t1 = a.x[k][b + m], t2 = a.x[k][b + 2 * m], t3 = a.x[k][b + 3 * m];
                lo[k] = fold_ints(kf, t0, t2);
                hi[k] = fold_ints(kf, t1, t3);
                f9tab_st(a.work[k], b, lo[k]);
                f9tab_st(a.work[k], b + m, hi[k]);
            }
            const F9 w = fr_unpack(tab_ld(a.wsuf, b));
            const F9 wl = f9_mul(lo[0], w), wh = f9_mul(hi[0], w);
            const F9 w2 = f9_norm(f9_add(wh, f9_norm(f9_sub(wh, wl))));
            const F9 e2 = f9_add(hi[1], f9_norm(f9_sub(hi[1], lo[1])));
            acc[0] = f9_add(acc[0], f9_mul(wl, lo[1]));
            acc[1] = f9_add(acc[1], f9_mul(wh, hi[1]));
            acc[2] = f9_add(acc[2], f9_mul(w2, e2));
#pragma unroll
            for (int x = 0; x < 3; ++x) acc[x] = f9_norm_reduce(acc[x]);
        }
    }
    const Fr s = block_sum_lazy<3>(acc, red);
    if (threadIdx.x < 3) a.part[(uint64_t)blockIdx.x * 3 + threadIdx.x] = s;
}

// x: X0, X1 (packed, 2^d entries); wsuf[t], t < d - 10: beta~(p_[t+1:], .) with 2^(d-t-1) entries;
// eq_tail: 2^11 work-table entries; p_idx: challenge index of p_0.  d >= ZK_HD_MIN_LOG.
// xi != nullptr: both sources are int32 arrays (device); x and wsuf[0] are not read, the first round
// takes its weights as split[0][b >> split_lb] split[1][b & (2^split_lb - 1)].
int zk_hadamard_eq(zkdl_ctx* ctx, const FrTab* x, const int32_t* const* xi, const FrTab* wsuf, const FrTab* split,
                   int split_lb, void* work_mem, F9Tab eq_tail, int d, int p_idx, int finals_scal_base) {
    constexpr int SC_TAIL_LOG = 10;
    if (d < ZK_HD_MIN_LOG || ctx->n_chal + d > ZK_MAX_CHAL) return ZKDL_EINVAL;
    zk_flush_frames(ctx);
    uint32_t hdr[4] = {SC_MAGIC, 3, 3, (uint32_t)d};
    zk_write_proof_words(ctx, hdr, 4);
    const uint32_t claim_off = (uint32_t)ctx->proof_len;
    const uint32_t rounds_off = claim_off + 32;
    const uint32_t finals_off = rounds_off + (uint32_t)d * 128;
    if (finals_off + 96 > (uint32_t)ZK_PROOF_CAP) return ZKDL_ESMALL;
    ctx->proof_len = finals_off + 96;
    const uint64_t half = (uint64_t)1 << (d - 1);
    F9Tab work[2];
    for (int k = 0; k < 2; ++k) {
        work[k].p = (uint32_t*)work_mem + (size_t)k * half * 9;
        work[k].ps = half;
    }
    const int first_chal = ctx->n_chal;
    const int t_tail = d - SC_TAIL_LOG;
    const int c_slot = 32;   // the scalar factor c_t of the last round closed
    for (int t = 0; t < t_tail; ++t) {
        const int mode = t == 0 ? 0 : t == 1 ? 1 : 2;
        const uint64_t m = (uint64_t)1 << (d - t - 1);
        const uint64_t want = (m + ZK_BLOCK - 1) / ZK_BLOCK;
        const unsigned grid = (unsigned)(want > ZK_MAX_PART_BLOCKS ? ZK_MAX_PART_BLOCKS : want);
        FtRoundArgs fa;
        for (int k = 0; k < 2; ++k) {
            fa.src8[k] = xi ? make_tab(nullptr, 0) : x[k];
            fa.work[k] = work[k];
        }
        fa.m = m;
        fa.log_inner = 0;
        fa.wsuf = wsuf[t];
        fa.chal = mode ? &ctx->dev->chal[first_chal + t - 1] : nullptr;
        fa.part = ctx->partials;
        if (xi && mode < 2) {
            HdIntArgs ia;
            for (int k = 0; k < 2; ++k) {
                ia.x[k] = xi[k];
                ia.work[k] = work[k];
            }
            ia.m = m;
            ia.wsuf = wsuf[t];
            ia.wH = split[0];
            ia.wL = split[1];
            ia.lb = split_lb;
            ia.chal = fa.chal;
            ia.part = ctx->partials;
            // algorithmic bytes: the integers (2 or 4 per table), one weight, round 1 also the folded tables
            zk_prof_begin(ctx, mode ? ZKDL_PROF_SC_ROUND_FUSED : ZKDL_PROF_SC_ROUND_FIRST,
                          (mode ? 2.0 * (16.0 + 64.0) + 32.0 : 2.0 * 8.0 + 32.0) * (double)m);
            if (mode == 0) hipLaunchKernelGGL(k_hd_round_i32<0>, dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, ia);
            else hipLaunchKernelGGL(k_hd_round_i32<1>, dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, ia);
            zk_prof_end(ctx);
        } else {
            // algorithmic bytes: two tables as in the product rounds, plus one weight per pair index
            zk_prof_begin(ctx, mode ? ZKDL_PROF_SC_ROUND_FUSED : ZKDL_PROF_SC_ROUND_FIRST,
                          (2.0 * (mode ? 192.0 : 64.0) + 32.0) * (double)m);
            if (mode == 0) hipLaunchKernelGGL(k_ft_round<0>, dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, fa);
            else if (mode == 1) hipLaunchKernelGGL(k_ft_round<1>, dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, fa);
            else hipLaunchKernelGGL(k_ft_round<2>, dim3(grid), dim3(ZK_BLOCK), 0, ctx->stream, fa);
            zk_prof_end(ctx);
        }
        HdFinArgs hf;
        hf.part = ctx->partials;
        hf.nblk = (int)grid;
        hf.st = ctx->dev;
        hf.chal_idx = ctx->n_chal++;
        hf.p_idx = p_idx + t;
        hf.c_slot = c_slot;
        hf.proof_off = rounds_off + (uint32_t)t * 128;
        hf.first = t == 0;
        hf.claim_off = claim_off;
        zk_prof_begin(ctx, ZKDL_PROF_FINALISE, 128.0);
        hipLaunchKernelGGL(k_hd_finalise, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, hf);
        zk_prof_end(ctx);
    }
    // the single-block kernel folds its tables with the last challenge drawn above before its first
    // round: the equality factor's table stands one challenge back, c_{t_tail - 1} beta~(p_[t_tail-1:], .)
    const int nv = SC_TAIL_LOG + 1;
    hipLaunchKernelGGL(k_hd_eq_tail, dim3((1u << nv) / ZK_BLOCK), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev, c_slot,
                       p_idx + t_tail - 1, nv, eq_tail);
    ScTailArgs ta;
    ta.ra.work[0] = eq_tail;
    for (int k = 0; k < 2; ++k) ta.ra.work[1 + k] = work[k];
    for (int k = 0; k < 3; ++k) ta.ra.src8[k] = make_tab(nullptr, 0);   // the tail reads the work tables only
    ta.ra.m = (uint64_t)1 << (d - t_tail - 1);
    ta.ra.chal = nullptr;
    ta.ra.part = nullptr;
    ta.rounds = d - t_tail;
    ta.first_chal = first_chal + t_tail - 1;
    ta.st = ctx->dev;
    ta.rounds_off = rounds_off + (uint32_t)t_tail * 128;
    ta.finals_off = finals_off;
    ta.scal_base = finals_scal_base;
    ctx->n_chal += d - t_tail;
    launch_tail<3>(ctx, ta);
    return ZKDL_OK;
}
