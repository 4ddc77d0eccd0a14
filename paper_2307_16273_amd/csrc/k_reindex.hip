// Re-indexing of stacked tensors (Sec. 4, Eq. sc-reindex; the re-indexing line of Protocol zkdl).
//
// K sub-stacks of a stack X [N, D] carry one claim each, X_k~(u_k, u), with X_k the tensors
// X^(map_k[0]), X^(map_k[1]), .. (an entry -1 is a zero tensor).  With coefficients r_k from
// the verifier,  sum_k r_k X_k~(u_k, u) = sum_i P[i] X~(i, u),
//   P[i] = sum_k r_k sum_{j : map_k[j] = i} beta~(u_k, j),
// and the right-hand side is a product sumcheck over i on the tables P and T = X~(., u).
// This file holds the three steps around that sumcheck: the sub-stack claims, their absorption
// with the draw of r, and the table P.
#include "dev_common.cuh"

struct RiMaps {
    const int32_t* map[ZKDL_REINDEX_MAX_K];   // device
    uint64_t len[ZKDL_REINDEX_MAX_K];
    FrTab beta[ZKDL_REINDEX_MAX_K];           // beta~(u_k, .), len[k] entries
};

// block k: claim_k = sum_j beta_k[j] * T[map_k[j]]  ->  st->scal[scal_base + k]
__global__ __launch_bounds__(ZK_BLOCK) void k_ri_claims(DevState* st, RiMaps m, FrTab t, int scal_base) {
    __shared__ uint32_t red[64];
    const int k = blockIdx.x;
    const int32_t* map = m.map[k];
    Fr acc = fr_zero();
    for (uint64_t j = threadIdx.x; j < m.len[k]; j += blockDim.x) {
        const int32_t i = map[j];
        if (i >= 0) acc = fr_add(acc, fr_mul(tab_ld(m.beta[k], j), tab_ld(t, (uint64_t)i)));
    }
    acc = block_sum(acc, red);
    if (threadIdx.x == 0) st->scal[scal_base + k] = acc;
}

// absorbs the K claims under "c" (and writes them to the proof), draws r_0 .. r_{K-1}
__global__ __launch_bounds__(ZK_BLOCK) void k_ri_absorb(DevState* st, int scal_base, int K, uint32_t proof_off,
                                                        int chal_base) {
    __shared__ TsShared S;
    block_ts_load(S, st);
    block_absorb_frs(S, 'c', &st->scal[scal_base], K, (uint32_t*)(st->proof + proof_off));
    block_challenges(S, st, chal_base, K);
    block_ts_store(S, st);
}

// P[i] = sum over the entries e of row i of the inverse maps of r_{k(e)} * beta_{k(e)}[j(e)];
// an entry packs k in its top 3 bits and j in the other 29
__global__ __launch_bounds__(ZK_BLOCK) void k_ri_weights(const DevState* st, RiMaps m, const uint32_t* row_off,
                                                         const uint32_t* ent, uint64_t n, int chal_base, FrTab p) {
    const uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (i >= n) return;
    Fr acc = fr_zero();
    for (uint32_t e = row_off[i]; e < row_off[i + 1]; ++e) {
        const uint32_t k = ent[e] >> 29, j = ent[e] & 0x1fffffffu;
        acc = fr_add(acc, fr_mul(st->chal[chal_base + k], tab_ld(m.beta[k], j)));
    }
    tab_st(p, i, acc);
}

int zk_reindex(zkdl_ctx* ctx, const ReindexJob& job, FrTab t, FrTab p, int ln, void* work_mem) {
    RiMaps m;
    for (int k = 0; k < ZKDL_REINDEX_MAX_K; ++k) {
        m.map[k] = k < job.K ? job.map[k] : nullptr;
        m.len[k] = k < job.K ? job.len[k] : 0;
        m.beta[k] = k < job.K ? job.beta[k] : make_tab(nullptr, 0);
    }
    const int claims_scal = 8;
    zk_flush_frames(ctx);
    hipLaunchKernelGGL(k_ri_claims, dim3(job.K), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev, m, t, claims_scal);
    const int chal_base = ctx->n_chal;
    hipLaunchKernelGGL(k_ri_absorb, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev, claims_scal, job.K,
                       (uint32_t)ctx->proof_len, chal_base);
    ctx->proof_len += 32 * (size_t)job.K;
    ctx->n_chal += job.K;
    const uint64_t n = (uint64_t)1 << ln;
    hipLaunchKernelGGL(k_ri_weights, dim3((unsigned)((n + ZK_BLOCK - 1) / ZK_BLOCK)), dim3(ZK_BLOCK), 0, ctx->stream,
                       ctx->dev, m, job.row_off, job.ent, n, chal_base, p);
    FrTab src[2] = {p, t};
    return zk_sumcheck_product(ctx, 2, src, work_mem, ln, 0);
}
