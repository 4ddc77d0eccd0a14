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

// ---------------------------------------------------------------------------
// Several claims on one tensor -> one: sum_k r_k X~(p_k) = sum_b P[b] X(b) with
// P = sum_k r_k beta~(p_k, .), the defining sum of the multilinear extension (Sec. 2.2) taken
// for K points at once; Eq. sc-reindex with every sub-stack the stack itself and the sum over
// all variables.  Protocol zkdl opens one evaluation per stack: this produces it.
// ---------------------------------------------------------------------------
struct MgTabs {
    FrTab beta[ZKDL_REINDEX_MAX_K];   // beta~(p_k, .), n entries each
};

// part[k * gridDim.x + block] = the block's share of sum_b beta_k[b] X[b]
__global__ __launch_bounds__(ZK_BLOCK) void k_mg_claims_part(MgTabs m, int K, FrTab x, uint64_t n, Fr* part) {
    __shared__ uint32_t red[64];
    for (int k = 0; k < K; ++k) {
        Fr acc = fr_zero();
        for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; b < n; b += (uint64_t)gridDim.x * blockDim.x)
            acc = fr_add(acc, fr_mul(tab_ld(m.beta[k], b), tab_ld(x, b)));
        acc = block_sum(acc, red);
        if (threadIdx.x == 0) part[(size_t)k * gridDim.x + blockIdx.x] = acc;
        __syncthreads();
    }
}

// block k: claim_k = sum of its nblk partial sums -> st->scal[scal_base + k]
__global__ __launch_bounds__(ZK_BLOCK) void k_mg_claims_sum(DevState* st, const Fr* part, int nblk, int scal_base) {
    __shared__ uint32_t red[64];
    const int k = blockIdx.x;
    Fr acc = fr_zero();
    for (int i = threadIdx.x; i < nblk; i += blockDim.x) acc = fr_add(acc, part[(size_t)k * nblk + i]);
    acc = block_sum(acc, red);
    if (threadIdx.x == 0) st->scal[scal_base + k] = acc;
}

// P[b] = sum_k r_k beta_k[b], r_k = chal[chal_base + k]
__global__ __launch_bounds__(ZK_BLOCK) void k_mg_weights(const DevState* st, MgTabs m, int K, int chal_base,
                                                         uint64_t n, FrTab p) {
    __shared__ Fr r[ZKDL_REINDEX_MAX_K];
    if (threadIdx.x < K) r[threadIdx.x] = st->chal[chal_base + threadIdx.x];
    __syncthreads();
    for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; b < n; b += (uint64_t)gridDim.x * blockDim.x) {
        Fr acc = fr_mul(r[0], tab_ld(m.beta[0], b));
        for (int k = 1; k < K; ++k) acc = fr_add(acc, fr_mul(r[k], tab_ld(m.beta[k], b)));
        tab_st(p, b, acc);
    }
}

int zk_merge(zkdl_ctx* ctx, int K, const FrTab* beta, FrTab x, FrTab p, int d, void* work_mem) {
    MgTabs m;
    for (int k = 0; k < ZKDL_REINDEX_MAX_K; ++k) m.beta[k] = k < K ? beta[k] : make_tab(nullptr, 0);
    const uint64_t n = (uint64_t)1 << d;
    const int claims_scal = 8;
    uint64_t blocks = (n + ZK_BLOCK - 1) / ZK_BLOCK;
    const unsigned nblk = (unsigned)(blocks < (uint64_t)ZK_MAX_PART_BLOCKS ? blocks : (uint64_t)ZK_MAX_PART_BLOCKS);
    zk_flush_frames(ctx);
    // ctx->partials holds ZK_MAX_PART_BLOCKS * ZK_MAX_EVALS * 2 elements >= K * nblk for K <= 8
    hipLaunchKernelGGL(k_mg_claims_part, dim3(nblk), dim3(ZK_BLOCK), 0, ctx->stream, m, K, x, n, ctx->partials);
    hipLaunchKernelGGL(k_mg_claims_sum, dim3(K), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev,
                       (const Fr*)ctx->partials, (int)nblk, claims_scal);
    const int chal_base = ctx->n_chal;
    hipLaunchKernelGGL(k_ri_absorb, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev, claims_scal, K,
                       (uint32_t)ctx->proof_len, chal_base);
    ctx->proof_len += 32 * (size_t)K;
    ctx->n_chal += K;
    const unsigned wblk = (unsigned)(blocks < 4096 ? blocks : 4096);
    hipLaunchKernelGGL(k_mg_weights, dim3(wblk), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev, m, K, chal_base, n, p);
    FrTab src[2] = {p, x};
    return zk_sumcheck_product(ctx, 2, src, work_mem, d, 0);
}
