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

// absorbs the K claims under "c" (and writes them to the proof), then draws n_draw challenges
__global__ __launch_bounds__(ZK_BLOCK) void k_ri_absorb(DevState* st, int scal_base, int K, uint32_t proof_off,
                                                        int chal_base, int n_draw) {
    __shared__ TsShared S;
    block_ts_load(S, st);
    block_absorb_frs(S, 'c', &st->scal[scal_base], K, (uint32_t*)(st->proof + proof_off));
    block_challenges(S, st, chal_base, n_draw);
    block_ts_store(S, st);
}

void zk_launch_absorb_claims(zkdl_ctx* ctx, int scal_base, int K, uint32_t proof_off, int chal_base, int n_draw) {
    zk_flush_frames(ctx);
    hipLaunchKernelGGL(k_ri_absorb, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev, scal_base, K, proof_off, chal_base,
                       n_draw);
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

// The index maps of a chained window, written on the device (no copy from the host in the middle of a
// proof): sub-stack "down" has slot j -> j + 1, none (-1) for the last of every L slots; with
// with_ident the stack itself comes first (k = 0) and "down" is k = 1.  maps: the maps one after the
// other; row_off / ent: their inverse by stack index, as ReindexJob takes it.
__global__ void k_ri_layer_maps(uint32_t N, uint32_t L, int with_ident, int32_t* maps, uint32_t* row_off,
                                uint32_t* ent) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > N) return;
    const uint32_t shifted_before = i - (i + L - 1) / L;   // stack indices below i that "down" reaches
    uint32_t off = with_ident ? i + shifted_before : shifted_before;
    row_off[i] = off;
    if (i == N) return;
    const uint32_t kd = with_ident ? 1u : 0u;
    if (with_ident) {
        maps[i] = (int32_t)i;
        ent[off++] = i;
    }
    maps[(with_ident ? N : 0u) + i] = (i % L != L - 1) ? (int32_t)(i + 1) : -1;
    if (i % L != 0) ent[off] = (kd << 29) | (i - 1);
}

void zk_launch_layer_maps(zkdl_ctx* ctx, uint32_t N, uint32_t L, int with_ident, int32_t* maps, uint32_t* row_off,
                          uint32_t* ent) {
    hipLaunchKernelGGL(k_ri_layer_maps, dim3((N + 1 + ZK_BLOCK - 1) / ZK_BLOCK), dim3(ZK_BLOCK), 0, ctx->stream, N, L,
                       with_ident, maps, row_off, ent);
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
                       (uint32_t)ctx->proof_len, chal_base, job.K);
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
    FrTab x[ZKDL_REINDEX_MAX_K];      // the table claim k is taken on
};

// part[k * gridDim.x + block] = the block's share of sum_b beta_k[b] x_k[b]
__global__ __launch_bounds__(ZK_BLOCK) void k_mg_claims_part(MgTabs m, int K, uint64_t n, Fr* part) {
    __shared__ uint32_t red[64];
    for (int k = 0; k < K; ++k) {
        Fr acc = fr_zero();
        for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; b < n; b += (uint64_t)gridDim.x * blockDim.x)
            acc = fr_add(acc, fr_mul(tab_ld(m.beta[k], b), tab_ld(m.x[k], b)));
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
    for (int k = 0; k < ZKDL_REINDEX_MAX_K; ++k) {
        m.beta[k] = k < K ? beta[k] : make_tab(nullptr, 0);
        m.x[k] = k < K ? x : make_tab(nullptr, 0);
    }
    const uint64_t n = (uint64_t)1 << d;
    const int claims_scal = 8;
    uint64_t blocks = (n + ZK_BLOCK - 1) / ZK_BLOCK;
    const unsigned nblk = (unsigned)(blocks < (uint64_t)ZK_MAX_PART_BLOCKS ? blocks : (uint64_t)ZK_MAX_PART_BLOCKS);
    zk_flush_frames(ctx);
    // ctx->partials holds ZK_MAX_PART_BLOCKS * ZK_MAX_EVALS * 2 elements >= K * nblk for K <= 8
    hipLaunchKernelGGL(k_mg_claims_part, dim3(nblk), dim3(ZK_BLOCK), 0, ctx->stream, m, K, n, ctx->partials);
    hipLaunchKernelGGL(k_mg_claims_sum, dim3(K), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev,
                       (const Fr*)ctx->partials, (int)nblk, claims_scal);
    const int chal_base = ctx->n_chal;
    hipLaunchKernelGGL(k_ri_absorb, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev, claims_scal, K,
                       (uint32_t)ctx->proof_len, chal_base, K);
    ctx->proof_len += 32 * (size_t)K;
    ctx->n_chal += K;
    const unsigned wblk = (unsigned)(blocks < 4096 ? blocks : 4096);
    hipLaunchKernelGGL(k_mg_weights, dim3(wblk), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev, m, K, chal_base, n, p);
    FrTab src[2] = {p, x};
    return zk_sumcheck_product(ctx, 2, src, work_mem, d, 0);
}

// ---------------------------------------------------------------------------
// The same statement for a stack X [N, D] on tables of D (not N D) entries.  Claims X~(s_k, q_k):
//  1. T[k, x] = X~(s_k, x) (the stack axis bound), E[k, x] = r_k beta~(q_k, x);
//     sum_k r_k X~(s_k, q_k) = sum_{k, x} E[k, x] T[k, x]: product sumcheck over (k, x), k leading,
//     challenges (rho, v); it leaves T~(rho, v) = sum_k beta~(rho, k) X~(s_k, v);
//  2. Eq. sc-reindex with the common inner point v: T~(rho, v) = sum_i Pn[i] X~(i, v),
//     Pn[i] = sum_k beta~(rho, k) beta~(s_k, i): product sumcheck over i, leaves X~(v_n, v).
// ---------------------------------------------------------------------------
// E[k, x] *= r_k for k < K (r_k = chal[chal_base + k]); rows K .. K2 - 1 of E and T are cleared
__global__ __launch_bounds__(ZK_BLOCK) void k_ms_scale(const DevState* st, int chal_base, int K, int K2, uint64_t D,
                                                       FrTab e, FrTab t) {
    const uint64_t total = (uint64_t)K2 * D;
    for (uint64_t b = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; b < total; b += (uint64_t)gridDim.x * blockDim.x) {
        const int k = (int)(b / D);
        if (k < K) {
            tab_st(e, b, fr_mul(st->chal[chal_base + k], tab_ld(e, b)));
        } else {
            tab_st(e, b, fr_zero());
            tab_st(t, b, fr_zero());
        }
    }
}

// Pn[i] = sum_k brho[k] bs_k[i]
__global__ __launch_bounds__(ZK_BLOCK) void k_ms_stack_weights(MgTabs bs, FrTab brho, int K, uint64_t N, FrTab pn) {
    const uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (i >= N) return;
    Fr acc = fr_mul(tab_ld(brho, 0), tab_ld(bs.beta[0], i));
    for (int k = 1; k < K; ++k) acc = fr_add(acc, fr_mul(tab_ld(brho, k), tab_ld(bs.beta[k], i)));
    tab_st(pn, i, acc);
}

int zk_stack_merge(zkdl_ctx* ctx, const StackMergeJob& job, std::vector<void*>& keep) {
    const int K = job.K;
    const uint64_t N = job.N, rows = job.rows, cols = job.cols, D = rows * cols;
    int ln = 0, lr = 0, lc = 0, lk = 0;
    while (((uint64_t)1 << ln) < N) ++ln;
    while (((uint64_t)1 << lr) < rows) ++lr;
    while (((uint64_t)1 << lc) < cols) ++lc;
    while ((1 << lk) < K) ++lk;
    const int ld = lr + lc, K2 = 1 << lk;
    if (ctx->n_chal + K + lk + ld + ln > ZK_MAX_CHAL) return ZKDL_EINVAL;
    size_t work = zk_sumcheck_work_bytes(2, lk + ld);
    if (zk_sumcheck_work_bytes(2, ln) > work) work = zk_sumcheck_work_bytes(2, ln);
    const uint64_t fr_elems = (uint64_t)K * N + K2 + rows + cols + 2 * (uint64_t)K2 * D + N * rows + 2 * N;
    void* mem = zk_alloc(ctx, fr_elems * 32 + work);
    if (!mem) return ZKDL_ENOMEM;
    keep.push_back(mem);
    uint32_t* w = (uint32_t*)mem;
    auto take = [&](uint64_t n) {
        FrTab t = make_tab(w, n);
        w += 8 * n;
        return t;
    };
    MgTabs bs, cl;
    for (int k = 0; k < ZKDL_REINDEX_MAX_K; ++k) bs.beta[k] = bs.x[k] = cl.beta[k] = cl.x[k] = make_tab(nullptr, 0);
    for (int k = 0; k < K; ++k) bs.beta[k] = take(N);
    const FrTab brho = take(K2), br = take(rows), bc = take(cols);
    const FrTab E = take((uint64_t)K2 * D), T = take((uint64_t)K2 * D);
    const FrTab by_row = take(N * rows), Tn = take(N), Pn = take(N);
    void* work_mem = w;

    // beta~(s_k, .), beta~(q_k, .) into row k of E; T[k, .] = X~(s_k, .)
    BetaJob jobs[2 * ZKDL_REINDEX_MAX_K];
    for (int k = 0; k < K; ++k) {
        jobs[2 * k] = BetaJob{job.point[k], ln, bs.beta[k]};
        jobs[2 * k + 1] = BetaJob{job.point[k] + ln, ld, tab_offset(E, (uint64_t)k * D)};
    }
    int rc = zk_build_beta_many(ctx, jobs, 2 * K);
    for (int k = 0; k < K && rc == ZKDL_OK; ++k)
        rc = zk_partial_eval(ctx, job.kind, job.X, 1, N, D, bs.beta[k], tab_offset(T, (uint64_t)k * D));
    if (rc != ZKDL_OK) return rc;
    // the K claims sum_x beta~(q_k, x) T[k, x]
    for (int k = 0; k < K; ++k) {
        cl.beta[k] = tab_offset(E, (uint64_t)k * D);
        cl.x[k] = tab_offset(T, (uint64_t)k * D);
    }
    const int claims_scal = 8;
    const uint64_t blocks = (D + ZK_BLOCK - 1) / ZK_BLOCK;
    const unsigned nblk = (unsigned)(blocks < (uint64_t)ZK_MAX_PART_BLOCKS ? blocks : (uint64_t)ZK_MAX_PART_BLOCKS);
    zk_flush_frames(ctx);
    hipLaunchKernelGGL(k_mg_claims_part, dim3(nblk), dim3(ZK_BLOCK), 0, ctx->stream, cl, K, D, ctx->partials);
    hipLaunchKernelGGL(k_mg_claims_sum, dim3(K), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev,
                       (const Fr*)ctx->partials, (int)nblk, claims_scal);
    const int chal_base = ctx->n_chal;
    hipLaunchKernelGGL(k_ri_absorb, dim3(1), dim3(ZK_BLOCK), 0, ctx->stream, ctx->dev, claims_scal, K,
                       (uint32_t)ctx->proof_len, chal_base, K);
    ctx->proof_len += 32 * (size_t)K;
    ctx->n_chal += K;
    const uint64_t sblocks = ((uint64_t)K2 * D + ZK_BLOCK - 1) / ZK_BLOCK;
    hipLaunchKernelGGL(k_ms_scale, dim3((unsigned)(sblocks < 4096 ? sblocks : 4096)), dim3(ZK_BLOCK), 0, ctx->stream,
                       ctx->dev, chal_base, K, K2, D, E, T);
    const int c1 = ctx->n_chal;   // rho (lk), then v (rows first, then columns)
    FrTab src[2] = {E, T};
    rc = zk_sumcheck_product(ctx, 2, src, work_mem, lk + ld, 0);
    if (rc != ZKDL_OK) return rc;

    const Fr* chal = ctx->dev->chal;
    const BetaJob j2[3] = {{chal + c1, lk, brho}, {chal + c1 + lk, lr, br}, {chal + c1 + lk + lr, lc, bc}};
    rc = zk_build_beta_many(ctx, j2, 3);
    // X~(i, v): the columns first, then the rows
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, job.kind, job.X, N * rows, cols, 1, bc, by_row);
    if (rc == ZKDL_OK) rc = zk_partial_eval(ctx, TK_FR, &by_row, N, rows, 1, br, Tn);
    if (rc != ZKDL_OK) return rc;
    hipLaunchKernelGGL(k_ms_stack_weights, dim3((unsigned)((N + ZK_BLOCK - 1) / ZK_BLOCK)), dim3(ZK_BLOCK), 0,
                       ctx->stream, bs, brho, K, N, Pn);
    FrTab src2[2] = {Pn, Tn};
    return zk_sumcheck_product(ctx, 2, src2, work_mem, ln, 0);
}
